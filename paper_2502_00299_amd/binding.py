"""ctypes binding of libchunkkv.so: argument marshalling only.

Every function has the name and argument order of its C-ABI entry point in include/chunkkv.h
(ChunkKV Algorithms 1-3); tensors are passed as device pointers, the current torch stream is used,
and a non-zero status raises ChunkKVError.  There is no fallback: without the built HIP library every
call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libchunkkv.so")

F32, BF16, F16 = 0, 1, 2
FLAG_WHOLE_CHUNKS, FLAG_TWO_PASS = 1, 2     # chunkkv_problem.flags
SYMBOLS = ("chunkkv_status_string", "chunkkv_workspace_bytes", "chunkkv_score", "chunkkv_chunk_topk",
           "chunkkv_compact", "chunkkv_compress_stack", "chunkkv_score_lse", "chunkkv_compress_stack_lse",
           "chunkkv_compress_layer", "chunkkv_workspace_bytes_hybrid", "chunkkv_compress_stack_hybrid", "chunkkv_jaccard", "chunkkv_decode_workspace_bytes", "chunkkv_decode_attention",
           "chunkkv_decode_attention_static", "chunkkv_quality_workspace_bytes", "chunkkv_quality_metrics",
           "chunkkv_timing_begin",
           "chunkkv_timing_end")
TIMING_KINDS = ("score_stats", "stats_merge", "score_colsum", "chunk_sums", "chunk_topk", "compact", "decode")


class ChunkKVError(RuntimeError):
    def __init__(self, status: int, where: str, msg: str):
        super().__init__(f"{where}: status {status} ({msg})")
        self.status = status


class _CProblem(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("window", C.c_int32), ("chunk", C.c_int32), ("dtype", C.c_int32), ("softmax_scale", C.c_float),
        ("seqlen", C.POINTER(C.c_int32)), ("n_keep", C.POINTER(C.c_int32)), ("kv_base", C.POINTER(C.c_int64)),
        ("kv_stride_head", C.c_int64), ("kv_stride_tok", C.c_int64),
        ("out_base", C.POINTER(C.c_int64)), ("out_stride_head", C.c_int64), ("out_stride_tok", C.c_int64),
        ("sel_cap", C.c_int32), ("score_cap", C.c_int32), ("flags", C.c_uint32),
    ]


@dataclass
class Problem:
    """Python mirror of chunkkv_problem (see include/chunkkv.h for the meaning of every field)."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    chunk: int
    dtype: int
    seqlen: Sequence[int]
    n_keep: Sequence[int]
    kv_base: Sequence[int]
    kv_stride_head: int
    kv_stride_tok: int
    out_base: Optional[Sequence[int]] = None
    out_stride_head: int = 0
    out_stride_tok: int = 0
    sel_cap: int = 0
    score_cap: int = 0
    softmax_scale: float = 0.0
    flags: int = 0

    def __post_init__(self):
        c = self.chunk if self.chunk > 0 else 1
        if self.sel_cap == 0:
            self.sel_cap = max((max(int(n), 0) + c - 1) // c + 1 for n in self.n_keep)
        if self.score_cap == 0:
            self.score_cap = max(1, max((int(L) - self.window + c - 1) // c for L in self.seqlen))
        if self.out_base is None:
            kept = [int(n) + self.window for n in self.n_keep]
            if len(set(kept)) == 1:
                # default output [B][Hkv][n_kept][d]
                per_seq = self.n_kv_heads * kept[0] * self.head_dim
                self.out_base = [b * per_seq for b in range(len(kept))]
                self.out_stride_head = kept[0] * self.head_dim
                self.out_stride_tok = self.head_dim
            else:
                # ragged budgets: packed [sum n_kept][Hkv][d]
                run, base = 0, []
                for n in kept:
                    base.append(run * self.n_kv_heads * self.head_dim)
                    run += n
                self.out_base = base
                self.out_stride_head = self.head_dim
                self.out_stride_tok = self.n_kv_heads * self.head_dim

    def out_elements(self) -> int:
        """Elements of one output buffer (K' or V') under the default output layouts."""
        return sum(int(n) + self.window for n in self.n_keep) * self.n_kv_heads * self.head_dim

    @property
    def batch(self) -> int:
        return len(self.seqlen)

    def as_c(self):
        B = self.batch
        keep = {
            "seqlen": (C.c_int32 * B)(*[int(x) for x in self.seqlen]),
            "n_keep": (C.c_int32 * B)(*[int(x) for x in self.n_keep]),
            "kv_base": (C.c_int64 * B)(*[int(x) for x in self.kv_base]),
            "out_base": (C.c_int64 * B)(*[int(x) for x in self.out_base]),
        }
        cp = _CProblem(B, self.n_q_heads, self.n_kv_heads, self.head_dim, self.window, self.chunk, self.dtype,
                       self.softmax_scale, keep["seqlen"], keep["n_keep"], keep["kv_base"],
                       self.kv_stride_head, self.kv_stride_tok, keep["out_base"], self.out_stride_head,
                       self.out_stride_tok, self.sel_cap, self.score_cap, int(self.flags))
        cp._keep = keep
        return cp


_lib = None


def load_library(path: Optional[str] = None):
    """Loads libchunkkv.so (built in-tree by `python -m paper_2502_00299_amd.build`)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(f"{p} is missing: build it with `python -m paper_2502_00299_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(p)
    vp, i32p, f32p = C.c_void_p, C.c_void_p, C.c_void_p
    lib.chunkkv_status_string.restype = C.c_char_p
    lib.chunkkv_status_string.argtypes = [C.c_int]
    lib.chunkkv_workspace_bytes.restype = C.c_size_t
    lib.chunkkv_workspace_bytes.argtypes = [C.POINTER(_CProblem), C.c_int32, C.c_int32]
    lib.chunkkv_score.restype = C.c_int
    lib.chunkkv_score.argtypes = [C.POINTER(_CProblem), vp, vp, f32p, f32p, vp, C.c_size_t, vp]
    lib.chunkkv_chunk_topk.restype = C.c_int
    lib.chunkkv_chunk_topk.argtypes = [C.POINTER(_CProblem), f32p, i32p, i32p, i32p, vp, C.c_size_t, vp]
    lib.chunkkv_compact.restype = C.c_int
    lib.chunkkv_compact.argtypes = [C.POINTER(_CProblem), vp, vp, i32p, i32p, i32p, vp, vp, vp]
    lib.chunkkv_compress_stack.restype = C.c_int
    lib.chunkkv_compress_stack.argtypes = [C.POINTER(_CProblem), C.c_int32, C.c_int32, C.POINTER(vp), C.POINTER(vp),
                                           C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), i32p, i32p, i32p, vp,
                                           C.c_size_t, vp]
    lib.chunkkv_score_lse.restype = C.c_int
    lib.chunkkv_score_lse.argtypes = [C.POINTER(_CProblem), vp, vp, f32p, f32p, f32p, vp, C.c_size_t, vp]
    lib.chunkkv_compress_stack_lse.restype = C.c_int
    lib.chunkkv_compress_stack_lse.argtypes = [C.POINTER(_CProblem), C.c_int32, C.c_int32, C.POINTER(vp),
                                               C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                               C.POINTER(vp), i32p, i32p, i32p, vp, C.c_size_t, vp]
    lib.chunkkv_compress_layer.restype = C.c_int
    lib.chunkkv_compress_layer.argtypes = [C.POINTER(_CProblem), C.c_int32, C.c_int32, vp, f32p, vp, vp, vp, vp,
                                           i32p, i32p, i32p, vp, C.c_size_t, vp]
    lib.chunkkv_workspace_bytes_hybrid.restype = C.c_size_t
    lib.chunkkv_workspace_bytes_hybrid.argtypes = [C.POINTER(_CProblem), C.c_int32, C.c_int32, i32p]
    lib.chunkkv_compress_stack_hybrid.restype = C.c_int
    lib.chunkkv_compress_stack_hybrid.argtypes = [C.POINTER(_CProblem), C.c_int32, C.c_int32, i32p, C.POINTER(vp),
                                                  C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                                  C.POINTER(vp), i32p, i32p, i32p, vp, C.c_size_t, vp]
    lib.chunkkv_jaccard.restype = C.c_int
    lib.chunkkv_jaccard.argtypes = [C.POINTER(_CProblem), C.c_int32, i32p, i32p, i32p, f32p, vp]
    lib.chunkkv_decode_workspace_bytes.restype = C.c_size_t
    lib.chunkkv_decode_workspace_bytes.argtypes = [C.POINTER(_CProblem), C.c_int32]
    lib.chunkkv_decode_attention.restype = C.c_int
    lib.chunkkv_decode_attention.argtypes = [C.POINTER(_CProblem), C.c_int32, i32p, vp, vp, vp, f32p, f32p, vp,
                                             C.c_size_t, vp]
    lib.chunkkv_quality_workspace_bytes.restype = C.c_size_t
    lib.chunkkv_quality_workspace_bytes.argtypes = [C.POINTER(_CProblem)]
    lib.chunkkv_quality_metrics.restype = C.c_int
    lib.chunkkv_quality_metrics.argtypes = [C.POINTER(_CProblem), i32p, vp, vp, vp, vp, vp, f32p, f32p, vp, C.c_size_t, vp]
    lib.chunkkv_decode_attention_static.restype = C.c_int
    lib.chunkkv_decode_attention_static.argtypes = [C.POINTER(_CProblem), C.c_int32, i32p, vp, vp, vp, f32p, f32p, vp]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise ChunkKVError(rc, where, load_library().chunkkv_status_string(rc).decode())


def chunkkv_status_string(status: int) -> str:
    return load_library().chunkkv_status_string(int(status)).decode()


def chunkkv_workspace_bytes(prob: Problem, n_layers: int = 1, reuse: int = 1) -> int:
    return int(load_library().chunkkv_workspace_bytes(C.byref(prob.as_c()), n_layers, reuse))


def chunkkv_score(prob: Problem, q_obs, k, chunk_scores, token_importance, workspace, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_score(C.byref(cp), _ptr(q_obs), _ptr(k), _ptr(chunk_scores),
                                        _ptr(token_importance), _ptr(workspace),
                                        0 if workspace is None else workspace.numel() * workspace.element_size(),
                                        _stream(stream)), "chunkkv_score")


def chunkkv_chunk_topk(prob: Problem, chunk_scores, sel_chunk, sel_len, sel_count, workspace=None, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_chunk_topk(C.byref(cp), _ptr(chunk_scores), _ptr(sel_chunk), _ptr(sel_len),
                                             _ptr(sel_count), _ptr(workspace),
                                             0 if workspace is None else workspace.numel() * workspace.element_size(),
                                             _stream(stream)), "chunkkv_chunk_topk")


def chunkkv_compact(prob: Problem, k, v, sel_chunk, sel_len, sel_count, k_out, v_out, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_compact(C.byref(cp), _ptr(k), _ptr(v), _ptr(sel_chunk), _ptr(sel_len),
                                          _ptr(sel_count), _ptr(k_out), _ptr(v_out), _stream(stream)),
           "chunkkv_compact")


def chunkkv_compress_stack(prob: Problem, reuse: int, q_obs: Sequence, k: Sequence, v: Sequence, k_out: Sequence,
                           v_out: Sequence, sel_chunk, sel_len, sel_count, workspace, stream=None) -> None:
    n = len(k)
    cp = prob.as_c()

    def table(ts):
        return (C.c_void_p * n)(*[None if t is None else t.data_ptr() for t in ts])

    _check(load_library().chunkkv_compress_stack(
        C.byref(cp), n, reuse, table(q_obs), table(k), table(v), table(k_out), table(v_out), _ptr(sel_chunk),
        _ptr(sel_len), _ptr(sel_count), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)),
        "chunkkv_compress_stack")


def chunkkv_score_lse(prob: Problem, q_obs, k, lse, chunk_scores, token_importance, workspace, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_score_lse(C.byref(cp), _ptr(q_obs), _ptr(k), _ptr(lse), _ptr(chunk_scores),
                                            _ptr(token_importance), _ptr(workspace),
                                            0 if workspace is None else workspace.numel() * workspace.element_size(),
                                            _stream(stream)), "chunkkv_score_lse")


def chunkkv_compress_stack_lse(prob: Problem, reuse: int, q_obs: Sequence, k: Sequence, v: Sequence, lse: Sequence,
                               k_out: Sequence, v_out: Sequence, sel_chunk, sel_len, sel_count, workspace,
                               stream=None) -> None:
    n = len(k)
    cp = prob.as_c()

    def table(ts):
        return (C.c_void_p * n)(*[None if t is None else t.data_ptr() for t in ts])

    _check(load_library().chunkkv_compress_stack_lse(
        C.byref(cp), n, reuse, table(q_obs), table(k), table(v), table(lse), table(k_out), table(v_out),
        _ptr(sel_chunk), _ptr(sel_len), _ptr(sel_count), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)),
        "chunkkv_compress_stack_lse")


def chunkkv_compress_layer(prob: Problem, layer: int, reuse: int, q_obs, lse, k, v, k_out, v_out, sel_chunk, sel_len,
                           sel_count, workspace, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_compress_layer(
        C.byref(cp), layer, reuse, _ptr(q_obs), _ptr(lse), _ptr(k), _ptr(v), _ptr(k_out), _ptr(v_out),
        _ptr(sel_chunk), _ptr(sel_len), _ptr(sel_count), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)),
        "chunkkv_compress_layer")


def _chunk_table(chunk_per_group):
    return None if chunk_per_group is None else (C.c_int32 * len(chunk_per_group))(*[int(c) for c in chunk_per_group])


def chunkkv_workspace_bytes_hybrid(prob: Problem, n_layers: int, reuse: int, chunk_per_group) -> int:
    return int(load_library().chunkkv_workspace_bytes_hybrid(C.byref(prob.as_c()), n_layers, reuse,
                                                             _chunk_table(chunk_per_group)))


def chunkkv_compress_stack_hybrid(prob: Problem, reuse: int, chunk_per_group, q_obs: Sequence, k: Sequence,
                                  v: Sequence, lse, k_out: Sequence, v_out: Sequence, sel_chunk, sel_len, sel_count,
                                  workspace, stream=None) -> None:
    n = len(k)
    cp = prob.as_c()

    def table(ts):
        return None if ts is None else (C.c_void_p * n)(*[None if t is None else t.data_ptr() for t in ts])

    _check(load_library().chunkkv_compress_stack_hybrid(
        C.byref(cp), n, reuse, _chunk_table(chunk_per_group), table(q_obs), table(k), table(v), table(lse),
        table(k_out), table(v_out), _ptr(sel_chunk), _ptr(sel_len), _ptr(sel_count), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)),
        "chunkkv_compress_stack_hybrid")


def chunkkv_jaccard(prob: Problem, n_groups: int, sel_chunk, sel_len, sel_count, jaccard, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_jaccard(C.byref(cp), n_groups, _ptr(sel_chunk), _ptr(sel_len), _ptr(sel_count),
                                          _ptr(jaccard), _stream(stream)), "chunkkv_jaccard")


def chunkkv_quality_workspace_bytes(prob: Problem) -> int:
    return int(load_library().chunkkv_quality_workspace_bytes(C.byref(prob.as_c())))


def chunkkv_quality_metrics(prob: Problem, kv_len, q, k, v, k_out, v_out, l1_loss, attn_cos, workspace, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_quality_metrics(
        C.byref(cp), _ptr(kv_len), _ptr(q), _ptr(k), _ptr(v), _ptr(k_out), _ptr(v_out), _ptr(l1_loss), _ptr(attn_cos),
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)),
        "chunkkv_quality_metrics")


def chunkkv_decode_workspace_bytes(prob: Problem, compacted: bool = True) -> int:
    return int(load_library().chunkkv_decode_workspace_bytes(C.byref(prob.as_c()), 1 if compacted else 0))


def chunkkv_decode_attention(prob: Problem, compacted: bool, kv_len, q, k, v, out, lse, workspace, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_decode_attention(
        C.byref(cp), 1 if compacted else 0, _ptr(kv_len), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)),
        "chunkkv_decode_attention")


def chunkkv_decode_attention_static(prob: Problem, compacted: bool, kv_len, q, k, v, out, lse, stream=None) -> None:
    cp = prob.as_c()
    _check(load_library().chunkkv_decode_attention_static(
        C.byref(cp), 1 if compacted else 0, _ptr(kv_len), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
        _stream(stream)), "chunkkv_decode_attention_static")


def chunkkv_timing_begin(max_records: int = 4096) -> None:
    lib = load_library()
    lib.chunkkv_timing_begin.restype = C.c_int
    lib.chunkkv_timing_begin.argtypes = [C.c_int32]
    _check(lib.chunkkv_timing_begin(max_records), "chunkkv_timing_begin")


def chunkkv_timing_end() -> dict:
    """-> {kind: (total milliseconds, launches)} for the kernels launched since chunkkv_timing_begin."""
    lib = load_library()
    n = len(TIMING_KINDS)
    ms, cnt = (C.c_double * n)(), (C.c_int64 * n)()
    lib.chunkkv_timing_end.restype = C.c_int
    lib.chunkkv_timing_end.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    _check(lib.chunkkv_timing_end(ms, cnt), "chunkkv_timing_end")
    return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(TIMING_KINDS)}
