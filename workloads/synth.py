"""Seeded synthetic inputs with the shapes of the paper's workloads.

The paper times LLaMA-3-8B-Instruct prompts of 4k-16k tokens (Section 4.3,
efficiency table) and evaluates on long-context prompts; neither the prompts
nor a model that turns them into K/V exist here, so these tensors stand in for
them: standard-normal Q/K/V with a few planted "salient spans" (runs of
consecutive tokens whose keys share a direction with the window queries), the
structure chunk-level selection is meant to find.

Recipe, per layer ``l`` of workload ``cfg`` (seed = 299 + 1000*cfg + l):
  * one unit vector ``u`` (numpy, CPU, so it does not depend on the device);
  * spans: ``(start, length)`` pairs, length uniform in ``span_len``, start
    uniform in ``[0, P - length]``; layer ``l+1`` keeps each span of layer
    ``l`` with probability ``span_overlap`` and redraws the others;
  * ``Q_obs, K, V ~ N(0, 1)`` in fp32 from a ``torch.Generator`` on the target
    device; ``K[:, span, :] += strength * u`` for every kv-head and
    ``Q_obs += strength * u`` for every window row; one round-to-nearest-even
    cast to the storage type.

Nothing here computes a score, a selection or a gather.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np
import torch

SEED_BASE = 299


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    seqlens: Tuple[int, ...]
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    chunk: int
    keep_pct: int
    dtype: str  # "f32" | "bf16" | "f16"
    n_layers: int
    n_spans: Tuple[int, ...]  # per sequence
    span_len: Tuple[int, int]
    strength: float
    span_overlap: float = 0.8
    layout: str = "hnd"  # "hnd": [B][Hkv][L][d] ; "nhd": [sum L][Hkv][d]

    @property
    def batch(self) -> int:
        return len(self.seqlens)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self):
        return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[self.dtype]

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def with_(self, **kw) -> "Workload":
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


def keep_budget(seqlen: int, window: int, pct: int) -> int:
    """Number of non-window tokens the harness asks to keep: floor(pct * P / 100)."""
    return (pct * (seqlen - window)) // 100


def _ragged_lengths(batch: int = 8) -> Tuple[int, ...]:
    rng = np.random.default_rng(SEED_BASE + 5000)
    return tuple(int(4096 + rng.integers(0, 61441)) for _ in range(batch))


def _mk() -> dict:
    w = {}
    w["tiny"] = Workload("tiny", 1, (512,), 4, 2, 64, 16, 8, 25, "f32", 1, (3,), (5, 20), 2.0)
    w["llama8b_8k"] = Workload("llama8b_8k", 2, (8192,), 32, 8, 128, 32, 10, 10, "bf16", 1,
                               (40,), (3, 30), 1.5)
    w["llama8b_32k_stack"] = Workload("llama8b_32k_stack", 3, (32768,), 32, 8, 128, 32, 10, 10,
                                      "bf16", 32, (160,), (3, 30), 1.5)
    w["llama8b_128k_stack"] = Workload("llama8b_128k_stack", 4, (131072,), 32, 8, 128, 64, 10, 10,
                                       "bf16", 32, (400,), (3, 30), 1.5)
    lens = _ragged_lengths()
    w["ragged_b8"] = Workload("ragged_b8", 5, lens, 28, 4, 128, 32, 10, 10, "bf16", 28,
                              tuple(L // 200 for L in lens), (3, 30), 1.5, layout="nhd")
    return w


WORKLOADS = _mk()


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


@dataclass
class LayerInputs:
    """One layer's tensors plus the layout description the C-ABI needs."""
    q: torch.Tensor            # [B][Hq][w][d], contiguous
    k: torch.Tensor            # storage buffer (see layout)
    v: torch.Tensor
    seqlens: Tuple[int, ...]
    kv_base: Tuple[int, ...]   # element offset of sequence b inside k / v
    kv_stride_head: int
    kv_stride_tok: int
    spans: List[List[Tuple[int, int]]] = field(default_factory=list)

    def seq_view(self, t: torch.Tensor, b: int, n_kv_heads: int, head_dim: int) -> torch.Tensor:
        """Strided [Hkv][L_b][d] view of sequence ``b`` inside buffer ``t``."""
        return torch.as_strided(t.reshape(-1), (n_kv_heads, self.seqlens[b], head_dim),
                                (self.kv_stride_head, self.kv_stride_tok, 1), self.kv_base[b])


def kv_layout(wl: Workload):
    """(buffer shape, kv_base, stride_head, stride_tok) for the workload's layout."""
    d, h = wl.head_dim, wl.n_kv_heads
    if wl.layout == "hnd":
        L = wl.seqlens[0]
        if any(x != L for x in wl.seqlens):
            raise ValueError("hnd layout needs equal sequence lengths")
        shape = (wl.batch, h, L, d)
        base = tuple(b * h * L * d for b in range(wl.batch))
        return shape, base, L * d, d
    if wl.layout == "nhd":
        cu = np.concatenate([[0], np.cumsum(wl.seqlens)])
        shape = (int(cu[-1]), h, d)
        base = tuple(int(c) * h * d for c in cu[:-1])
        return shape, base, d, h * d
    raise ValueError(wl.layout)


def _draw_span(rng, P: int, span_len) -> Tuple[int, int]:
    n = int(rng.integers(span_len[0], span_len[1] + 1))
    n = max(1, min(n, P))
    s = int(rng.integers(0, P - n + 1))
    return s, n


def layer_spans(wl: Workload, layer: int) -> List[List[Tuple[int, int]]]:
    """Span sets of every sequence at ``layer`` (chained from layer 0)."""
    out = []
    for b, L in enumerate(wl.seqlens):
        P = L - wl.window
        spans: List[Tuple[int, int]] = []
        for l in range(layer + 1):
            rng = np.random.default_rng([SEED_BASE + 1000 * wl.cfg_id + l, b, 17])
            if l == 0 or P <= 0:
                spans = [_draw_span(rng, P, wl.span_len) for _ in range(wl.n_spans[b])] if P > 0 else []
            else:
                keep = rng.random(len(spans)) < wl.span_overlap
                spans = [s if kp else _draw_span(rng, P, wl.span_len) for s, kp in zip(spans, keep)]
        out.append(spans)
    return out


def layer_direction(wl: Workload, layer: int) -> np.ndarray:
    rng = np.random.default_rng([SEED_BASE + 1000 * wl.cfg_id + layer, 23])
    u = rng.standard_normal(wl.head_dim)
    return (u / np.linalg.norm(u)).astype(np.float32)


def make_layer(wl: Workload, layer: int, device="cpu") -> LayerInputs:
    """Draw one layer's Q_obs, K, V in the workload's storage type and layout."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED_BASE + 1000 * wl.cfg_id + layer)
    shape, base, s_head, s_tok = kv_layout(wl)
    B, Hq, Hkv, d, w = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window
    u = torch.from_numpy(layer_direction(wl, layer)).to(dev)
    spans = layer_spans(wl, layer)

    q = torch.randn((B, Hq, w, d), generator=gen, device=dev, dtype=torch.float32)
    q += wl.strength * u
    k = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32)
    li = LayerInputs(q=q, k=k, v=k, seqlens=tuple(wl.seqlens), kv_base=base,
                     kv_stride_head=s_head, kv_stride_tok=s_tok, spans=spans)
    for b in range(B):
        kb = li.seq_view(k, b, Hkv, d)
        for (s, n) in spans[b]:
            kb[:, s:s + n, :] += wl.strength * u
    k = k.to(wl.torch_dtype)
    v = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(wl.torch_dtype)
    li.q = q.to(wl.torch_dtype).contiguous()
    li.k = k
    li.v = v
    return li


def tensor_bits(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor's stored bits: float32 or float16 array, or uint16 array for bf16."""
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
