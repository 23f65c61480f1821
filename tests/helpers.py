"""Shared plumbing of the GPU parity tests: build the C-ABI problem for a workload, run the oracle on
the same stored bits, and compare selections under the tie-band rule."""
from __future__ import annotations

from typing import List, Tuple

import numpy as np
import torch

import workloads as W
from oracle import chunkkv_oracle as orc

REL_TOL = 1e-3     # scores: relative tolerance stated by the task (fp32 accumulation on the GPU)
DEFAULT_FLAGS = 0   # chunkkv_problem.flags of every problem make_problem builds (set by the scoring_path fixtures)


def make_problem(pkg, wl: W.Workload, li: W.LayerInputs, n_keep=None, **kw):
    if n_keep is None:
        n_keep = [W.keep_budget(L, wl.window, wl.keep_pct) for L in li.seqlens]
    return pkg.Problem(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                       {"f32": pkg.F32, "bf16": pkg.BF16, "f16": pkg.F16}[wl.dtype], list(li.seqlens), list(n_keep),
                       list(li.kv_base), li.kv_stride_head, li.kv_stride_tok, **{"flags": DEFAULT_FLAGS, **kw})


def seq_arrays(wl: W.Workload, li: W.LayerInputs, b: int):
    """Stored bits of sequence b as numpy: q [Hq][w][d], k, v [Hkv][L][d] (uint16 for bf16, float16 for fp16)."""
    q = W.tensor_bits(li.q[b])
    k = W.tensor_bits(li.seq_view(li.k, b, wl.n_kv_heads, wl.head_dim))
    v = W.tensor_bits(li.seq_view(li.v, b, wl.n_kv_heads, wl.head_dim))
    return q, k, v


def out_view(prob, t: torch.Tensor, b: int) -> torch.Tensor:
    n_kept = int(prob.n_keep[b]) + prob.window
    return torch.as_strided(t.reshape(-1), (prob.n_kv_heads, n_kept, prob.head_dim),
                            (prob.out_stride_head, prob.out_stride_tok, 1), int(prob.out_base[b]))


def read_selection(prob, sel_chunk, sel_len, sel_count, group: int = 0):
    """-> sel[b][h] = (chunks, lens) numpy int32 arrays."""
    B, H = prob.batch, prob.n_kv_heads
    sc = sel_chunk.cpu().numpy().reshape(-1, B, H, prob.sel_cap)[group]
    sl = sel_len.cpu().numpy().reshape(-1, B, H, prob.sel_cap)[group]
    cnt = sel_count.cpu().numpy().reshape(-1, B, H)[group]
    return [[(sc[b, h, :cnt[b, h]].copy(), sl[b, h, :cnt[b, h]].copy()) for h in range(H)] for b in range(B)]


def check_selection(gpu_sel, orc_sel, orc_scores, P: int, c: int, n_keep: int) -> int:
    """Tie-band comparison of one (sequence, kv-head).  Returns the number of chunks that differ.

    Structure must always hold (ascending, valid lengths, exact budget).  Chunk sets must be equal
    except for chunks whose ORACLE score lies within REL_TOL (relative) of the oracle score of the
    oracle's lowest-ranked selected chunk; outside that band the kept lengths must agree too."""
    gc, gl = gpu_sel
    oc, ol = orc_sel
    assert int(gl.sum()) == n_keep, (int(gl.sum()), n_keep)
    assert np.all(np.diff(gc) > 0)
    if len(gc):
        assert gc[0] >= 0 and int(gc[-1]) * c < P
        natural = np.minimum(c, P - gc.astype(np.int64) * c)
        assert np.all((gl >= 1) & (gl <= natural))
        assert int(np.sum(gl < natural)) <= 1
    if n_keep == 0:
        assert len(gc) == 0
        return 0
    thr = float(orc_scores[oc].min())
    band = lambda ch: abs(float(orc_scores[ch]) - thr) <= REL_TOL * thr
    diff = set(gc.tolist()) ^ set(oc.tolist())
    for ch in diff:
        assert band(ch), f"chunk {ch} differs outside the tie band: score {orc_scores[ch]} vs threshold {thr}"
    gmap, omap = dict(zip(gc.tolist(), gl.tolist())), dict(zip(oc.tolist(), ol.tolist()))
    for ch in set(gmap) & set(omap):
        if not band(ch):
            assert gmap[ch] == omap[ch], (ch, gmap[ch], omap[ch])
    return len(diff)


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    gpu = np.asarray(gpu, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    assert np.all(ref > 0)
    return float(np.max(np.abs(gpu - ref) / ref))
