"""CPU oracle for ChunkKV prefill-time KV-cache compression.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 statement of what the compression path computes, written
from the paper (ChunkKV, arXiv 2502.00299): Algorithm 1 (Section 3.2),
Algorithm 2 (Section 3.3, layer-wise index reuse) and Algorithm 3 (Appendix
A.5, the mask-based formulation).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does.  It
shares no code with the HIP path.

Every function works on ONE sequence (no batch dimension); heads are explicit.

Readings taken where the paper is silent or its listings disagree
(each is also listed in the design document):
  R1  The listings write A = Q_obs K^T; the text calls A "attention scores" in
      the H2O/SnapKV sense, so A is softmax(Q_obs K^T / sqrt(d)) row by row.
  R2  A window row i (0-based, the query at position P+i) sees keys 0..P+i
      (causal prefill attention); its softmax runs over exactly those keys.
  R3  Only the P = L - w non-window columns are chunked and ranked; the window
      is kept unconditionally (Algorithm 3 ORs the window into the mask;
      Algorithm 1 appends it), so the budget counts non-window tokens.
  R4  Exactly n_keep non-window tokens are kept: chunks are taken whole in rank
      order and the last-ranked one is cut to its leading tokens (Algorithm 1's
      truncation to L_max - w rows and the "size of the last chunk" sentence
      of Section 3.2).
  R5  The ragged last chunk is a candidate scored by the sum over its fewer
      tokens (Algorithm 3, end = min((i+1)c, T_k)).
  R6  Equal chunk scores rank the lower chunk index first.
  R7  Grouped-query attention: the selection is per kv-head; a token's
      importance is the plain sum of its probabilities over the w window rows
      of all g query heads that share the kv-head (Algorithm 3 sums over q).
  R8  Kept tokens keep their original order; the window comes last.
  R15 The whole-chunk variant (Algorithm 3 as printed): k = min(floor(n_keep/c), C)
      chunks, none cut; the kept count then depends on the data (ragged tail).
  R16 Decoding over the compressed cache (the stage whose cache Eq. 1 sizes and
      whose latency Section 4.4 tabulates) is ordinary scaled-dot-product
      attention of ONE new query token per head over every token of K', V':
      softmax(q K'^T / sqrt(d)) V', query head i reading kv-head i // g; the
      paper does not restate it.
  R17 A chunk size per layer group (the hybrid ablation of Section 4.6 runs a different setting in the bottom
      and in the top half of the layers; chunk size 1 is token-level selection): every layer of a reuse group
      uses its group's chunk size, the budget is the same token count everywhere.
  R18 The two quality metrics of Appendix A.1 (the paper names them, gives no formula):
      KV cache L1 loss = sum |X - X~| / sum |X| over all K and V entries of a layer, X~ being the cache with
      the dropped tokens zeroed, i.e. the share of the cache's absolute mass that sits in dropped tokens
      (0 when everything is kept; about 0.9 at a 10 % budget, the range the paper's table shows);
      attention cosine similarity = cosine between the attention distribution of the decoding query over the
      full cache and the one over the kept tokens (scattered to their positions, zero elsewhere), per query
      head, averaged over the heads of the layer.
  R13 Caller-supplied row normalisation (the variant for callers that run behind
      a fused attention kernel): the natural log-sum-exp of the scaled logits
      over the keys the row sees, window keys up to its own position included.

Pins (tests/test_oracle_pins.py): rows of the softmax sum to one; invariance to
adding a constant vector to every key; w = g = 1 reduces to a library softmax;
identical keys give p = 1/(P+i+1) in closed form, which also fixes the chunk
grid and the ragged tail; a one-hot key gives a closed form that fixes the
scale 1/sqrt(d) and the query-head-to-kv-head map; brute-force enumeration of
the token order for tiny P; c = 1 reduces to a stable library argsort; uniform
scores keep tokens [0, n_keep); nesting of kept sets; identity at n_keep = P;
R = 1 equals per-layer compression; R >= N reuses layer 0 everywhere; the
log-sum-exp equals a library logsumexp over the visible logits, scores from it
equal the plain scores, and a shift of the log-sum-exp scales them by exp(-shift);
the Jaccard similarity is pinned on hand-counted overlaps; decode attention
is pinned on one token (returns its value row), identical keys (mean of the
value rows), a dominant key, a library scaled-dot-product attention, explicit
loops, a library logsumexp, and the rule that merges two partial results;
the quality metrics are pinned on identity (everything kept: loss 0, cosine 1), on closed forms for
constant-magnitude caches (loss = dropped share of tokens) and identical keys (cosine = sqrt(kept / all)),
on a hand-computed three-token example and on the identity cosine^2 = sum of squared full-cache
probabilities over the kept tokens / over all tokens;
the cache-size formula reproduces the worked example printed beside Eq. 1
(tests/golden/eq1_kv_cache_memory.json) and the reuse speed-up model its stated limit.
The paper prints no worked numeric example of this path, so parity on real
prompts is unpinned; everything above is pinned by mathematics only.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np


def widen(x: np.ndarray) -> np.ndarray:
    """Stored values to float64, exactly.  uint16 arrays are bf16 bit patterns; float16 and float32 arrays widen as is."""
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def n_chunks(P: int, c: int) -> int:
    """C = ceil(P / c) (Algorithm 1; applied to the non-window columns, reading R3)."""
    return (P + c - 1) // c


def window_probabilities(q_rows: np.ndarray, k: np.ndarray, w: int, scale: Optional[float] = None):
    """Softmax attention of the window rows of ONE kv-head (Algorithm 1, first
    step, with readings R1 and R2).

    q_rows: [g*w][d] float64, row r = (query head within the group)*w + i.
    k:      [L][d]  float64.
    Returns p [g*w][L] with p[r, j] = 0 for the keys row r cannot see.
    """
    L, d = k.shape
    P = L - w
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    s = (q_rows @ k.T) * scale                      # logits, [g*w][L]
    i_of_row = np.arange(q_rows.shape[0]) % w       # window position of each row
    visible = np.arange(L)[None, :] <= (P + i_of_row)[:, None]
    s = np.where(visible, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)                                   # exp(-inf) = 0 for hidden keys
    return e / e.sum(axis=1, keepdims=True)


def token_importance(q_obs: np.ndarray, k: np.ndarray, w: int, scale: Optional[float] = None) -> np.ndarray:
    """Per-kv-head importance of every non-window token (reading R7).

    q_obs: [Hq][w][d], k: [Hkv][L][d] (stored values or float64).  Returns [Hkv][P].
    """
    q_obs, k = widen(q_obs), widen(k)
    Hq, Hkv = q_obs.shape[0], k.shape[0]
    g = Hq // Hkv
    L = k.shape[1]
    P = L - w
    out = np.zeros((Hkv, P))
    for h in range(Hkv):
        rows = q_obs[h * g:(h + 1) * g].reshape(g * w, -1)   # heads h*g .. h*g+g-1
        p = window_probabilities(rows, k[h], w, scale)
        out[h] = p[:, :P].sum(axis=0)
    return out


def chunk_sums(imp: np.ndarray, c: int) -> np.ndarray:
    """Chunk scores: chunk i sums tokens i*c .. min((i+1)c, P)-1 (Algorithm 3's
    chunk-score loop; reading R5 for the ragged tail).  imp: [..., P]."""
    P = imp.shape[-1]
    C = n_chunks(P, c)
    out = np.zeros(imp.shape[:-1] + (C,))
    for i in range(C):
        out[..., i] = imp[..., i * c:min((i + 1) * c, P)].sum(axis=-1)
    return out


def score(q_obs: np.ndarray, k: np.ndarray, w: int, c: int, scale: Optional[float] = None):
    """(chunk_scores [Hkv][C], token_importance [Hkv][P]) of one sequence."""
    imp = token_importance(q_obs, k, w, scale)
    return chunk_sums(imp, c), imp


def row_log_sum_exp(q_obs: np.ndarray, k: np.ndarray, w: int, scale: Optional[float] = None) -> np.ndarray:
    """ln of the softmax denominator of every window row: lse[hq][i] = ln sum_{j <= P+i} exp(scale * q_i . k_j)
    over the keys the row sees (readings R1, R2).  This is what a fused prefill attention kernel leaves
    behind for each query row (the paper runs behind FlashAttention-2, Section 4.1 setup).
    q_obs: [Hq][w][d], k: [Hkv][L][d].  Returns [Hq][w]."""
    q_obs, k = widen(q_obs), widen(k)
    Hq, Hkv = q_obs.shape[0], k.shape[0]
    g = Hq // Hkv
    L, d = k.shape[1], k.shape[2]
    P = L - w
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((Hq, w))
    for hq in range(Hq):
        s = (q_obs[hq] @ k[hq // g].T) * scale               # [w][L]
        for i in range(w):
            row = s[i, :P + i + 1]
            m = row.max()
            out[hq, i] = m + math.log(np.exp(row - m).sum())
    return out


def token_importance_from_lse(q_obs: np.ndarray, k: np.ndarray, lse: np.ndarray, w: int,
                              scale: Optional[float] = None) -> np.ndarray:
    """Per-kv-head token importance when the caller supplies each window row's log-sum-exp:
    p[r, j] = exp(scale * q_r . k_j - lse_r) for the non-window keys j < P, summed over the g*w rows of the
    group (reading R7).  With lse = row_log_sum_exp(...) this is token_importance(...).
    q_obs: [Hq][w][d], k: [Hkv][L][d], lse: [Hq][w].  Returns [Hkv][P]."""
    q_obs, k, lse = widen(q_obs), widen(k), np.asarray(lse, dtype=np.float64)
    Hq, Hkv = q_obs.shape[0], k.shape[0]
    g = Hq // Hkv
    L, d = k.shape[1], k.shape[2]
    P = L - w
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((Hkv, P))
    for hq in range(Hq):
        s = (q_obs[hq] @ k[hq // g][:P].T) * scale           # [w][P]: every window row sees all of [0, P)
        out[hq // g] += np.exp(s - lse[hq][:, None]).sum(axis=0)
    return out


def score_from_lse(q_obs: np.ndarray, k: np.ndarray, lse: np.ndarray, w: int, c: int,
                   scale: Optional[float] = None):
    """(chunk_scores [Hkv][C], token_importance [Hkv][P]) of one sequence from caller-supplied row log-sum-exps."""
    imp = token_importance_from_lse(q_obs, k, lse, w, scale)
    return chunk_sums(imp, c), imp


def chunk_topk(scores: np.ndarray, P: int, c: int, n_keep: int) -> Tuple[np.ndarray, np.ndarray]:
    """Selection of ONE (sequence, kv-head) from its chunk scores (Algorithm 1's
    top-k step under readings R4-R6, R8).

    The P non-window tokens are put in the order (chunk score descending, chunk
    index ascending, position ascending); the first n_keep of them are kept.
    Returned as ascending (chunk index, number of leading tokens kept) pairs.
    """
    C = n_chunks(P, c)
    assert scores.shape == (C,)
    assert 0 <= n_keep <= P
    assert np.all(np.isfinite(scores))
    rank = np.argsort(-scores, kind="stable")      # ties: lower index first
    order = np.concatenate([np.arange(i * c, min((i + 1) * c, P)) for i in rank]) if C else np.zeros(0, int)
    kept = np.sort(order[:n_keep])
    chunks, lens = np.unique(kept // c, return_counts=True)
    return chunks.astype(np.int32), lens.astype(np.int32)


def chunk_topk_whole(scores: np.ndarray, P: int, c: int, n_keep: int) -> Tuple[np.ndarray, np.ndarray]:
    """Selection of ONE (sequence, kv-head) as Algorithm 3 prints it (Appendix A.5): the
    k = min(floor(n_keep / c), C) highest-scoring chunks are kept whole (ties to the lower index, reading
    R6) and nothing is cut, so k*c tokens are kept, or fewer when the ragged last chunk is among them.
    Returned as ascending (chunk index, chunk size) pairs."""
    C = n_chunks(P, c)
    assert scores.shape == (C,) and 0 <= n_keep <= P
    k = min(n_keep // c, C)
    rank = np.argsort(-scores, kind="stable")[:k]
    chunks = np.sort(rank)
    lens = np.minimum(c, P - chunks * c)
    return chunks.astype(np.int32), lens.astype(np.int32)


def kept_token_indices(sel_chunk: np.ndarray, sel_len: np.ndarray, L: int, w: int, c: int) -> np.ndarray:
    """Token indices a selection keeps, ascending, window last (reading R8)."""
    P = L - w
    parts = [np.arange(int(ch) * c, int(ch) * c + int(n)) for ch, n in zip(sel_chunk, sel_len)]
    parts.append(np.arange(P, L))
    return np.concatenate(parts).astype(np.int64)


def kept_prefix_tokens(sel_chunk: Sequence[int], sel_len: Sequence[int], c: int) -> np.ndarray:
    """Non-window token indices a selection keeps: the leading sel_len[e] tokens of chunk sel_chunk[e]."""
    if len(sel_chunk) == 0:
        return np.zeros(0, dtype=np.int64)
    return np.concatenate([np.arange(int(ch) * c, int(ch) * c + int(ln)) for ch, ln in zip(sel_chunk, sel_len)])


def jaccard(sel_a, sel_b, c: int) -> float:
    """Jaccard similarity |A n B| / |A u B| of the non-window token sets two selections keep (the
    adjacent-layer similarity of preserved indices that motivates index reuse, Section 3.3 and the tables
    of Appendix B.2).  The window is left out (every layer keeps it).  Two empty sets are identical: 1.
    sel_a, sel_b: (chunks, lens) pairs as chunk_topk returns them."""
    a = kept_prefix_tokens(sel_a[0], sel_a[1], c)
    b = kept_prefix_tokens(sel_b[0], sel_b[1], c)
    union = np.union1d(a, b).size
    return 1.0 if union == 0 else np.intersect1d(a, b).size / union


def compact(k: np.ndarray, v: np.ndarray, sel_chunk: Sequence[np.ndarray], sel_len: Sequence[np.ndarray],
            w: int, c: int):
    """Gather of one sequence (Algorithm 1's index_select + concatenation).

    k, v: [Hkv][L][d] in their stored type (copied verbatim, no arithmetic).
    sel_chunk[h], sel_len[h]: selection of kv-head h.  Returns K', V' [Hkv][n_kept][d].
    """
    Hkv, L, _ = k.shape
    ko, vo = [], []
    for h in range(Hkv):
        idx = kept_token_indices(sel_chunk[h], sel_len[h], L, w, c)
        ko.append(k[h][idx])
        vo.append(v[h][idx])
    return np.stack(ko), np.stack(vo)


def kv_cache_bytes(batch: int, seq_len: int, n_layers: int, n_heads: int, head_dim: int, bytes_per_value: int = 2) -> int:
    """Memory of the KV cache in the decoding stage, Eq. 1: 2 (K and V) * B * S * L * N * D * bytes per value
    (2 for float16)."""
    return 2 * batch * seq_len * n_layers * n_heads * head_dim * bytes_per_value


def reuse_speedup(n_layers: int, n_reuse: int, t_compress: float, t_select: float) -> float:
    """Speed-up model of layer-wise index reuse (Appendix B.1.1): N*Tc over (N/R)*Tc + (N - N/R)*Ts, with
    N/R taken as the real-valued quotient the formula prints."""
    scored = n_layers / n_reuse
    return n_layers * t_compress / (scored * t_compress + (n_layers - scored) * t_select)


def decode_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: Optional[float] = None):
    """One decoding step over a (compressed) cache, reading R16.

    q: [Hq][d], one new query token per head; k, v: [Hkv][n][d], every token visible.
    Returns (out [Hq][d], lse [Hq]): out_i = sum_t p_it v_t with p_i = softmax_t(scale * q_i . k_t) over
    the n tokens of kv-head i // g, and lse_i = ln sum_t exp(scale * q_i . k_t).
    """
    q, k, v = widen(q), widen(k), widen(v)
    Hq, d = q.shape
    Hkv, n, _ = k.shape
    g = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((Hq, d))
    lse = np.zeros(Hq)
    for i in range(Hq):
        h = i // g
        s = (k[h] @ q[i]) * scale          # [n] logits
        m = s.max()
        e = np.exp(s - m)
        out[i] = (e / e.sum()) @ v[h]
        lse[i] = m + math.log(e.sum())
    return out, lse


def compress_layer(q_obs, k, v, w: int, c: int, n_keep: int, scale: Optional[float] = None):
    """Algorithm 1 for one layer of one sequence: returns (K', V', selection, chunk_scores)."""
    P = k.shape[1] - w
    cs, _ = score(q_obs, k, w, c, scale)
    sel = [chunk_topk(cs[h], P, c, n_keep) for h in range(k.shape[0])]
    ko, vo = compact(k, v, [s[0] for s in sel], [s[1] for s in sel], w, c)
    return ko, vo, sel, cs


def compress_stack(q_obs_layers, k_layers, v_layers, w: int, c, n_keep: int, reuse: int,
                   scale: Optional[float] = None):
    """Algorithm 2: layer l recomputes its selection when l mod reuse == 0 and
    otherwise gathers with the selection of layer floor(l/reuse)*reuse.

    q_obs_layers[l] may be None for layers that do not recompute.
    c: one chunk size, or one per reuse group (reading R17: group l // reuse scores, selects and gathers with
    its own chunk size; the budget n_keep is the same token count everywhere).
    Returns (list of K', list of V', list of selections per reuse group).
    """
    assert reuse >= 1
    P = k_layers[0].shape[1] - w
    n_groups = (len(k_layers) + reuse - 1) // reuse
    cs_group = [int(c)] * n_groups if np.isscalar(c) else [int(x) for x in c]
    assert len(cs_group) == n_groups
    store = {}
    k_out, v_out, groups = [], [], []
    for l in range(len(k_layers)):
        cg = cs_group[l // reuse]
        if l % reuse == 0:
            cs, _ = score(q_obs_layers[l], k_layers[l], w, cg, scale)
            store[l] = [chunk_topk(cs[h], P, cg, n_keep) for h in range(k_layers[l].shape[0])]
            groups.append(store[l])
        sel = store[(l // reuse) * reuse]
        ko, vo = compact(k_layers[l], v_layers[l], [s[0] for s in sel], [s[1] for s in sel], w, cg)
        k_out.append(ko)
        v_out.append(vo)
    return k_out, v_out, groups


def kv_l1_loss(k: np.ndarray, v: np.ndarray, kept: Sequence[np.ndarray]) -> float:
    """KV cache L1 loss of one layer of one sequence (Appendix A.1, reading R18).

    k, v: [Hkv][L][d]; kept[h]: token indices kv-head h keeps (window included).  The compressed cache is
    compared entry by entry with the full one, dropped tokens counting as zeros:
    sum |X - X~| / sum |X| over K and V."""
    k, v = widen(k), widen(v)
    num = den = 0.0
    for h in range(k.shape[0]):
        mask = np.zeros(k.shape[1], dtype=bool)
        mask[np.asarray(kept[h], dtype=np.int64)] = True
        for x in (k[h], v[h]):
            x_tilde = np.where(mask[:, None], x, 0.0)
            num += np.abs(x - x_tilde).sum()
            den += np.abs(x).sum()
    return num / den if den > 0 else 0.0


def attention_cosine(q: np.ndarray, k: np.ndarray, kept: Sequence[np.ndarray], scale: Optional[float] = None) -> np.ndarray:
    """Attention cosine similarity of one layer of one sequence (Appendix A.1, reading R18), per query head.

    q: [Hq][d], the decoding query; k: [Hkv][L][d]; kept[h]: token indices kv-head h keeps.  For query head i
    (kv-head i // g): p = softmax over all L tokens, p~ = softmax over the kept tokens, written at their
    positions in a vector of zeros; returns cos(p, p~) = p . p~ / (|p| |p~|) for every head."""
    q, k = widen(q), widen(k)
    Hq, d = q.shape
    Hkv, L, _ = k.shape
    g = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros(Hq)
    for i in range(Hq):
        h = i // g
        s = (k[h] @ q[i]) * scale
        p = np.exp(s - s.max())
        p /= p.sum()
        idx = np.asarray(kept[h], dtype=np.int64)
        pc = np.zeros(L)
        if idx.size:
            e = np.exp(s[idx] - s[idx].max())
            pc[idx] = e / e.sum()
        nrm = math.sqrt((p * p).sum()) * math.sqrt((pc * pc).sum())
        out[i] = (p * pc).sum() / nrm if nrm > 0 else 0.0
    return out
