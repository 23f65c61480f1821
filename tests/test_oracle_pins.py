"""Pins for the CPU oracle: each test checks it against something the paper or
the mathematics fixes (closed forms, invariants, library special cases, brute
force on tiny inputs), never against the oracle's own formula or the HIP path.
The paper (ChunkKV, Algorithms 1-3) prints no worked numeric example of the
compression step, so there are no paper values to compare with.
"""
import itertools
import math

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import chunkkv_oracle as orc


def rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------- S1-S2 softmax
@pytest.mark.parametrize("g,w,L,d", [(1, 4, 37, 8), (3, 5, 64, 16), (4, 16, 130, 64)])
def test_rows_sum_to_one_over_visible_keys(g, w, L, d):
    r = rng(1)
    q = r.standard_normal((g * w, d))
    k = r.standard_normal((L, d))
    p = orc.window_probabilities(q, k, w)
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-12)
    P = L - w
    for row in range(g * w):
        i = row % w
        assert np.all(p[row, P + i + 1:] == 0.0)          # hidden keys carry no mass
        assert np.all(p[row, :P + i + 1] > 0.0)


def test_shift_invariance_of_keys():
    # adding one vector to every key adds a per-row constant to the logits
    r = rng(2)
    q = r.standard_normal((2, 4, 16))   # Hq=2, w=4
    k = r.standard_normal((1, 50, 16))
    a = orc.token_importance(q, k, 4)
    b = orc.token_importance(q, k + r.standard_normal(16)[None, None, :], 4)
    assert np.allclose(a, b, rtol=1e-10, atol=1e-14)


def test_single_query_reduces_to_library_softmax():
    # w = 1, g = 1: the only window row sees all L keys -> textbook softmax(K q / sqrt(d))
    r = rng(3)
    d, L = 32, 77
    q = r.standard_normal((1, 1, d))
    k = r.standard_normal((1, L, d))
    imp = orc.token_importance(q, k, 1)
    ref = softmax((k[0] @ q[0, 0]) / math.sqrt(d))
    assert np.allclose(imp[0], ref[:L - 1], rtol=1e-12)


def test_identical_keys_closed_form_and_chunk_grid():
    # all keys equal -> row i is uniform over its P+i+1 visible keys, whatever Q is;
    # importance of every prefix token = g * sum_i 1/(P+i+1); chunk score = size * that
    r = rng(4)
    Hq, Hkv, w, d, L, c = 6, 2, 5, 16, 48, 10     # P = 43 -> chunks of 10,10,10,10,3
    g = Hq // Hkv
    P = L - w
    q = r.standard_normal((Hq, w, d))
    k = np.tile(r.standard_normal((Hkv, 1, d)), (1, L, 1))
    cs, imp = orc.score(q, k, w, c)
    per_tok = g * sum(1.0 / (P + i + 1) for i in range(w))
    assert imp.shape == (Hkv, P)
    assert np.allclose(imp, per_tok, rtol=1e-12)
    sizes = np.array([10, 10, 10, 10, 3])
    assert cs.shape == (Hkv, 5)
    assert np.allclose(cs, sizes[None, :] * per_tok, rtol=1e-12)
    # mass identity: chunk scores sum to the window rows' mass on the prefix
    assert np.allclose(cs.sum(axis=1), g * sum(P / (P + i + 1) for i in range(w)), rtol=1e-12)


def test_one_hot_key_closed_form_pins_scale_and_gqa_map():
    # kv-head 1 has a single non-zero key kappa*u at j*; query head qh has beta_qh*u in
    # every window row.  Logit of (qh, i) on j* is beta_qh*kappa/sqrt(d), zero elsewhere:
    #   p = e^t / (e^t + P + i)   with t = beta_qh*kappa/sqrt(d).
    # kv-head 0 has identical keys (uniform rows).  Heads 3,4,5 belong to kv-head 1.
    Hq, Hkv, w, d, L = 6, 2, 3, 16, 40
    g, P, jstar, kappa = 3, 37, 11, 4.0
    u = np.zeros(d)
    u[2] = 1.0
    beta = np.array([0.5, 1.0, 1.5, 2.0, 2.5, 3.0])
    q = beta[:, None, None] * u[None, None, :] * np.ones((Hq, w, 1))
    k = np.zeros((Hkv, L, d))
    k[0, :, :] = 0.3
    k[1, jstar, :] = kappa * u
    imp = orc.token_importance(q, k, w)
    exp1 = sum(math.exp(beta[qh] * kappa / math.sqrt(d)) /
               (math.exp(beta[qh] * kappa / math.sqrt(d)) + P + i)
               for qh in (3, 4, 5) for i in range(w))
    assert imp[1, jstar] == pytest.approx(exp1, rel=1e-12)
    other = sum(1.0 / (math.exp(beta[qh] * kappa / math.sqrt(d)) + P + i)
                for qh in (3, 4, 5) for i in range(w))
    assert np.allclose(np.delete(imp[1], jstar), other, rtol=1e-12)
    assert np.allclose(imp[0], g * sum(1.0 / (P + i + 1) for i in range(w)), rtol=1e-12)


def test_window_row_i_sees_exactly_its_causal_keys():
    # a huge key placed inside the window at P+2 is visible to rows i >= 2 only
    w, d, L = 4, 8, 20
    P = L - w
    q = np.ones((1, w, d))
    k = np.zeros((1, L, d))
    k[0, P + 2, :] = 50.0
    p = orc.window_probabilities(q[0], k[0], w)
    assert np.allclose(p[0, :P + 1], 1.0 / (P + 1))
    assert np.allclose(p[1, :P + 2], 1.0 / (P + 2))
    assert p[2, P + 2] > 1 - 1e-12 and p[3, P + 2] > 1 - 1e-12


def test_importance_matches_library_logsumexp_per_row():
    # p[r, j] = exp(s_rj - logsumexp_r) with the library's logsumexp over the visible keys
    r = rng(5)
    Hq, Hkv, w, d, L = 4, 2, 3, 8, 21
    g, P = 2, 18
    q = r.standard_normal((Hq, w, d))
    k = r.standard_normal((Hkv, L, d))
    imp = orc.token_importance(q, k, w)
    for h in range(Hkv):
        acc = np.zeros(P)
        for qh in range(h * g, (h + 1) * g):
            for i in range(w):
                s = k[h, :P + i + 1] @ q[qh, i] / math.sqrt(d)
                acc += np.exp(s - logsumexp(s))[:P]
        assert np.allclose(imp[h], acc, rtol=1e-11)


def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x3DCD], dtype=np.uint16)
    vals = orc.widen(bits)
    assert vals[0] == 1.0 and vals[1] == -1.0 and vals[3] == 0.0
    assert vals[2] == 3.140625                      # 0x4049 = 1.5703125 * 2
    assert vals[4] == 0.10009765625


# ----------------------------------------------------------------- S4 selection
def brute_force_kept(scores, P, c, n_keep):
    """Enumerate tokens, sort by (chunk score desc, chunk index asc, position asc)."""
    toks = sorted(range(P), key=lambda t: (-float(scores[t // c]), t // c, t))
    return sorted(toks[:n_keep])


def expand(sel_chunk, sel_len, c):
    return [int(ch) * c + t for ch, n in zip(sel_chunk, sel_len) for t in range(int(n))]


@pytest.mark.parametrize("seed", range(40))
def test_selection_matches_brute_force_on_tiny_inputs(seed):
    r = rng(100 + seed)
    P = int(r.integers(1, 25))
    c = int(r.integers(1, 8))
    C = (P + c - 1) // c
    # few distinct values -> many exact ties
    scores = r.integers(0, 4, size=C).astype(np.float64) / 4.0
    for n_keep in range(P + 1):
        ch, ln = orc.chunk_topk(scores, P, c, n_keep)
        assert expand(ch, ln, c) == brute_force_kept(scores, P, c, n_keep)


def test_chunk_size_one_is_stable_topk():
    r = rng(7)
    P = 200
    imp = np.round(r.random(P), 2)          # ties present
    for n_keep in (0, 1, 17, 100, 200):
        ch, ln = orc.chunk_topk(imp, P, 1, n_keep)
        ref = np.sort(np.argsort(-imp, kind="stable")[:n_keep])
        assert np.array_equal(ch, ref) and np.all(ln == 1)


@pytest.mark.parametrize("P,c,n_keep", [(43, 10, 25), (40, 8, 40), (7, 10, 3), (30, 7, 0)])
def test_uniform_scores_keep_leading_tokens(P, c, n_keep):
    C = (P + c - 1) // c
    ch, ln = orc.chunk_topk(np.full(C, 0.5), P, c, n_keep)
    assert expand(ch, ln, c) == list(range(n_keep))


@pytest.mark.parametrize("seed", range(10))
def test_selection_invariants_and_nesting(seed):
    r = rng(200 + seed)
    P, c = int(r.integers(30, 400)), int(r.integers(2, 21))
    C = (P + c - 1) // c
    scores = r.random(C)
    prev = set()
    for n_keep in range(0, P + 1):
        ch, ln = orc.chunk_topk(scores, P, c, n_keep)
        assert int(ln.sum()) == n_keep
        assert np.all(np.diff(ch) > 0)
        natural = np.minimum(c, P - ch.astype(np.int64) * c)
        assert np.all((ln >= 1) & (ln <= natural))
        assert int(np.sum(ln < natural)) <= 1           # at most one truncated chunk
        kept = set(expand(ch, ln, c))
        assert prev <= kept                              # budget n_keep nests in n_keep+1
        prev = kept


def test_ragged_tail_selected_pulls_next_ranked_chunk():
    # P=23, c=10: chunks of 10, 10, 3.  Tail ranks first; budget 13 = tail + whole chunk 1.
    scores = np.array([0.1, 0.5, 0.9])
    ch, ln = orc.chunk_topk(scores, 23, 10, 13)
    assert list(ch) == [1, 2] and list(ln) == [10, 3]
    ch, ln = orc.chunk_topk(scores, 23, 10, 10)          # tail (3) + 7 leading of chunk 1
    assert list(ch) == [1, 2] and list(ln) == [7, 3]
    ch, ln = orc.chunk_topk(scores, 23, 10, 14)          # spills one token into chunk 0
    assert list(ch) == [0, 1, 2] and list(ln) == [1, 10, 3]


# ----------------------------------------------------------------- S5 gather
def test_gather_identity_and_window():
    r = rng(9)
    Hkv, L, d, w, c = 2, 53, 4, 5, 6
    P = L - w
    k = r.standard_normal((Hkv, L, d)).astype(np.float32)
    v = r.standard_normal((Hkv, L, d)).astype(np.float32)
    full = [orc.chunk_topk(np.arange(orc.n_chunks(P, c), dtype=float), P, c, P) for _ in range(Hkv)]
    ko, vo = orc.compact(k, v, [s[0] for s in full], [s[1] for s in full], w, c)
    assert ko.tobytes() == k.tobytes() and vo.tobytes() == v.tobytes()
    none = [(np.zeros(0, np.int32), np.zeros(0, np.int32))] * Hkv
    ko, vo = orc.compact(k, v, [s[0] for s in none], [s[1] for s in none], w, c)
    assert np.array_equal(ko, k[:, P:]) and np.array_equal(vo, v[:, P:])
    # chunks 1 (whole) and 4 (two leading tokens): tokens 6..11 and 24,25, then the window
    ch, ln = np.array([1, 4], np.int32), np.array([6, 2], np.int32)
    idx = orc.kept_token_indices(ch, ln, L, w, c)
    assert list(idx) == [6, 7, 8, 9, 10, 11, 24, 25] + list(range(P, L))
    ko, vo = orc.compact(k, v, [ch, ch], [ln, ln], w, c)
    for h in range(Hkv):
        assert np.array_equal(ko[h], np.concatenate([k[h, 6:12], k[h, 24:26], k[h, P:]]))
        assert np.array_equal(vo[h], np.concatenate([v[h, 6:12], v[h, 24:26], v[h, P:]]))


def test_gather_rows_are_verbatim_copies():
    r = rng(10)
    Hkv, L, d, w, c = 1, 40, 8, 4, 5
    k = r.integers(0, 65536, size=(Hkv, L, d)).astype(np.uint16)   # arbitrary bf16 bit patterns, NaNs included
    v = r.integers(0, 65536, size=(Hkv, L, d)).astype(np.uint16)
    ch, ln = np.array([0, 3, 6], np.int32), np.array([5, 2, 5], np.int32)
    ko, vo = orc.compact(k, v, [ch], [ln], w, c)
    rows = list(range(0, 5)) + [15, 16] + list(range(30, 35)) + list(range(36, 40))
    assert ko.shape == (1, len(rows), d)
    assert np.array_equal(ko[0], k[0, rows]) and np.array_equal(vo[0], v[0, rows])


# ----------------------------------------------------------------- S6 reuse
def _stack(seed, N, Hq=4, Hkv=2, L=60, d=8, w=4):
    r = rng(seed)
    qs = [r.standard_normal((Hq, w, d)) for _ in range(N)]
    ks = [r.standard_normal((Hkv, L, d)) for _ in range(N)]
    vs = [r.standard_normal((Hkv, L, d)) for _ in range(N)]
    return qs, ks, vs


def test_reuse_one_equals_per_layer():
    qs, ks, vs = _stack(11, 5)
    w, c, n_keep = 4, 6, 20
    ko, vo, groups = orc.compress_stack(qs, ks, vs, w, c, n_keep, 1)
    assert len(groups) == 5
    for l in range(5):
        k1, v1, sel, _ = orc.compress_layer(qs[l], ks[l], vs[l], w, c, n_keep)
        assert np.array_equal(ko[l], k1) and np.array_equal(vo[l], v1)


@pytest.mark.parametrize("N,R", [(5, 2), (5, 3), (4, 7), (6, 6)])
def test_reuse_groups_share_the_leader_selection(N, R):
    qs, ks, vs = _stack(12, N)
    w, c, n_keep = 4, 6, 20
    ko, vo, groups = orc.compress_stack([q if l % R == 0 else None for l, q in enumerate(qs)],
                                        ks, vs, w, c, n_keep, R)
    assert len(groups) == (N + R - 1) // R
    for l in range(N):
        leader = (l // R) * R
        _, _, sel, _ = orc.compress_layer(qs[leader], ks[leader], vs[leader], w, c, n_keep)
        k1, v1 = orc.compact(ks[l], vs[l], [s[0] for s in sel], [s[1] for s in sel], w, c)
        assert np.array_equal(ko[l], k1) and np.array_equal(vo[l], v1)
        assert ko[l].shape == (2, n_keep + w, 8)


def test_keep_everything_is_identity_through_the_stack():
    qs, ks, vs = _stack(13, 3)
    w, c = 4, 6
    ko, vo, _ = orc.compress_stack(qs, ks, vs, w, c, 60 - w, 2)
    for l in range(3):
        assert np.array_equal(ko[l], ks[l]) and np.array_equal(vo[l], vs[l])


def test_per_group_chunk_sizes_equal_separate_stacks():
    # reading R17: a stack with a chunk size per reuse group is the concatenation of uniform stacks over the
    # runs of groups; chunk size 1 in a group is plain token-level top-k there
    qs, ks, vs = _stack(15, 7)
    w, n_keep, R = 4, 20, 2
    cs = [6, 1, 9, 3]
    ko, vo, groups = orc.compress_stack([q if l % R == 0 else None for l, q in enumerate(qs)],
                                        ks, vs, w, cs, n_keep, R)
    assert len(groups) == 4
    for g, c in enumerate(cs):
        lo, hi = g * R, min(7, (g + 1) * R)
        k1, v1, g1 = orc.compress_stack([qs[lo]] + [None] * (hi - lo - 1), ks[lo:hi], vs[lo:hi], w, c, n_keep, R)
        for l in range(lo, hi):
            assert np.array_equal(ko[l], k1[l - lo]) and np.array_equal(vo[l], v1[l - lo])
            assert ko[l].shape == (2, n_keep + w, 8)
    # the token-level group keeps exactly the n_keep highest-importance prefix tokens of its leader
    _, imp = orc.score(qs[2], ks[2], w, 1)
    for h in range(2):
        top = np.sort(np.argsort(-imp[h], kind="stable")[:n_keep])
        assert np.array_equal(np.sort(groups[1][h][0]), top)
        assert np.all(groups[1][h][1] == 1)


def test_uniform_chunk_list_equals_scalar_chunk():
    qs, ks, vs = _stack(16, 5)
    a = orc.compress_stack(qs, ks, vs, 4, 6, 20, 2)
    b = orc.compress_stack(qs, ks, vs, 4, [6, 6, 6], 20, 2)
    for x, y in zip(a[0] + a[1], b[0] + b[1]):
        assert np.array_equal(x, y)


def test_planted_span_is_found_when_strong():
    # a strongly planted span must be among the kept chunks (sanity of the whole path)
    r = rng(14)
    Hq, Hkv, w, d, L, c = 2, 1, 4, 32, 200, 10
    P = L - w
    u = r.standard_normal(d)
    u /= np.linalg.norm(u)
    q = r.standard_normal((Hq, w, d)) + 6.0 * u
    k = r.standard_normal((Hkv, L, d))
    k[0, 70:80] += 6.0 * u
    v = r.standard_normal((Hkv, L, d))
    _, _, sel, cs = orc.compress_layer(q, k, v, w, c, 20)
    assert 7 in list(sel[0][0]) and int(np.argmax(cs[0])) == 7


# ---------------------------------------------------------------- caller-supplied log-sum-exp (reading R13)
def test_row_log_sum_exp_is_library_logsumexp_over_visible_keys():
    r = rng(31)
    Hq, Hkv, w, d, L = 6, 2, 4, 8, 27
    g, P = 3, L - w
    q = r.standard_normal((Hq, w, d)) * 2
    k = r.standard_normal((Hkv, L, d)) * 2
    lse = orc.row_log_sum_exp(q, k, w, scale=0.3)
    for hq in range(Hq):
        for i in range(w):
            s = 0.3 * (k[hq // g, :P + i + 1] @ q[hq, i])
            assert abs(lse[hq, i] - logsumexp(s)) < 1e-12


def test_identical_keys_log_sum_exp_closed_form():
    # all keys equal: every visible logit is s0, so lse = s0 + ln(P + i + 1)
    w, d, L = 3, 4, 11
    P = L - w
    q = np.full((1, w, d), 0.5)
    k = np.full((1, L, d), 2.0)
    s0 = (0.5 * 2.0 * d) / math.sqrt(d)
    lse = orc.row_log_sum_exp(q, k, w)
    assert np.allclose(lse[0], s0 + np.log(P + np.arange(w) + 1), rtol=0, atol=1e-13)


def test_scores_from_own_log_sum_exp_equal_plain_scores():
    r = rng(32)
    Hq, Hkv, w, d, L, c = 8, 2, 5, 16, 64, 7
    q = r.standard_normal((Hq, w, d))
    k = r.standard_normal((Hkv, L, d))
    lse = orc.row_log_sum_exp(q, k, w)
    cs0, imp0 = orc.score(q, k, w, c)
    cs1, imp1 = orc.score_from_lse(q, k, lse, w, c)
    assert np.allclose(imp1, imp0, rtol=1e-12, atol=0) and np.allclose(cs1, cs0, rtol=1e-12, atol=0)


def test_log_sum_exp_shift_scales_one_heads_contribution():
    # lse enters as exp(-lse): raising one query head's values by ln 2 halves exactly that head's share
    r = rng(33)
    Hq, Hkv, w, d, L, c = 4, 2, 3, 8, 30, 4
    q = r.standard_normal((Hq, w, d))
    k = r.standard_normal((Hkv, L, d))
    lse = orc.row_log_sum_exp(q, k, w)
    _, imp = orc.score_from_lse(q, k, lse, w, c)
    only0 = orc.token_importance_from_lse(q[:1], k[:1], lse[:1], w)      # head 0 alone (g = 1 there)
    lse2 = lse.copy()
    lse2[0] += math.log(2.0)
    _, imp2 = orc.score_from_lse(q, k, lse2, w, c)
    assert np.allclose(imp[0] - imp2[0], 0.5 * only0[0], rtol=1e-12)
    assert np.array_equal(imp[1], imp2[1])                                # the other kv-head is untouched


# ---------------------------------------------------------------- adjacent-layer Jaccard similarity
def test_jaccard_hand_counted_cases():
    c = 4
    a = (np.array([0, 2, 5]), np.array([4, 4, 2]))        # tokens 0-3, 8-11, 20-21      (10 tokens)
    b = (np.array([2, 5, 7]), np.array([3, 4, 4]))        # tokens 8-10, 20-23, 28-31    (11 tokens)
    # shared: 8, 9, 10, 20, 21 -> 5 ; union 10 + 11 - 5 = 16
    assert orc.jaccard(a, b, c) == 5 / 16
    assert orc.jaccard(b, a, c) == 5 / 16
    assert orc.jaccard(a, a, c) == 1.0
    assert orc.jaccard(a, (np.array([1, 3]), np.array([4, 4])), c) == 0.0
    empty = (np.zeros(0, int), np.zeros(0, int))
    assert orc.jaccard(empty, empty, c) == 1.0 and orc.jaccard(a, empty, c) == 0.0


def test_jaccard_of_nested_selections_is_the_size_ratio():
    # selections of the same scores with budgets n1 < n2 are nested, so J = n1 / n2
    r = rng(41)
    P, c = 97, 5
    scores = r.random(orc.n_chunks(P, c))
    s1, s2 = orc.chunk_topk(scores, P, c, 23), orc.chunk_topk(scores, P, c, 61)
    assert abs(orc.jaccard(s1, s2, c) - 23 / 61) < 1e-15


# ---------------------------------------------------------------- whole-chunk selection (Algorithm 3 as printed)
@pytest.mark.parametrize("seed", range(6))
def test_whole_chunk_selection_matches_brute_force(seed):
    r = rng(50 + seed)
    P, c = int(r.integers(5, 40)), int(r.integers(1, 7))
    C = orc.n_chunks(P, c)
    scores = r.integers(0, 4, C).astype(np.float64)          # many ties
    n_keep = int(r.integers(0, P + 1))
    chunks, lens = orc.chunk_topk_whole(scores, P, c, n_keep)
    k = min(n_keep // c, C)
    # brute force: the k best chunks under (score desc, index asc), found by repeated selection
    left, best = list(range(C)), []
    for _ in range(k):
        j = max(left, key=lambda i: (scores[i], -i))
        best.append(j)
        left.remove(j)
    assert sorted(best) == chunks.tolist()
    assert lens.tolist() == [min(c, P - ch * c) for ch in sorted(best)]
    assert int(lens.sum()) <= n_keep


def test_whole_chunk_selection_equals_exact_budget_when_nothing_is_cut():
    # n_keep a multiple of c and the ragged tail not among the best: both rules keep the same tokens
    r = rng(57)
    P, c, n_keep = 103, 10, 40
    scores = r.random(orc.n_chunks(P, c))
    scores[-1] = -1.0 + 1.0                                   # tail chunk ranks last (score 0)
    a = orc.chunk_topk(scores, P, c, n_keep)
    b = orc.chunk_topk_whole(scores, P, c, n_keep)
    assert a[0].tolist() == b[0].tolist() and a[1].tolist() == b[1].tolist()
    # a budget that is no multiple of c: the whole-chunk rule keeps floor(n_keep / c) chunks
    assert len(orc.chunk_topk_whole(scores, P, c, 47)[0]) == 4 and int(orc.chunk_topk(scores, P, c, 47)[1].sum()) == 47


# ------------------------------------------------------------------ decode attention over the compressed cache
def _rand_decode(seed, Hq=6, Hkv=2, n=37, d=8):
    r = np.random.default_rng(seed)
    return r.normal(size=(Hq, d)), r.normal(size=(Hkv, n, d)), r.normal(size=(Hkv, n, d))


def test_decode_one_token_returns_its_value_row():
    q, k, v = _rand_decode(0, n=1)
    out, lse = orc.decode_attention(q, k, v)
    for i in range(6):
        assert np.allclose(out[i], v[i // 3, 0], rtol=0, atol=1e-15)
        assert math.isclose(lse[i], float(q[i] @ k[i // 3, 0]) / math.sqrt(8), rel_tol=1e-13, abs_tol=1e-13)


def test_decode_identical_keys_average_the_value_rows():
    q, k, v = _rand_decode(1)
    k[:] = k[:, :1]                                   # every token of a head carries the same key
    out, lse = orc.decode_attention(q, k, v)
    for i in range(6):
        assert np.allclose(out[i], v[i // 3].mean(axis=0), rtol=1e-13, atol=1e-13)
        assert math.isclose(lse[i], float(q[i] @ k[i // 3, 0]) / math.sqrt(8) + math.log(37), rel_tol=1e-12)


def test_decode_dominant_key_pins_scale_and_head_map():
    """Head 4 (kv-head 1 when g = 3) meets one key aligned with it: weight 1/(1 + (n-1) exp(-scale*|q|^2))."""
    Hq, Hkv, n, d = 6, 2, 9, 16
    q = np.zeros((Hq, d)); k = np.zeros((Hkv, n, d)); v = np.random.default_rng(2).normal(size=(Hkv, n, d))
    q[4, 3] = 5.0
    k[1, 6, 3] = 5.0                                   # only kv-head 1 holds the matching key
    out, _ = orc.decode_attention(q, k, v)
    pw = 1.0 / (1.0 + (n - 1) * math.exp(-25.0 / 4.0))  # scale = 1/sqrt(16)
    rest = (v[1].sum(axis=0) - v[1, 6]) * (1 - pw) / (n - 1)
    assert np.allclose(out[4], pw * v[1, 6] + rest, rtol=1e-12, atol=1e-12)
    assert np.allclose(out[1], v[0].mean(axis=0), rtol=1e-12, atol=1e-12)   # a zero query averages kv-head 0
    out2, _ = orc.decode_attention(q, k, v, scale=1.0)
    pw2 = 1.0 / (1.0 + (n - 1) * math.exp(-25.0))
    assert np.allclose(out2[4], pw2 * v[1, 6] + (v[1].sum(axis=0) - v[1, 6]) * (1 - pw2) / (n - 1), rtol=1e-12)


def test_decode_equals_library_attention_and_logsumexp():
    import torch
    import torch.nn.functional as F
    q, k, v = _rand_decode(3, Hq=8, Hkv=2, n=53, d=16)
    out, lse = orc.decode_attention(q, k, v)
    tq = torch.from_numpy(q)[None, :, None, :]                         # [1][Hq][1][d]
    tk = torch.from_numpy(k).repeat_interleave(4, dim=0)[None]         # kv-head h serves heads 4h..4h+3
    tv = torch.from_numpy(v).repeat_interleave(4, dim=0)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv)[0, :, 0].numpy()
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
    for i in range(8):
        assert math.isclose(lse[i], float(logsumexp(k[i // 4] @ q[i] / 4.0)), rel_tol=1e-13)


def test_decode_equals_explicit_loops_on_tiny_input():
    q, k, v = _rand_decode(4, Hq=4, Hkv=2, n=5, d=3)
    out, _ = orc.decode_attention(q, k, v, scale=0.7)
    for i in range(4):
        h = i // 2
        wts = [math.exp(0.7 * sum(q[i, e] * k[h, t, e] for e in range(3))) for t in range(5)]
        for e in range(3):
            assert math.isclose(out[i, e], sum(wts[t] * v[h, t, e] for t in range(5)) / sum(wts), rel_tol=1e-12, abs_tol=1e-14)


def test_decode_partial_results_merge_by_their_log_sum_exps():
    """Attention over a cache split in two equals the lse-weighted mean of the parts (what lets key ranges be
    processed independently); a wrong lse or a transposed operand breaks it."""
    q, k, v = _rand_decode(5, n=41)
    out, lse = orc.decode_attention(q, k, v)
    oa, la = orc.decode_attention(q, k[:, :17], v[:, :17])
    ob, lb = orc.decode_attention(q, k[:, 17:], v[:, 17:])
    wa = 1.0 / (1.0 + np.exp(lb - la))
    assert np.allclose(out, wa[:, None] * oa + (1 - wa)[:, None] * ob, rtol=1e-12, atol=1e-13)
    assert np.allclose(lse, np.logaddexp(la, lb), rtol=1e-13)


def test_decode_widens_stored_16_bit_values_exactly():
    import torch
    r = np.random.default_rng(6)
    qf, kf, vf = r.normal(size=(2, 8)), r.normal(size=(1, 11, 8)), r.normal(size=(1, 11, 8))
    want, _ = orc.decode_attention(torch.tensor(qf).bfloat16().double().numpy(), torch.tensor(kf).bfloat16().double().numpy(),
                                   torch.tensor(vf).bfloat16().double().numpy())
    bits = lambda x: torch.tensor(x).bfloat16().view(torch.int16).numpy().view(np.uint16)
    got, _ = orc.decode_attention(bits(qf), bits(kf), bits(vf))
    assert np.array_equal(got, want)
    got16, _ = orc.decode_attention(qf.astype(np.float16), kf.astype(np.float16), vf.astype(np.float16))
    want16, _ = orc.decode_attention(qf.astype(np.float16).astype(np.float64), kf.astype(np.float16).astype(np.float64),
                                     vf.astype(np.float16).astype(np.float64))
    assert np.array_equal(got16, want16)


# ------------------------------------------------------------------ sizing formulas the paper states
def test_cache_size_formula_reproduces_the_papers_worked_example():
    import json
    import os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "eq1_kv_cache_memory.json")))
    m = orc.kv_cache_bytes(**g["inputs"])
    assert m == g["bytes"] == 2 ** 30                    # "nearly 1 GB": exactly 1 GiB
    inp = dict(g["inputs"])
    inp["batch"] = 24
    assert orc.kv_cache_bytes(**inp) <= g["card_bytes"]  # 24 sequences still fit a 24 GiB card ...
    inp["batch"] = 25
    assert orc.kv_cache_bytes(**inp) > g["card_bytes"]   # ... "exceeds 24" does not
    # linear in every factor
    assert orc.kv_cache_bytes(2, 3, 5, 7, 11, 2) == 2 * 2 * 3 * 5 * 7 * 11 * 2


def test_reuse_speedup_model_limits():
    assert orc.reuse_speedup(32, 1, 3.0, 0.5) == 1.0                       # no reuse, no gain
    assert math.isclose(orc.reuse_speedup(32, 2, 1.0, 0.0), 2.0)          # negligible gather time: about R
    assert math.isclose(orc.reuse_speedup(32, 4, 1.0, 0.0), 4.0)
    # a gather as expensive as a full compression gains nothing; in between the closed form by hand
    assert math.isclose(orc.reuse_speedup(32, 2, 1.0, 1.0), 1.0)
    assert math.isclose(orc.reuse_speedup(32, 2, 1.0, 0.287), 32 / (16 + 16 * 0.287))


# ----------------------------------------------------------------- quality metrics (Appendix A.1, reading R18)
def test_quality_metrics_keep_everything_is_lossless():
    r = rng(40)
    k, v, q = r.standard_normal((2, 30, 8)), r.standard_normal((2, 30, 8)), r.standard_normal((4, 8))
    kept = [np.arange(30), np.arange(30)]
    assert orc.kv_l1_loss(k, v, kept) == 0.0
    assert np.allclose(orc.attention_cosine(q, k, kept), 1.0, rtol=0, atol=1e-15)


def test_l1_loss_of_constant_magnitude_cache_is_dropped_token_share():
    # every entry has magnitude 1: the dropped share of absolute mass is the dropped share of (head, token) pairs
    r = rng(41)
    k = np.sign(r.standard_normal((3, 40, 8)))
    v = np.sign(r.standard_normal((3, 40, 8)))
    kept = [np.arange(0, 40, 2), np.arange(10), np.arange(40)]          # 20, 10, 40 kept of 40 each
    assert orc.kv_l1_loss(k, v, kept) == pytest.approx(1.0 - 70.0 / 120.0, rel=1e-15)


def test_l1_loss_hand_example():
    # one head, three tokens, d=1: |K| = 1,2,3 and |V| = 4,0,2; dropping token 1 loses 2 of 12
    k = np.array([[[1.0], [-2.0], [3.0]]])
    v = np.array([[[-4.0], [0.0], [2.0]]])
    assert orc.kv_l1_loss(k, v, [np.array([0, 2])]) == pytest.approx(2.0 / 12.0, rel=1e-15)
    assert orc.kv_l1_loss(k, v, [np.array([1])]) == pytest.approx(10.0 / 12.0, rel=1e-15)
    assert orc.kv_l1_loss(k, v, [np.array([], dtype=np.int64)]) == 1.0


def test_attention_cosine_of_identical_keys_is_sqrt_of_kept_share():
    # uniform attention over L tokens against uniform over n kept ones: cos = (n/(L n)) / (1/sqrt(L) 1/sqrt(n))
    r = rng(42)
    L, d = 50, 8
    k = np.broadcast_to(r.standard_normal((2, 1, d)), (2, L, d)).copy()
    q = r.standard_normal((4, d))
    kept = [np.arange(0, 50, 5), np.arange(25)]
    cos = orc.attention_cosine(q, k, kept)
    assert np.allclose(cos[:2], math.sqrt(10 / 50), rtol=1e-13)
    assert np.allclose(cos[2:], math.sqrt(25 / 50), rtol=1e-13)


def test_attention_cosine_hand_example_pins_scale_and_head_map():
    # d=1, scale given: scores of head 0 are s = ln 1, ln 2, ln 3 -> p = (1,2,3)/6; keeping tokens {1,2}:
    # p~ = (0,2,3)/5, cos = 13 / (sqrt(14) sqrt(13)).  Query head 1 reads kv-head 1 (g = 1) whose scores are
    # ln 4, ln 1, ln 1 with token 0 kept alone: cos = 4 / sqrt(18).
    k = np.array([[[math.log(1.0)], [math.log(2.0)], [math.log(3.0)]],
                  [[math.log(4.0)], [0.0], [0.0]]])
    q = np.array([[2.0], [2.0]])
    cos = orc.attention_cosine(q, k, [np.array([1, 2]), np.array([0])], scale=0.5)
    assert cos[0] == pytest.approx(13.0 / math.sqrt(14.0 * 13.0), rel=1e-14)
    assert cos[1] == pytest.approx(4.0 / math.sqrt(18.0), rel=1e-14)
    # grouped heads: two query heads share kv-head 0 and see the same kept set
    cos2 = orc.attention_cosine(np.array([[2.0], [2.0]]), k[:1], [np.array([1, 2])], scale=0.5)
    assert cos2[0] == cos2[1] == cos[0]


def test_attention_cosine_squared_is_kept_share_of_squared_probabilities():
    # p~ is p restricted to the kept set and renormalised, so cos^2 = sum_kept p^2 / sum_all p^2
    r = rng(43)
    Hq, Hkv, L, d = 6, 2, 70, 16
    q, k = r.standard_normal((Hq, d)) * 2, r.standard_normal((Hkv, L, d))
    kept = [np.sort(r.choice(L, 20, replace=False)) for _ in range(Hkv)]
    cos = orc.attention_cosine(q, k, kept)
    for i in range(Hq):
        h = i // 3
        p = softmax((k[h] @ q[i]) / math.sqrt(d))
        assert cos[i] ** 2 == pytest.approx((p[kept[h]] ** 2).sum() / (p ** 2).sum(), rel=1e-12)
    # dropping more tokens never raises the similarity
    fewer = [x[:10] for x in kept]
    assert np.all(orc.attention_cosine(q, k, fewer) <= cos + 1e-15)
