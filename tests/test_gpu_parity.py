"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

Bars: chunk scores / token importance within 1e-3 relative; selections bit-exact on hand-made
scores (ties included) and, when the scores come from the GPU, equal up to chunks inside the
1e-3 tie band around the threshold (count printed); gathered K/V bit-exact for the given indices."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import chunkkv_oracle as orc
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(params=["single_pass", "two_pass"], autouse=True)
def scoring_path(request, lib):
    """Every test runs with the single-pass scoring kernel enabled (used where it applies) and with
    the two-pass kernels forced (CHUNKKV_FLAG_TWO_PASS in every problem the helpers build)."""
    H.DEFAULT_FLAGS = lib.FLAG_TWO_PASS if request.param == "two_pass" else 0
    yield request.param
    H.DEFAULT_FLAGS = 0


def small(name, **kw):
    return W.get_workload(name).with_(**kw)


def alloc_sel(prob, groups=1):
    B, Hk = prob.batch, prob.n_kv_heads
    return (torch.full((groups, B, Hk, prob.sel_cap), -7, dtype=torch.int32, device=DEV),
            torch.full((groups, B, Hk, prob.sel_cap), -7, dtype=torch.int32, device=DEV),
            torch.full((groups, B, Hk), -7, dtype=torch.int32, device=DEV))


def workspace(lib, prob, n_layers=1, reuse=1):
    n = lib.chunkkv_workspace_bytes(prob, n_layers, reuse)
    assert n > 0
    return torch.empty(n, dtype=torch.uint8, device=DEV)


# ------------------------------------------------------------------ scoring
SCORE_CASES = {
    # name: workload (sizes span several 64..256-key tiles, ragged tails, every row-block geometry)
    "tiny_f32": small("tiny"),
    "f32_d128": small("tiny", head_dim=128, seqlens=(300,), window=8, chunk=7),
    "f32_rows160": small("tiny", n_q_heads=10, n_kv_heads=2, window=32, seqlens=(333,), chunk=5),
    "bf16_8k": small("llama8b_8k"),
    "bf16_rows32": small("llama8b_8k", n_q_heads=2, n_kv_heads=2, window=32, seqlens=(1000,), n_spans=(5,)),
    "bf16_rows64_d64": small("llama8b_8k", n_q_heads=4, n_kv_heads=2, head_dim=64, window=32, seqlens=(1531,),
                             chunk=3, n_spans=(5,)),
    "bf16_rows96": small("llama8b_8k", n_q_heads=6, n_kv_heads=2, window=16, seqlens=(777,), chunk=20, n_spans=(5,)),
    "bf16_rows224_g7": small("ragged_b8", seqlens=(2049, 517), n_spans=(10, 2), n_layers=1),
    "bf16_rows256_w64": small("llama8b_128k_stack", seqlens=(4100,), n_spans=(20,), n_layers=1),
    "bf16_rows512": small("llama8b_8k", n_q_heads=16, n_kv_heads=2, window=64, seqlens=(700,), n_spans=(4,)),
    # single-pass kernel geometries: head_dim 64 with 1, 2 and 4 row blocks per wavefront, and chunk sizes
    # whose period against 32-key blocks is 1, 2, 3, 5 and 7 blocks long
    "bf16_d64_rows128_c12": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, head_dim=64, window=32, seqlens=(1531,),
                                  chunk=12, n_spans=(6,)),
    "bf16_d64_rows256_c14": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, head_dim=64, window=64, seqlens=(2100,),
                                  chunk=14, n_spans=(8,)),
    "bf16_d64_rows512_c8": small("llama8b_8k", n_q_heads=16, n_kv_heads=2, head_dim=64, window=64, seqlens=(900,),
                                 chunk=8, n_spans=(4,)),
    "bf16_rows128_c64": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(1300,), chunk=64, n_spans=(5,)),
    "bf16_rows128_c40": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(1111,), chunk=40, n_spans=(5,)),
    "bf16_rows256_c6": small("llama8b_128k_stack", seqlens=(3000,), chunk=6, n_spans=(12,), n_layers=1),
    "bf16_chunk1": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(515,), chunk=1, n_spans=(4,)),
    "bf16_chunk_gt_tile": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(1200,), chunk=300, n_spans=(4,)),
    "bf16_P0": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(32,), n_spans=(0,)),
    "bf16_P_lt_chunk": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(37,), n_spans=(0,)),
    # fp16 caches (the paper's storage type, Eq. 1): the 16-bit kernels with the fp16 matrix instruction
    "f16_8k": small("llama8b_8k", dtype="f16"),
    "f16_rows32": small("llama8b_8k", dtype="f16", n_q_heads=2, n_kv_heads=2, window=32, seqlens=(1000,), n_spans=(5,)),
    "f16_rows224_g7": small("ragged_b8", dtype="f16", seqlens=(2049, 517), n_spans=(10, 2), n_layers=1),
    "f16_rows256_w64": small("llama8b_128k_stack", dtype="f16", seqlens=(4100,), n_spans=(20,), n_layers=1),
    "f16_d64_rows256_c14": small("llama8b_8k", dtype="f16", n_q_heads=8, n_kv_heads=2, head_dim=64, window=64,
                                 seqlens=(2100,), chunk=14, n_spans=(8,)),
    "f16_rows512_c3": small("llama8b_8k", dtype="f16", n_q_heads=16, n_kv_heads=2, window=64, seqlens=(700,), chunk=3,
                            n_spans=(4,)),
}


@pytest.mark.parametrize("case", list(SCORE_CASES))
def test_score_matches_oracle(lib, case, scoring_path):
    wl = SCORE_CASES[case]
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li)
    B, Hk = wl.batch, wl.n_kv_heads
    cs = torch.full((B, Hk, prob.score_cap), -1.0, dtype=torch.float32, device=DEV)
    imp = torch.full((B, Hk, prob.score_cap * wl.chunk), -1.0, dtype=torch.float32, device=DEV)
    ws = workspace(lib, prob)
    print(f"case={case} L={wl.seqlens} rows={wl.group * wl.window}", flush=True)
    lib.chunkkv_score(prob, li.q, li.k, cs, imp, ws)
    torch.cuda.synchronize()
    cs_h, imp_h = cs.cpu().numpy(), imp.cpu().numpy()
    worst = 0.0
    for b in range(B):
        q, k, _ = H.seq_arrays(wl, li, b)
        P = wl.seqlens[b] - wl.window
        o_cs, o_imp = orc.score(q, k, wl.window, wl.chunk)
        C = orc.n_chunks(P, wl.chunk)
        for h in range(Hk):
            worst = max(worst, H.rel_err(imp_h[b, h, :P], o_imp[h]), H.rel_err(cs_h[b, h, :C], o_cs[h]))
            assert np.all(cs_h[b, h, C:] == -1.0) and np.all(imp_h[b, h, P:] == -1.0)  # nothing written past the end
    print(f"max relative error {worst:.3e}")
    assert worst <= H.REL_TOL
    # without the optional importance output: the same kernels in two-pass mode (bit-identical scores);
    # in single-pass mode the other scoring kernel may run, held to the same tolerance
    cs2 = torch.zeros_like(cs)
    lib.chunkkv_score(prob, li.q, li.k, cs2, None, ws)
    torch.cuda.synchronize()
    cs2_h = cs2.cpu().numpy()
    worst2 = 0.0
    for b in range(B):
        q, k, _ = H.seq_arrays(wl, li, b)
        C = orc.n_chunks(wl.seqlens[b] - wl.window, wl.chunk)
        if scoring_path == "two_pass":
            assert torch.equal(cs2[b, :, :C], cs[b, :, :C])
        o_cs, _ = orc.score(q, k, wl.window, wl.chunk)
        for h in range(Hk):
            worst2 = max(worst2, H.rel_err(cs2_h[b, h, :C], o_cs[h]))
    print(f"max relative error without importance output {worst2:.3e}")
    assert worst2 <= H.REL_TOL


def test_score_custom_scale_and_determinism(lib):
    wl = small("llama8b_8k", seqlens=(2000,), n_spans=(8,))
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li, softmax_scale=0.05)
    cs = torch.zeros((1, 8, prob.score_cap), dtype=torch.float32, device=DEV)
    ws = workspace(lib, prob)
    lib.chunkkv_score(prob, li.q, li.k, cs, None, ws)
    first = cs.clone()
    lib.chunkkv_score(prob, li.q, li.k, cs, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(first, cs)                       # fixed-order reductions: bit-identical reruns
    q, k, _ = H.seq_arrays(wl, li, 0)
    o_cs, _ = orc.score(q, k, wl.window, wl.chunk, scale=0.05)
    assert H.rel_err(cs.cpu().numpy()[0], o_cs) <= H.REL_TOL


# ------------------------------------------------------------------ selection
def topk_case(lib, P, c, n_keep_list, scores_rows):
    """scores_rows: [B][Hkv][C] float32.  Compares with the oracle bit-exactly."""
    B, Hk = len(n_keep_list), len(scores_rows[0])
    w = 4
    prob = lib.Problem(Hk, Hk, 64, w, c, lib.F32, [P + w] * B, n_keep_list, [0] * B, (P + w) * 64, 64)
    C = orc.n_chunks(P, c)
    sc = torch.zeros((B, Hk, prob.score_cap), dtype=torch.float32, device=DEV)
    if C:
        sc[:, :, :C] = torch.tensor(np.asarray(scores_rows, dtype=np.float32), device=DEV)
    sel_chunk, sel_len, sel_count = alloc_sel(prob)
    lib.chunkkv_chunk_topk(prob, sc, sel_chunk, sel_len, sel_count)
    torch.cuda.synchronize()
    got = H.read_selection(prob, sel_chunk, sel_len, sel_count)
    for b in range(B):
        for h in range(Hk):
            oc, ol = orc.chunk_topk(np.asarray(scores_rows[b][h], dtype=np.float32).astype(np.float64), P, c, n_keep_list[b])
            gc, gl = got[b][h]
            assert np.array_equal(gc, oc) and np.array_equal(gl, ol), (P, c, n_keep_list[b], b, h)


@pytest.mark.parametrize("seed", range(6))
def test_topk_random_with_ties_bit_exact(lib, seed):
    r = np.random.default_rng(500 + seed)
    P = int(r.integers(1, 5000))
    c = int(r.choice([1, 2, 3, 5, 8, 10, 20, 33]))
    C = orc.n_chunks(P, c)
    B, Hk = 3, 4
    levels = int(r.choice([2, 5, 50, 100000]))
    rows = (r.integers(0, levels, size=(B, Hk, C)) / levels).astype(np.float32)
    if seed % 2:
        rows[:, :, -1] = 1.5          # the ragged tail ranks first
    n_keep = [int(r.integers(0, P + 1)) for _ in range(B)]
    print(f"P={P} c={c} levels={levels} n_keep={n_keep}", flush=True)
    topk_case(lib, P, c, n_keep, rows)


def test_topk_edge_cases(lib):
    topk_case(lib, 23, 10, [13, 10, 14, 0, 23, 1], [[[0.1, 0.5, 0.9]]] * 6)      # ragged tail spill-over
    topk_case(lib, 43, 10, [25, 43, 7], [[[0.5] * 5]] * 3)                         # all equal: leading tokens
    topk_case(lib, 7, 10, [0, 3, 7], [[[0.25]]] * 3)                               # one ragged chunk (c > P)
    topk_case(lib, 40, 1, [0, 17, 40], [[list(np.linspace(0, 1, 40) % 0.3)]] * 3)  # token-level
    topk_case(lib, 3000, 10, [300], [[list(np.zeros(300))]])                       # all-zero scores
    big = np.random.default_rng(3).random(13101).astype(np.float32)                # 128K-token chunk count
    topk_case(lib, 131008, 10, [13100, 26201], [[big]] * 2)


def test_topk_negative_zero_and_tiny_values(lib):
    rows = np.array([[[0.0, -0.0, 1e-38, 0.0, 1e-45, -0.0, 3.0, 0.0]]], dtype=np.float32)
    for nk in range(0, 17):
        topk_case(lib, 16, 2, [nk], rows)


# ------------------------------------------------------------------ gather
def random_selection(r, P, c, n_keep):
    """A valid selection that keeps exactly n_keep tokens (not necessarily what top-k would give)."""
    C = orc.n_chunks(P, c)
    return orc.chunk_topk(r.random(C), P, c, n_keep)


@pytest.mark.parametrize("case", ["tiny_f32", "bf16_8k", "bf16_rows224_g7", "bf16_rows64_d64", "f32_d128",
                                  "bf16_chunk1", "bf16_P0", "bf16_P_lt_chunk"])
def test_compact_bit_exact(lib, case):
    wl = SCORE_CASES[case]
    li = W.make_layer(wl, 0, DEV)
    r = np.random.default_rng(11)
    B, Hk = wl.batch, wl.n_kv_heads
    for variant in ("budget", "all", "none"):
        n_keep = [{"budget": W.keep_budget(L, wl.window, wl.keep_pct), "all": L - wl.window, "none": 0}[variant]
                  for L in wl.seqlens]
        prob = H.make_problem(lib, wl, li, n_keep=n_keep)
        sel_chunk, sel_len, sel_count = alloc_sel(prob)
        sels = [[random_selection(r, L - wl.window, wl.chunk, n_keep[b]) for _ in range(Hk)]
                for b, L in enumerate(wl.seqlens)]
        for b in range(B):
            for h in range(Hk):
                ch, ln = sels[b][h]
                sel_chunk[0, b, h, :len(ch)] = torch.from_numpy(ch).to(DEV)
                sel_len[0, b, h, :len(ln)] = torch.from_numpy(ln).to(DEV)
                sel_count[0, b, h] = len(ch)
        k_out = torch.zeros(prob.out_elements(), dtype=li.k.dtype, device=DEV)
        v_out = torch.zeros_like(k_out)
        print(f"case={case} variant={variant} n_keep={n_keep}", flush=True)
        lib.chunkkv_compact(prob, li.k, li.v, sel_chunk, sel_len, sel_count, k_out, v_out)
        torch.cuda.synchronize()
        for b in range(B):
            _, k, v = H.seq_arrays(wl, li, b)
            ok, ov = orc.compact(k, v, [s[0] for s in sels[b]], [s[1] for s in sels[b]], wl.window, wl.chunk)
            assert np.array_equal(W.tensor_bits(H.out_view(prob, k_out, b)), ok)
            assert np.array_equal(W.tensor_bits(H.out_view(prob, v_out, b)), ov)
        if variant == "all" and wl.layout == "hnd":
            assert torch.equal(k_out.view_as(li.k), li.k) and torch.equal(v_out.view_as(li.v), li.v)


# ------------------------------------------------------------------ whole stack
STACK_CASES = {
    "tiny_f32_x3": (small("tiny", n_layers=3), [1, 2, 3]),
    "bf16_4k_x5": (small("llama8b_32k_stack", seqlens=(4096,), n_spans=(20,), n_layers=5), [1, 2, 4, 7]),
    "ragged_x4": (small("ragged_b8", seqlens=(1500, 640, 2304), n_spans=(7, 3, 11), n_layers=4, chunk=5, keep_pct=30), [1, 3]),
    "w64_20pct_x2": (small("llama8b_128k_stack", seqlens=(3000,), n_spans=(9,), n_layers=2, keep_pct=20), [2]),
    # more sequences and more layers than one launch carries as kernel arguments (16 and 32): the host slices
    "sliced_b19_x35": (small("ragged_b8", seqlens=tuple(90 + 37 * i for i in range(19)), n_spans=(1,) * 19, n_layers=35,
                             keep_pct=20), [1, 2]),
    "f16_4k_x4": (small("llama8b_128k_stack", dtype="f16", seqlens=(4096,), n_spans=(20,), n_layers=4), [1, 2]),
}


@pytest.mark.parametrize("case", list(STACK_CASES))
def test_compress_stack_matches_oracle(lib, case):
    wl, reuses = STACK_CASES[case]
    N, B, Hk = wl.n_layers, wl.batch, wl.n_kv_heads
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0])
    # oracle scores and selections of every layer (each may be a leader for some R)
    o_scores = [[orc.score(*H.seq_arrays(wl, layers[l], b)[:2], wl.window, wl.chunk)[0] for b in range(B)]
                for l in range(N)]
    for R in reuses:
        G = (N + R - 1) // R
        sel_chunk, sel_len, sel_count = alloc_sel(prob, G)
        k_out = [torch.zeros(prob.out_elements(), dtype=layers[0].k.dtype, device=DEV) for _ in range(N)]
        v_out = [torch.zeros_like(k_out[0]) for _ in range(N)]
        ws = workspace(lib, prob, N, R)
        q_list = [layers[l].q if l % R == 0 else None for l in range(N)]
        print(f"case={case} R={R}", flush=True)
        lib.chunkkv_compress_stack(prob, R, q_list, [x.k for x in layers], [x.v for x in layers], k_out, v_out,
                                   sel_chunk, sel_len, sel_count, ws)
        torch.cuda.synchronize()
        n_diff = 0
        for grp in range(G):
            leader = grp * R
            got = H.read_selection(prob, sel_chunk, sel_len, sel_count, grp)
            for b in range(B):
                P, nk = wl.seqlens[b] - wl.window, int(prob.n_keep[b])
                for h in range(Hk):
                    o_sel = orc.chunk_topk(o_scores[leader][b][h], P, wl.chunk, nk)
                    n_diff += H.check_selection(got[b][h], o_sel, o_scores[leader][b][h], P, wl.chunk, nk)
            # gather of every layer of the group, bit-exact for the selection the GPU produced
            for l in range(leader, min(leader + R, N)):
                for b in range(B):
                    _, k, v = H.seq_arrays(wl, layers[l], b)
                    ok, ov = orc.compact(k, v, [s[0] for s in got[b]], [s[1] for s in got[b]], wl.window, wl.chunk)
                    assert np.array_equal(W.tensor_bits(H.out_view(prob, k_out[l], b)), ok), (l, b)
                    assert np.array_equal(W.tensor_bits(H.out_view(prob, v_out[l], b)), ov), (l, b)
        print(f"R={R}: chunks differing inside the tie band: {n_diff}")


def test_stack_keep_everything_is_identity(lib):
    wl = small("llama8b_8k", seqlens=(1111,), n_spans=(3,), n_layers=3, keep_pct=100)
    layers = [W.make_layer(wl, l, DEV) for l in range(3)]
    prob = H.make_problem(lib, wl, layers[0])
    sel_chunk, sel_len, sel_count = alloc_sel(prob, 2)
    k_out = [torch.zeros_like(x.k) for x in layers]
    v_out = [torch.zeros_like(x.v) for x in layers]
    lib.chunkkv_compress_stack(prob, 2, [layers[0].q, None, layers[2].q], [x.k for x in layers], [x.v for x in layers],
                               k_out, v_out, sel_chunk, sel_len, sel_count, workspace(lib, prob, 3, 2))
    torch.cuda.synchronize()
    for l in range(3):
        assert torch.equal(k_out[l], layers[l].k) and torch.equal(v_out[l], layers[l].v)


# ------------------------------------------------------------------ caller-supplied log-sum-exp
def device_lse(wl, li, shift_head=None):
    """The caller's [B][Hq][w] log-sum-exps: the oracle's float64 values of the same stored inputs, rounded to
    fp32 (what the GPU and the oracle's score_from_lse then both take as given)."""
    out = np.zeros((wl.batch, wl.n_q_heads, wl.window), dtype=np.float32)
    for b in range(wl.batch):
        q, k, _ = H.seq_arrays(wl, li, b)
        out[b] = orc.row_log_sum_exp(q, k, wl.window).astype(np.float32)
    if shift_head is not None:
        out[:, shift_head] += np.float32(np.log(2.0))
    return out


LSE_CASES = ["f16_8k", "f16_rows256_w64", "tiny_f32", "f32_rows160", "bf16_8k", "bf16_rows32", "bf16_rows224_g7", "bf16_rows256_w64",
             "bf16_d64_rows256_c14", "bf16_rows512", "bf16_chunk_gt_tile", "bf16_P0", "bf16_P_lt_chunk"]


@pytest.mark.parametrize("case", LSE_CASES)
def test_score_lse_matches_oracle(lib, case):
    wl = SCORE_CASES[case]
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li)
    B, Hk = wl.batch, wl.n_kv_heads
    ws = workspace(lib, prob)
    print(f"case={case} L={wl.seqlens} rows={wl.group * wl.window}", flush=True)
    # the true normalisation, then one query head's raised by ln 2 (the library must take it as given)
    for shift_head in (None, wl.n_q_heads - 1):
        lse = device_lse(wl, li, shift_head)
        cs = torch.full((B, Hk, prob.score_cap), -1.0, dtype=torch.float32, device=DEV)
        imp = torch.full((B, Hk, prob.score_cap * wl.chunk), -1.0, dtype=torch.float32, device=DEV)
        lib.chunkkv_score_lse(prob, li.q, li.k, torch.from_numpy(lse).to(DEV), cs, imp, ws)
        torch.cuda.synchronize()
        cs_h, imp_h = cs.cpu().numpy(), imp.cpu().numpy()
        worst = 0.0
        for b in range(B):
            q, k, _ = H.seq_arrays(wl, li, b)
            P = wl.seqlens[b] - wl.window
            o_cs, o_imp = orc.score_from_lse(q, k, lse[b].astype(np.float64), wl.window, wl.chunk)
            C = orc.n_chunks(P, wl.chunk)
            for h in range(Hk):
                worst = max(worst, H.rel_err(imp_h[b, h, :P], o_imp[h]), H.rel_err(cs_h[b, h, :C], o_cs[h]))
                assert np.all(cs_h[b, h, C:] == -1.0) and np.all(imp_h[b, h, P:] == -1.0)
        print(f"shifted head {shift_head}: max relative error {worst:.3e}")
        assert worst <= H.REL_TOL


@pytest.mark.parametrize("R", [2, 3])
def test_compress_stack_lse_matches_oracle(lib, R):
    wl = small("llama8b_32k_stack", seqlens=(4096,), n_spans=(20,), n_layers=5)
    N, B, Hk = wl.n_layers, wl.batch, wl.n_kv_heads
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0])
    G = (N + R - 1) // R
    sel_chunk, sel_len, sel_count = alloc_sel(prob, G)
    k_out = [torch.zeros(prob.out_elements(), dtype=layers[0].k.dtype, device=DEV) for _ in range(N)]
    v_out = [torch.zeros_like(k_out[0]) for _ in range(N)]
    lses = [device_lse(wl, layers[l]) if l % R == 0 else None for l in range(N)]
    lib.chunkkv_compress_stack_lse(prob, R, [layers[l].q if l % R == 0 else None for l in range(N)],
                                   [x.k for x in layers], [x.v for x in layers],
                                   [None if x is None else torch.from_numpy(x).to(DEV) for x in lses],
                                   k_out, v_out, sel_chunk, sel_len, sel_count, workspace(lib, prob, N, R))
    torch.cuda.synchronize()
    n_diff = 0
    for grp in range(G):
        leader = grp * R
        got = H.read_selection(prob, sel_chunk, sel_len, sel_count, grp)
        for b in range(B):
            q, k, _ = H.seq_arrays(wl, layers[leader], b)
            P, nk = wl.seqlens[b] - wl.window, int(prob.n_keep[b])
            o_cs, _ = orc.score_from_lse(q, k, lses[leader][b].astype(np.float64), wl.window, wl.chunk)
            for h in range(Hk):
                n_diff += H.check_selection(got[b][h], orc.chunk_topk(o_cs[h], P, wl.chunk, nk), o_cs[h], P, wl.chunk, nk)
        for l in range(leader, min(leader + R, N)):
            for b in range(B):
                _, k, v = H.seq_arrays(wl, layers[l], b)
                ok, ov = orc.compact(k, v, [s[0] for s in got[b]], [s[1] for s in got[b]], wl.window, wl.chunk)
                assert np.array_equal(W.tensor_bits(H.out_view(prob, k_out[l], b)), ok), (l, b)
                assert np.array_equal(W.tensor_bits(H.out_view(prob, v_out[l], b)), ov), (l, b)
    print(f"chunks differing inside the tie band: {n_diff}")


# ------------------------------------------------------------------ streaming per-layer call, Jaccard diagnostic
@pytest.mark.parametrize("case,R,with_lse", [("bf16_4k_x5", 2, False), ("bf16_4k_x5", 3, True), ("ragged_x4", 1, False),
                                             ("tiny_f32_x3", 2, False)])
def test_compress_layer_equals_stack_call(lib, case, R, with_lse):
    """One chunkkv_compress_layer call per layer gives bit for bit what chunkkv_compress_stack(_lse) gives
    (which the tests above hold against the oracle)."""
    wl, _ = STACK_CASES[case]
    N = wl.n_layers
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0])
    G = (N + R - 1) // R
    qs = [layers[l].q if l % R == 0 else None for l in range(N)]
    lses = [torch.from_numpy(device_lse(wl, layers[l])).to(DEV) if (with_lse and l % R == 0) else None for l in range(N)]
    ref_sel = alloc_sel(prob, G)
    ref_k = [torch.zeros(prob.out_elements(), dtype=layers[0].k.dtype, device=DEV) for _ in range(N)]
    ref_v = [torch.zeros_like(ref_k[0]) for _ in range(N)]
    if with_lse:
        lib.chunkkv_compress_stack_lse(prob, R, qs, [x.k for x in layers], [x.v for x in layers], lses, ref_k, ref_v,
                                       *ref_sel, workspace(lib, prob, N, R))
    else:
        lib.chunkkv_compress_stack(prob, R, qs, [x.k for x in layers], [x.v for x in layers], ref_k, ref_v,
                                   *ref_sel, workspace(lib, prob, N, R))
    got_sel = alloc_sel(prob, G)
    got_k = [torch.zeros_like(ref_k[0]) for _ in range(N)]
    got_v = [torch.zeros_like(ref_k[0]) for _ in range(N)]
    ws = workspace(lib, prob, 1, 1)
    for l in range(N):
        ws.fill_(0xAB)                      # nothing in the workspace may have to survive between calls
        lib.chunkkv_compress_layer(prob, l, R, qs[l], lses[l], layers[l].k, layers[l].v, got_k[l], got_v[l],
                                   *got_sel, ws)
    torch.cuda.synchronize()
    counts = ref_sel[2].cpu().numpy()
    assert np.array_equal(got_sel[2].cpu().numpy(), counts)
    rc, rl, gc, gl = (t.cpu().numpy() for t in (ref_sel[0], ref_sel[1], got_sel[0], got_sel[1]))
    for idx in np.ndindex(*counts.shape):
        m = counts[idx]
        assert np.array_equal(gc[idx][:m], rc[idx][:m]) and np.array_equal(gl[idx][:m], rl[idx][:m])
    for l in range(N):
        assert torch.equal(got_k[l], ref_k[l]) and torch.equal(got_v[l], ref_v[l]), l


def test_jaccard_matches_oracle(lib):
    wl = small("llama8b_32k_stack", seqlens=(4096, 1500), n_spans=(20, 8), n_layers=6, layout="nhd")
    N, R, B, Hk = wl.n_layers, 1, wl.batch, wl.n_kv_heads
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0])
    sel = alloc_sel(prob, N)
    k_out = [torch.zeros(prob.out_elements(), dtype=layers[0].k.dtype, device=DEV) for _ in range(N)]
    v_out = [torch.zeros_like(k_out[0]) for _ in range(N)]
    lib.chunkkv_compress_stack(prob, R, [x.q for x in layers], [x.k for x in layers], [x.v for x in layers], k_out, v_out,
                               *sel, workspace(lib, prob, N, R))
    jac = torch.full((N - 1, B, Hk), -1.0, dtype=torch.float32, device=DEV)
    lib.chunkkv_jaccard(prob, N, *sel, jac)
    torch.cuda.synchronize()
    jac_h = jac.cpu().numpy()
    got = [H.read_selection(prob, *sel, g) for g in range(N)]
    for g in range(N - 1):
        for b in range(B):
            for h in range(Hk):
                want = orc.jaccard(got[g][b][h], got[g + 1][b][h], wl.chunk)
                assert abs(jac_h[g, b, h] - want) <= 1e-6, (g, b, h, jac_h[g, b, h], want)
    # the planted spans persist from layer to layer with probability 0.8, fresh noise otherwise
    print("mean adjacent-layer Jaccard similarity:", float(jac_h.mean()))
    # hand-made selections: identical, disjoint, partial overlap, both empty
    sc, sl, cnt = alloc_sel(prob, 5)
    def put(g, chunks, lens):
        for b in range(B):
            for h in range(Hk):
                sc[g, b, h, :len(chunks)] = torch.tensor(chunks, dtype=torch.int32)
                sl[g, b, h, :len(lens)] = torch.tensor(lens, dtype=torch.int32)
                cnt[g, b, h] = len(chunks)
    c = wl.chunk
    put(0, [0, 2, 5], [c, c, 2]); put(1, [0, 2, 5], [c, c, 2]); put(2, [1, 3], [c, c]); put(3, [1, 4], [c, 3]); put(4, [], [])
    jac2 = torch.full((4, B, Hk), -1.0, dtype=torch.float32, device=DEV)
    lib.chunkkv_jaccard(prob, 5, sc, sl, cnt, jac2)
    torch.cuda.synchronize()
    j = jac2.cpu().numpy()
    assert np.all(j[0] == 1.0) and np.all(j[1] == 0.0)
    assert np.allclose(j[2], c / (2 * c + c + 3 - c), atol=1e-7) and np.all(j[3] == 0.0)
    put(3, [], [])
    lib.chunkkv_jaccard(prob, 5, sc, sl, cnt, jac2)
    torch.cuda.synchronize()
    assert np.all(jac2.cpu().numpy()[3] == 1.0)


# ------------------------------------------------------------------ graph capture
def test_stack_call_replays_from_a_hip_graph(lib):
    """The stack call issues kernels only (no copies, memsets or allocations), so a caller can capture it;
    every replay, with eager work and synchronisation in between, reproduces the eager result."""
    wl = small("llama8b_32k_stack", seqlens=(4096,), n_spans=(20,), n_layers=4)
    N, R = wl.n_layers, 2
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0])
    G = N // R
    qs = [layers[l].q if l % R == 0 else None for l in range(N)]
    ks, vs = [x.k for x in layers], [x.v for x in layers]
    ws = workspace(lib, prob, N, R)

    def buffers():
        return (alloc_sel(prob, G), [torch.zeros(prob.out_elements(), dtype=ks[0].dtype, device=DEV) for _ in range(N)],
                [torch.zeros(prob.out_elements(), dtype=ks[0].dtype, device=DEV) for _ in range(N)])
    e_sel, e_k, e_v = buffers()
    lib.chunkkv_compress_stack(prob, R, qs, ks, vs, e_k, e_v, *e_sel, ws)
    torch.cuda.synchronize()
    g_sel, g_k, g_v = buffers()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        lib.chunkkv_compress_stack(prob, R, qs, ks, vs, g_k, g_v, *g_sel, ws)   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            lib.chunkkv_compress_stack(prob, R, qs, ks, vs, g_k, g_v, *g_sel, ws)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for t in g_k + g_v:
            t.fill_(1.0)                      # eager work between the replays
        g_sel[2].fill_(-3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g_sel[2], e_sel[2]), rep
        cnt = e_sel[2].cpu().numpy()
        for idx in np.ndindex(*cnt.shape):
            m = int(cnt[idx])
            assert torch.equal(g_sel[0][idx][:m], e_sel[0][idx][:m]) and torch.equal(g_sel[1][idx][:m], e_sel[1][idx][:m])
        for l in range(N):
            assert torch.equal(g_k[l], e_k[l]) and torch.equal(g_v[l], e_v[l]), (rep, l)


# ------------------------------------------------------------------ extreme logit spread
@pytest.mark.parametrize("window", [32, 64])
@pytest.mark.parametrize("kscale", [10.0, 40.0])
def test_scores_under_extreme_logit_spread(lib, scoring_path, kscale, window):
    """Keys scaled by 10 (40): the logits of a row spread over ~80 (~300) nats, the mass sits in a few keys and
    the chunk scores span twenty orders of magnitude.  Both scoring paths keep exponentials and sums in fp32, so
    the plain relative bar holds on every chunk, and a selection that keeps 90 % of the tokens (which reaches
    deep into the chunks that hold almost no mass) stays inside the tie band.  window 32 / 64: 128 / 256 window
    rows per kv-head (one and two row blocks per wavefront in the single-pass kernel)."""
    wl = small("llama8b_8k", n_q_heads=8, n_kv_heads=2, window=window, seqlens=(3000,), n_spans=(6,), keep_pct=90)
    li = W.make_layer(wl, 0, DEV)
    li.k.mul_(kscale)                    # re-rounded to bf16 once; both sides read the same stored bits
    prob = H.make_problem(lib, wl, li)
    cs = torch.zeros((1, wl.n_kv_heads, prob.score_cap), dtype=torch.float32, device=DEV)
    lib.chunkkv_score(prob, li.q, li.k, cs, None, workspace(lib, prob))
    sel = alloc_sel(prob)
    lib.chunkkv_chunk_topk(prob, cs, *sel)
    torch.cuda.synchronize()
    q, k, _ = H.seq_arrays(wl, li, 0)
    o_cs, _ = orc.score(q, k, wl.window, wl.chunk)
    C = o_cs.shape[1]
    got = cs[0, :, :C].cpu().numpy().astype(np.float64)
    rel = np.abs(got - o_cs) / o_cs
    print(f"{scoring_path}: chunk scores span {o_cs.min():.2e} .. {o_cs.max():.2e}; max relative error {rel.max():.2e}")
    assert rel.max() <= H.REL_TOL
    P, n_keep = wl.seqlens[0] - wl.window, int(prob.n_keep[0])
    g_sel = H.read_selection(prob, *sel)
    differ = 0
    for h in range(wl.n_kv_heads):
        differ += H.check_selection(g_sel[0][h], orc.chunk_topk(o_cs[h], P, wl.chunk, n_keep), o_cs[h], P, wl.chunk, n_keep)
    print(f"keep 90 %: {differ} chunks differ, all inside the tie band")


# ------------------------------------------------------------------ seeded sweep of random shapes
def _random_cases(n=24, seed=20250299, force_dtype=None):
    r = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        g = int(r.choice([1, 2, 4, 7, 8]))
        w = int(r.choice([8, 16, 32, 64]))
        if g * w > 512:
            continue
        hkv = int(r.choice([1, 2, 3]))
        d = int(r.choice([64, 128]))
        c = int(r.choice([1, 3, 5, 8, 10, 12, 14, 20, 40, 64, 100]))
        B = int(r.choice([1, 1, 2, 3]))
        lens = tuple(int(w + 1 + r.integers(0, 4000)) for _ in range(B))
        pct = int(r.choice([5, 10, 20, 35, 100]))
        dtype = "f32" if (r.random() < 0.15 and d == 64) else "bf16"
        dtype = force_dtype or dtype
        cases.append(dict(n_q_heads=g * hkv, n_kv_heads=hkv, head_dim=d, window=w, chunk=c, seqlens=lens,
                          n_spans=tuple(max(1, L // 300) for L in lens), keep_pct=pct, dtype=dtype, n_layers=2,
                          layout="nhd" if B > 1 else str(r.choice(["hnd", "nhd"]))))
    return cases


@pytest.mark.parametrize("idx", range(24 + 10))
def test_random_shapes_match_oracle(lib, idx):
    """Scores, selection and gather of 24 seeded random geometries (row counts 8..512, both head dims, chunk
    sizes with and without a short period, ragged batches, both layouts) against the oracle, and of 10 more
    with fp16 caches."""
    kw = _random_cases()[idx] if idx < 24 else _random_cases(10, 20250300, "f16")[idx - 24]
    wl = W.get_workload("llama8b_8k").with_(**kw)
    N, R, B, Hk = 2, 2, wl.batch, wl.n_kv_heads
    print(f"case {idx}: {kw}", flush=True)
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0])
    cs = torch.full((B, Hk, prob.score_cap), -1.0, dtype=torch.float32, device=DEV)
    lib.chunkkv_score(prob, layers[0].q, layers[0].k, cs, None, workspace(lib, prob))
    sel = alloc_sel(prob, 1)
    k_out = [torch.zeros(prob.out_elements(), dtype=layers[0].k.dtype, device=DEV) for _ in range(N)]
    v_out = [torch.zeros_like(k_out[0]) for _ in range(N)]
    lib.chunkkv_compress_stack(prob, R, [layers[0].q, None], [x.k for x in layers], [x.v for x in layers], k_out, v_out,
                               *sel, workspace(lib, prob, N, R))
    torch.cuda.synchronize()
    cs_h = cs.cpu().numpy()
    got = H.read_selection(prob, *sel, 0)
    worst = 0.0
    for b in range(B):
        q, k, _ = H.seq_arrays(wl, layers[0], b)
        P, nk = wl.seqlens[b] - wl.window, int(prob.n_keep[b])
        o_cs, _ = orc.score(q, k, wl.window, wl.chunk)
        C = orc.n_chunks(P, wl.chunk)
        for h in range(Hk):
            worst = max(worst, H.rel_err(cs_h[b, h, :C], o_cs[h]))
            H.check_selection(got[b][h], orc.chunk_topk(o_cs[h], P, wl.chunk, nk), o_cs[h], P, wl.chunk, nk)
        for l in range(N):
            _, kl, vl = H.seq_arrays(wl, layers[l], b)
            ok, ov = orc.compact(kl, vl, [s[0] for s in got[b]], [s[1] for s in got[b]], wl.window, wl.chunk)
            assert np.array_equal(W.tensor_bits(H.out_view(prob, k_out[l], b)), ok), (l, b)
            assert np.array_equal(W.tensor_bits(H.out_view(prob, v_out[l], b)), ov), (l, b)
    assert worst <= H.REL_TOL, worst


# ------------------------------------------------------------------ whole-chunk selection mode (Algorithm 3 as printed)
@pytest.fixture
def whole_chunks(lib, scoring_path):
    """CHUNKKV_FLAG_WHOLE_CHUNKS in every problem the helpers build (beside the scoring-path flag)."""
    before = H.DEFAULT_FLAGS
    H.DEFAULT_FLAGS = before | lib.FLAG_WHOLE_CHUNKS
    yield
    H.DEFAULT_FLAGS = before


@pytest.mark.parametrize("case", ["bf16_8k", "bf16_rows96", "bf16_P_lt_chunk", "tiny_f32"])
def test_whole_chunk_topk_matches_oracle(lib, whole_chunks, case):
    wl = SCORE_CASES[case]
    li = W.make_layer(wl, 0, DEV)
    r = np.random.default_rng(5)
    B, Hk = wl.batch, wl.n_kv_heads
    for trial in range(3):
        # hand-made scores with many exact ties (both sides decide on the same fp32 values); the last trial
        # makes the ragged tail chunk the best one
        n_keep = [int(r.integers(0, L - wl.window + 1)) for L in wl.seqlens]
        prob = H.make_problem(lib, wl, li, n_keep=n_keep)
        scores = torch.zeros((B, Hk, prob.score_cap), dtype=torch.float32, device=DEV)
        host = []
        for b, L in enumerate(wl.seqlens):
            C = orc.n_chunks(L - wl.window, wl.chunk)
            s = r.integers(1, 6, (Hk, C)).astype(np.float32)
            if trial == 2 and C:
                s[:, -1] = 9.0
            host.append(s)
            scores[b, :, :C] = torch.from_numpy(s).to(DEV)
        sel = alloc_sel(prob)
        lib.chunkkv_chunk_topk(prob, scores, *sel)
        torch.cuda.synchronize()
        got = H.read_selection(prob, *sel, 0)
        for b, L in enumerate(wl.seqlens):
            for h in range(Hk):
                oc, ol = orc.chunk_topk_whole(host[b][h].astype(np.float64), L - wl.window, wl.chunk, n_keep[b])
                assert got[b][h][0].tolist() == oc.tolist() and got[b][h][1].tolist() == ol.tolist(), (trial, b, h)


def test_whole_chunk_stack_matches_oracle(lib, whole_chunks):
    wl = small("llama8b_32k_stack", seqlens=(4093,), n_spans=(20,), n_layers=3)   # P = 4061: ragged tail of 1
    N, R, Hk = wl.n_layers, 2, wl.n_kv_heads
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0], n_keep=[407])                        # 40 whole chunks, 7 tokens unused
    sel = alloc_sel(prob, 2)
    k_out = [torch.full((prob.out_elements(),), 7.0, dtype=layers[0].k.dtype, device=DEV) for _ in range(N)]
    v_out = [torch.full((prob.out_elements(),), 7.0, dtype=layers[0].k.dtype, device=DEV) for _ in range(N)]
    lib.chunkkv_compress_stack(prob, R, [layers[0].q, None, layers[2].q], [x.k for x in layers], [x.v for x in layers],
                               k_out, v_out, *sel, workspace(lib, prob, N, R))
    torch.cuda.synchronize()
    P, c, w = wl.seqlens[0] - wl.window, wl.chunk, wl.window
    for grp in range(2):
        got = H.read_selection(prob, *sel, grp)[0]
        q, k, _ = H.seq_arrays(wl, layers[grp * R], 0)
        o_cs, _ = orc.score(q, k, w, c)
        for h in range(Hk):
            oc, ol = orc.chunk_topk_whole(o_cs[h], P, c, 407)
            gc, gl = got[h]
            assert len(gc) == 40 and np.all(gl == np.minimum(c, P - gc.astype(np.int64) * c))
            thr = o_cs[h][oc].min()
            for ch in set(gc.tolist()) ^ set(oc.tolist()):
                assert abs(o_cs[h][ch] - thr) <= H.REL_TOL * thr
        for l in range(grp * R, min(grp * R + R, N)):
            _, kl, vl = H.seq_arrays(wl, layers[l], 0)
            ko, vo = W.tensor_bits(H.out_view(prob, k_out[l], 0)), W.tensor_bits(H.out_view(prob, v_out[l], 0))
            for h in range(Hk):
                idx = orc.kept_token_indices(got[h][0], got[h][1], wl.seqlens[0], w, c)   # kept tokens, then the window
                assert len(idx) == int(got[h][1].sum()) + w
                assert np.array_equal(ko[h][:len(idx)], kl[h][idx]) and np.array_equal(vo[h][:len(idx)], vl[h][idx])
                # rows past kept + w are untouched (still the fill value 7.0 = 0x40E0 in bf16)
                assert np.all(ko[h][len(idx):] == 0x40E0) and np.all(vo[h][len(idx):] == 0x40E0)
