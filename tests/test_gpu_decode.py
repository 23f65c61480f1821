"""GPU parity of chunkkv_decode_attention (one query token per head over the compressed or the full cache)
against the CPU oracle, through the C ABI.

Bar: every output element within 1e-3 of the oracle relative to the largest magnitude of its head's output
row (products and sums are fp32 on the GPU, float64 in the oracle; about 1e-6 is what the arithmetic gives),
log-sum-exps within 1e-4 absolute."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import chunkkv_oracle as orc
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
OUT_TOL = 1e-3
LSE_TOL = 1e-4


def small(name, **kw):
    return W.get_workload(name).with_(**kw)


def alloc_sel(prob, groups=1):
    B, Hk = prob.batch, prob.n_kv_heads
    return (torch.full((groups, B, Hk, prob.sel_cap), -7, dtype=torch.int32, device=DEV),
            torch.full((groups, B, Hk, prob.sel_cap), -7, dtype=torch.int32, device=DEV),
            torch.full((groups, B, Hk), -7, dtype=torch.int32, device=DEV))


def decode_query(li):
    """The new token's query: the last window row of every head, [B][Hq][d] contiguous."""
    return li.q[:, :, -1, :].contiguous()


def check_decode(out, lse, q_bits, k_bits, v_bits, scale=None, n=None):
    """out [Hq][d], lse [Hq] of one sequence against the oracle on the first n tokens of every kv-head
    (n: int or per-kv-head list)."""
    Hq, Hkv = q_bits.shape[0], k_bits.shape[0]
    g = Hq // Hkv
    worst = 0.0
    for h in range(Hkv):
        nh = k_bits.shape[1] if n is None else (n if np.isscalar(n) else int(n[h]))
        qs = q_bits[h * g:(h + 1) * g]
        if nh == 0:
            assert np.all(out[h * g:(h + 1) * g] == 0.0) and np.all(np.isneginf(lse[h * g:(h + 1) * g]))
            continue
        o_ref, l_ref = orc.decode_attention(qs, k_bits[h:h + 1, :nh], v_bits[h:h + 1, :nh], scale)
        for j in range(g):
            err = np.max(np.abs(out[h * g + j] - o_ref[j])) / np.max(np.abs(o_ref[j]))
            worst = max(worst, float(err))
            assert abs(float(lse[h * g + j]) - l_ref[j]) <= LSE_TOL, (h, j, lse[h * g + j], l_ref[j])
    assert worst <= OUT_TOL, worst
    return worst


DECODE_CASES = {
    # name: workload; lengths cross the 64-row step of a workgroup, one key range and several
    "bf16_g4_n1": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(1,), window=1, n_spans=(0,)),
    "bf16_g4_n63": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(63,), n_spans=(1,)),
    "bf16_g4_n65": small("llama8b_8k", n_q_heads=8, n_kv_heads=2, seqlens=(65,), n_spans=(1,)),
    "bf16_g4_8k": small("llama8b_8k"),
    "bf16_g1": small("llama8b_8k", n_q_heads=2, n_kv_heads=2, seqlens=(1000,), n_spans=(5,)),
    "bf16_g2_d64": small("llama8b_8k", n_q_heads=4, n_kv_heads=2, head_dim=64, seqlens=(1531,), n_spans=(5,)),
    "bf16_g7_ragged": small("ragged_b8", seqlens=(2049, 517, 33), n_spans=(10, 2, 0), n_layers=1),
    "bf16_g8_d64": small("llama8b_8k", n_q_heads=16, n_kv_heads=2, head_dim=64, seqlens=(3000,), n_spans=(5,)),
    "bf16_g5": small("llama8b_8k", n_q_heads=10, n_kv_heads=2, seqlens=(1777,), n_spans=(5,)),
    "f16_g6": small("llama8b_8k", dtype="f16", n_q_heads=12, n_kv_heads=2, seqlens=(2222,), n_spans=(5,)),
    "bf16_g16": small("llama8b_8k", n_q_heads=32, n_kv_heads=2, window=16, seqlens=(700,), n_spans=(4,)),
    "bf16_g3_nhd": small("llama8b_8k", n_q_heads=6, n_kv_heads=2, seqlens=(4100,), n_spans=(9,), layout="nhd"),
    "bf16_b19_sliced": small("ragged_b8", seqlens=tuple(40 + 53 * i for i in range(19)), n_spans=(1,) * 19, n_layers=1),
    "f16_g4": small("llama8b_8k", dtype="f16", seqlens=(5000,), n_spans=(20,)),
    "f16_g8_d64": small("llama8b_8k", dtype="f16", n_q_heads=16, n_kv_heads=2, head_dim=64, seqlens=(1300,), n_spans=(5,)),
    "f32_tiny": small("tiny"),
    "f32_d128_g5": small("tiny", head_dim=128, n_q_heads=10, n_kv_heads=2, seqlens=(777,), window=8),
    "f32_d64_g8": small("tiny", n_q_heads=16, n_kv_heads=2, seqlens=(2500,), window=8),
}


@pytest.mark.parametrize("case", list(DECODE_CASES))
def test_decode_over_full_cache_matches_oracle(lib, case):
    wl = DECODE_CASES[case]
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li)
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    q = decode_query(li)
    out = torch.full((B, Hq, d), 7.0, dtype=torch.float32, device=DEV)
    lse = torch.full((B, Hq), 7.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.chunkkv_decode_workspace_bytes(prob, False), dtype=torch.uint8, device=DEV)
    print(f"case={case} L={wl.seqlens} g={wl.group}", flush=True)
    lib.chunkkv_decode_attention(prob, False, None, q, li.k, li.v, out, lse, ws)
    torch.cuda.synchronize()
    out_h, lse_h = out.cpu().numpy(), lse.cpu().numpy()
    worst = 0.0
    for b in range(B):
        _, k, v = H.seq_arrays(wl, li, b)
        worst = max(worst, check_decode(out_h[b], lse_h[b], W.tensor_bits(q[b]), k, v))
    print(f"max error relative to the head's output scale {worst:.3e}")
    # without the optional lse output, and twice: bit-identical (fixed merge order)
    out2 = torch.zeros_like(out)
    lib.chunkkv_decode_attention(prob, False, None, q, li.k, li.v, out2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_decode_custom_scale(lib):
    wl = small("llama8b_8k", seqlens=(2000,), n_spans=(8,))
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li, softmax_scale=0.05)
    q = decode_query(li)
    out = torch.zeros((1, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=DEV)
    lse = torch.zeros((1, wl.n_q_heads), dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.chunkkv_decode_workspace_bytes(prob, False), dtype=torch.uint8, device=DEV)
    lib.chunkkv_decode_attention(prob, False, None, q, li.k, li.v, out, lse, ws)
    torch.cuda.synchronize()
    _, k, v = H.seq_arrays(wl, li, 0)
    check_decode(out.cpu().numpy()[0], lse.cpu().numpy()[0], W.tensor_bits(q[0]), k, v, scale=0.05)


def test_decode_token_counts_from_the_device(lib):
    """kv_len overrides the token count per (sequence, kv-head): shorter prefixes, zero tokens, and counts
    beyond the cache (clamped to it)."""
    wl = small("ragged_b8", seqlens=(1500, 640), n_spans=(7, 3), n_layers=1)
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li)
    B, Hk, Hq, d = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    lens = np.array([[1500, 1, 0, 777], [64, 100000, 639, 65]], dtype=np.int32)
    q = decode_query(li)
    out = torch.full((B, Hq, d), 7.0, dtype=torch.float32, device=DEV)
    lse = torch.full((B, Hq), 7.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.chunkkv_decode_workspace_bytes(prob, False), dtype=torch.uint8, device=DEV)
    lib.chunkkv_decode_attention(prob, False, torch.from_numpy(lens).to(DEV), q, li.k, li.v, out, lse, ws)
    torch.cuda.synchronize()
    for b in range(B):
        _, k, v = H.seq_arrays(wl, li, b)
        n = np.minimum(lens[b], wl.seqlens[b])
        check_decode(out.cpu().numpy()[b], lse.cpu().numpy()[b], W.tensor_bits(q[b]), k, v, n=n)


@pytest.mark.parametrize("case,whole", [("bf16_g4_8k", False), ("bf16_g7_ragged", False), ("f16_g4", False),
                                        ("f32_tiny", False), ("bf16_g4_8k", True), ("bf16_g7_ragged", True)])
def test_decode_over_the_compressed_cache(lib, case, whole):
    """Compress one layer on the GPU, then decode over K', V' as they lie in the output buffers.  The
    expected value is the oracle's attention over the oracle's gather for the GPU's selection (the gather is
    bit-exact, so both sides read the same rows).  In whole-chunk mode the kept count varies per head and
    travels as kv_len."""
    wl = DECODE_CASES[case]
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li, flags=lib.FLAG_WHOLE_CHUNKS if whole else 0)
    B, Hk, Hq, d, w, c = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim, wl.window, wl.chunk
    sel = alloc_sel(prob)
    k_out = torch.zeros(prob.out_elements(), dtype=li.k.dtype, device=DEV)
    v_out = torch.zeros_like(k_out)
    lib.chunkkv_compress_stack(prob, 1, [li.q], [li.k], [li.v], [k_out], [v_out], *sel,
                               torch.empty(lib.chunkkv_workspace_bytes(prob, 1, 1), dtype=torch.uint8, device=DEV))
    torch.cuda.synchronize()
    got = H.read_selection(prob, *sel, 0)
    kv_len = None
    if whole:
        kv_len = torch.tensor([[int(got[b][h][1].sum()) + w for h in range(Hk)] for b in range(B)], dtype=torch.int32, device=DEV)
    q = decode_query(li)
    out = torch.full((B, Hq, d), 7.0, dtype=torch.float32, device=DEV)
    lse = torch.full((B, Hq), 7.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.chunkkv_decode_workspace_bytes(prob, True), dtype=torch.uint8, device=DEV)
    lib.chunkkv_decode_attention(prob, True, kv_len, q, k_out, v_out, out, lse, ws)
    torch.cuda.synchronize()
    out_h, lse_h = out.cpu().numpy(), lse.cpu().numpy()
    g = Hq // Hk
    for b in range(B):
        _, k, v = H.seq_arrays(wl, li, b)
        L = wl.seqlens[b]
        qb = W.tensor_bits(q[b])
        for h in range(Hk):
            idx = orc.kept_token_indices(got[b][h][0], got[b][h][1], L, w, c)
            check_decode(out_h[b, h * g:(h + 1) * g], lse_h[b, h * g:(h + 1) * g], qb[h * g:(h + 1) * g],
                         k[h:h + 1, idx], v[h:h + 1, idx])


def test_decode_128k_full_and_compressed_sampled_heads(lib):
    """The benchmark's shape: one layer of the 128K workload, decode over the full cache and over the
    10 % cache; three query heads of each checked against the oracle."""
    wl = W.get_workload("llama8b_128k_stack").with_(n_layers=1)
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li)
    Hq, Hk, d, w, c = wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk
    g = Hq // Hk
    q = decode_query(li)
    out = torch.zeros((1, Hq, d), dtype=torch.float32, device=DEV)
    lse = torch.zeros((1, Hq), dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.chunkkv_decode_workspace_bytes(prob, False), dtype=torch.uint8, device=DEV)
    lib.chunkkv_decode_attention(prob, False, None, q, li.k, li.v, out, lse, ws)
    sel = alloc_sel(prob)
    k_out = torch.zeros(prob.out_elements(), dtype=li.k.dtype, device=DEV)
    v_out = torch.zeros_like(k_out)
    lib.chunkkv_compress_stack(prob, 1, [li.q], [li.k], [li.v], [k_out], [v_out], *sel,
                               torch.empty(lib.chunkkv_workspace_bytes(prob, 1, 1), dtype=torch.uint8, device=DEV))
    out_c, lse_c = torch.zeros_like(out), torch.zeros_like(lse)
    ws_c = torch.empty(lib.chunkkv_decode_workspace_bytes(prob, True), dtype=torch.uint8, device=DEV)
    lib.chunkkv_decode_attention(prob, True, None, q, k_out, v_out, out_c, lse_c, ws_c)
    torch.cuda.synchronize()
    got = H.read_selection(prob, *sel, 0)
    _, k, v = H.seq_arrays(wl, li, 0)
    qb = W.tensor_bits(q[0])
    for head in (0, 13, 31):
        h = head // g
        check_decode(out.cpu().numpy()[0, head:head + 1], lse.cpu().numpy()[0, head:head + 1], qb[head:head + 1],
                     k[h:h + 1], v[h:h + 1])
        idx = orc.kept_token_indices(got[0][h][0], got[0][h][1], wl.seqlens[0], w, c)
        check_decode(out_c.cpu().numpy()[0, head:head + 1], lse_c.cpu().numpy()[0, head:head + 1], qb[head:head + 1],
                     k[h:h + 1, idx], v[h:h + 1, idx])


def test_decode_call_replays_from_a_hip_graph(lib):
    """A decoding loop captures the call once and replays it with new queries in the same buffers: kernels
    only, no copies, memsets or allocations.  Every replay, with eager work in between, equals the eager call."""
    wl = small("llama8b_8k", seqlens=(6000,), n_spans=(20,))
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li)
    Hq, d = wl.n_q_heads, wl.head_dim
    ws = torch.empty(lib.chunkkv_decode_workspace_bytes(prob, False), dtype=torch.uint8, device=DEV)
    q_buf = decode_query(li).clone()
    out_g = torch.zeros((1, Hq, d), dtype=torch.float32, device=DEV)
    lse_g = torch.zeros((1, Hq), dtype=torch.float32, device=DEV)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        lib.chunkkv_decode_attention(prob, False, None, q_buf, li.k, li.v, out_g, lse_g, ws)   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            lib.chunkkv_decode_attention(prob, False, None, q_buf, li.k, li.v, out_g, lse_g, ws)
    torch.cuda.current_stream().wait_stream(side)
    ws_e = torch.empty_like(ws)
    for rep in range(3):
        q_new = li.q[:, :, rep, :].contiguous()          # another window row as the "next token"
        q_buf.copy_(q_new)
        out_g.fill_(3.0)
        lse_g.fill_(3.0)
        ws.fill_(0xA5)                                    # the workspace is scratch: its contents never matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        out_e = torch.zeros_like(out_g)
        lse_e = torch.zeros_like(lse_g)
        lib.chunkkv_decode_attention(prob, False, None, q_new, li.k, li.v, out_e, lse_e, ws_e)
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e) and torch.equal(lse_g, lse_e), rep
    _, k, v = H.seq_arrays(wl, li, 0)
    check_decode(out_g.cpu().numpy()[0], lse_g.cpu().numpy()[0], W.tensor_bits(q_buf[0]), k, v)
