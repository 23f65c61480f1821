"""GPU parity of the stack call with a chunk size per reuse group (the hybrid setting of Section 4.6):
selections against the oracle under the tie-band rule, gathered rows bit-exact, and the per-layer streaming
call with the same table bit for bit equal to the stack call."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import chunkkv_oracle as orc
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = {
    # bf16, 32 window rows x 4 heads: chunk sizes 5, 10, 20 take the single-pass kernel, the others the two-pass one
    "bf16_4k_x7_R2": (W.get_workload("llama8b_32k_stack").with_(seqlens=(4096,), n_spans=(20,), n_layers=7), 2,
                      [10, 1, 5, 3]),
    "bf16_w64_x5_R1": (W.get_workload("llama8b_128k_stack").with_(seqlens=(3000,), n_spans=(9,), n_layers=5, keep_pct=20),
                       1, [20, 20, 1, 7, 10]),
    "ragged_f32_x6_R3": (W.get_workload("tiny").with_(n_layers=6), 3, [1, 4]),
    "ragged_bf16_x4_R2": (W.get_workload("ragged_b8").with_(seqlens=(1500, 640, 2304), n_spans=(7, 3, 11), n_layers=4,
                                                            keep_pct=30), 2, [33, 2]),
}


def _alloc(prob, N, G, dtype):
    B, Hk = prob.batch, prob.n_kv_heads
    sel = (torch.full((G, B, Hk, prob.sel_cap), -7, dtype=torch.int32, device=DEV),
           torch.full((G, B, Hk, prob.sel_cap), -7, dtype=torch.int32, device=DEV),
           torch.full((G, B, Hk), -7, dtype=torch.int32, device=DEV))
    k_out = [torch.zeros(prob.out_elements(), dtype=dtype, device=DEV) for _ in range(N)]
    v_out = [torch.zeros_like(k_out[0]) for _ in range(N)]
    return sel, k_out, v_out


@pytest.mark.parametrize("case", list(CASES))
def test_hybrid_stack_matches_oracle(lib, case):
    wl, R, chunks = CASES[case]
    N, B, Hk = wl.n_layers, wl.batch, wl.n_kv_heads
    G = (N + R - 1) // R
    assert len(chunks) == G
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    # capacities for the smallest chunk size of the table (Problem derives them from `chunk`)
    prob = H.make_problem(lib, wl.with_(chunk=min(chunks)), layers[0])
    sel, k_out, v_out = _alloc(prob, N, G, layers[0].k.dtype)
    n_ws = lib.chunkkv_workspace_bytes_hybrid(prob, N, R, chunks)
    assert n_ws > 0
    ws = torch.empty(n_ws, dtype=torch.uint8, device=DEV)
    qs = [layers[l].q if l % R == 0 else None for l in range(N)]
    print(f"case={case} R={R} chunks={chunks}", flush=True)
    lib.chunkkv_compress_stack_hybrid(prob, R, chunks, qs, [x.k for x in layers], [x.v for x in layers], None,
                                      k_out, v_out, *sel, ws)
    torch.cuda.synchronize()
    n_diff = 0
    for grp in range(G):
        c, leader = chunks[grp], grp * R
        got = H.read_selection(prob, *sel, grp)
        for b in range(B):
            q, k, v = H.seq_arrays(wl, layers[leader], b)
            P, nk = wl.seqlens[b] - wl.window, int(prob.n_keep[b])
            o_scores, _ = orc.score(q, k, wl.window, c)
            for h in range(Hk):
                n_diff += H.check_selection(got[b][h], orc.chunk_topk(o_scores[h], P, c, nk), o_scores[h], P, c, nk)
        for l in range(leader, min(leader + R, N)):
            for b in range(B):
                _, k, v = H.seq_arrays(wl, layers[l], b)
                ok, ov = orc.compact(k, v, [s[0] for s in got[b]], [s[1] for s in got[b]], wl.window, c)
                assert np.array_equal(W.tensor_bits(H.out_view(prob, k_out[l], b)), ok), (l, b)
                assert np.array_equal(W.tensor_bits(H.out_view(prob, v_out[l], b)), ov), (l, b)
    print(f"chunks differing inside the tie band: {n_diff}")

    # the streaming call, given each layer's chunk size, reproduces the stack call bit for bit
    sel2, k2, v2 = _alloc(prob, N, G, layers[0].k.dtype)
    for l in range(N):
        pl = H.make_problem(lib, wl.with_(chunk=chunks[l // R]), layers[0], sel_cap=prob.sel_cap, score_cap=prob.score_cap)
        wsl = torch.empty(lib.chunkkv_workspace_bytes(pl, 1, 1), dtype=torch.uint8, device=DEV)
        lib.chunkkv_compress_layer(pl, l, R, qs[l], None, layers[l].k, layers[l].v, k2[l], v2[l], *sel2, wsl)
    torch.cuda.synchronize()
    cnt = sel[2].cpu().numpy()
    assert np.array_equal(sel2[2].cpu().numpy(), cnt)
    a_c, a_l, b_c, b_l = (t.cpu().numpy() for t in (sel[0], sel[1], sel2[0], sel2[1]))
    for idx in np.ndindex(*cnt.shape):
        m = cnt[idx]
        assert np.array_equal(a_c[idx][:m], b_c[idx][:m]) and np.array_equal(a_l[idx][:m], b_l[idx][:m])
    for l in range(N):
        assert torch.equal(k2[l], k_out[l]) and torch.equal(v2[l], v_out[l]), l


def test_uniform_table_equals_plain_stack_call(lib):
    wl, R = W.get_workload("llama8b_32k_stack").with_(seqlens=(2500,), n_spans=(5,), n_layers=4), 2
    layers = [W.make_layer(wl, l, DEV) for l in range(4)]
    prob = H.make_problem(lib, wl, layers[0])
    qs = [layers[l].q if l % R == 0 else None for l in range(4)]
    outs = []
    for hybrid in (False, True):
        sel, k_out, v_out = _alloc(prob, 4, 2, layers[0].k.dtype)
        ws = torch.empty(lib.chunkkv_workspace_bytes(prob, 4, R), dtype=torch.uint8, device=DEV)
        if hybrid:
            assert lib.chunkkv_workspace_bytes_hybrid(prob, 4, R, [wl.chunk] * 2) == ws.numel()
            lib.chunkkv_compress_stack_hybrid(prob, R, [wl.chunk] * 2, qs, [x.k for x in layers], [x.v for x in layers],
                                              None, k_out, v_out, *sel, ws)
        else:
            lib.chunkkv_compress_stack(prob, R, qs, [x.k for x in layers], [x.v for x in layers], k_out, v_out, *sel, ws)
        torch.cuda.synchronize()
        outs.append((sel, k_out, v_out))
    for a, b in zip(outs[0][1] + outs[0][2], outs[1][1] + outs[1][2]):
        assert torch.equal(a, b)
    assert torch.equal(outs[0][0][2], outs[1][0][2])
