"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(one chunkkv_compress_stack call over the whole stack).

The oracle cannot redo a 32-layer 128K cache in seconds, so:
  * selections are compared with the oracle on sampled (group, sequence, kv-head) problems (tie-band rule);
  * structural properties are checked for EVERY (group, sequence, kv-head): exact budget, ascending
    chunks, valid lengths, at most one cut chunk;
  * the gather is checked for EVERY layer and head against torch.index_select with the indices
    the GPU's own selection names (a library gather, independent of the HIP kernels), bit-exact;
  * chunk scores of sampled heads are compared with the oracle at full length (chunkkv_score).
"""
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


def run_stack(lib, wl, R, layers=None):
    N, B, Hk = wl.n_layers, wl.batch, wl.n_kv_heads
    layers = layers or [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0])
    G = (N + R - 1) // R
    sel_chunk = torch.zeros((G, B, Hk, prob.sel_cap), dtype=torch.int32, device=DEV)
    sel_len = torch.zeros_like(sel_chunk)
    sel_count = torch.zeros((G, B, Hk), dtype=torch.int32, device=DEV)
    k_out = [torch.zeros(prob.out_elements(), dtype=wl.torch_dtype, device=DEV) for _ in range(N)]
    v_out = [torch.zeros(prob.out_elements(), dtype=wl.torch_dtype, device=DEV) for _ in range(N)]
    ws = torch.empty(lib.chunkkv_workspace_bytes(prob, N, R), dtype=torch.uint8, device=DEV)
    qs = [layers[l].q if l % R == 0 else None for l in range(N)]
    lib.chunkkv_compress_stack(prob, R, qs, [x.k for x in layers], [x.v for x in layers], k_out, v_out,
                               sel_chunk, sel_len, sel_count, ws)
    torch.cuda.synchronize()
    return layers, prob, (sel_chunk, sel_len, sel_count), k_out, v_out


def check_structure_everywhere(wl, prob, sel, R):
    sel_chunk, sel_len, sel_count = (t.cpu().numpy() for t in sel)
    G = sel_chunk.shape[0]
    c = wl.chunk
    for g in range(G):
        for b in range(wl.batch):
            P, nk = wl.seqlens[b] - wl.window, int(prob.n_keep[b])
            for h in range(wl.n_kv_heads):
                m = int(sel_count[g, b, h])
                ch, ln = sel_chunk[g, b, h, :m].astype(np.int64), sel_len[g, b, h, :m].astype(np.int64)
                assert int(ln.sum()) == nk
                assert np.all(np.diff(ch) > 0) and (m == 0 or (ch[0] >= 0 and ch[-1] * c < P))
                natural = np.minimum(c, P - ch * c)
                assert np.all((ln >= 1) & (ln <= natural)) and int(np.sum(ln < natural)) <= 1


def check_gather_everywhere(wl, layers, prob, sel, k_out, v_out, R):
    """Every layer and head: output == index_select(input, tokens named by the GPU selection)."""
    sel_chunk, sel_len, sel_count = sel
    c, w = wl.chunk, wl.window
    for l in range(wl.n_layers):
        g = l // R
        for b in range(wl.batch):
            L = wl.seqlens[b]
            P = L - w
            kin = layers[l].seq_view(layers[l].k, b, wl.n_kv_heads, wl.head_dim)
            vin = layers[l].seq_view(layers[l].v, b, wl.n_kv_heads, wl.head_dim)
            ko, vo = H.out_view(prob, k_out[l], b), H.out_view(prob, v_out[l], b)
            for h in range(wl.n_kv_heads):
                m = int(sel_count[g, b, h])
                ch = sel_chunk[g, b, h, :m].long()
                ln = sel_len[g, b, h, :m].long()
                starts = torch.repeat_interleave(ch * c, ln)
                within = torch.arange(int(ln.sum()), device=DEV) - torch.repeat_interleave(torch.cumsum(ln, 0) - ln, ln)
                idx = torch.cat([starts + within, torch.arange(P, L, device=DEV)])
                # Gaussian inputs hold no NaN, so value equality of the stored type is bit equality
                assert torch.equal(ko[h], kin[h].index_select(0, idx)), (l, b, h)
                assert torch.equal(vo[h], vin[h].index_select(0, idx)), (l, b, h)


def check_sampled_selections(lib, wl, layers, prob, sel, R, samples):
    n_diff = 0
    for (g, b, h) in samples:
        leader = g * R
        li = layers[leader]
        q = W.tensor_bits(li.q[b, h * wl.group:(h + 1) * wl.group])                  # [g][w][d]
        k = W.tensor_bits(li.seq_view(li.k, b, wl.n_kv_heads, wl.head_dim)[h:h + 1])  # [1][L][d]
        P, nk = wl.seqlens[b] - wl.window, int(prob.n_keep[b])
        o_cs, _ = orc.score(q, k, wl.window, wl.chunk)
        o_sel = orc.chunk_topk(o_cs[0], P, wl.chunk, nk)
        got = H.read_selection(prob, *sel, g)[b][h]
        d = H.check_selection(got, o_sel, o_cs[0], P, wl.chunk, nk)
        print(f"group {g} seq {b} head {h}: {d} chunks differ inside the tie band", flush=True)
        n_diff += d
    return n_diff


def test_stack_128k_32_layers_reuse2(lib):
    wl = W.get_workload("llama8b_128k_stack")
    print("workload", wl.name, "R=2", flush=True)
    layers, prob, sel, k_out, v_out = run_stack(lib, wl, 2)
    check_structure_everywhere(wl, prob, sel, 2)
    check_gather_everywhere(wl, layers, prob, sel, k_out, v_out, 2)
    # 16 of the 128 (group, kv-head) selections against the oracle: every group once, every head twice
    check_sampled_selections(lib, wl, layers, prob, sel, 2, [(g, 0, (3 * g + g // 8) % 8) for g in range(16)])
    # chunk scores of two heads of one leader layer at full length
    li = layers[14]
    cs = torch.zeros((1, wl.n_kv_heads, prob.score_cap), dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.chunkkv_workspace_bytes(prob), dtype=torch.uint8, device=DEV)
    lib.chunkkv_score(prob, li.q, li.k, cs, None, ws)
    torch.cuda.synchronize()
    for h in (1, 6):
        q = W.tensor_bits(li.q[0, h * wl.group:(h + 1) * wl.group])
        k = W.tensor_bits(li.k[0, h:h + 1])
        o_cs, _ = orc.score(q, k, wl.window, wl.chunk)
        err = H.rel_err(cs[0, h, :o_cs.shape[1]].cpu().numpy(), o_cs[0])
        print(f"head {h}: max relative score error {err:.3e}", flush=True)
        assert err <= H.REL_TOL


@pytest.mark.parametrize("R", [1, 2])
def test_stack_32k_32_layers(lib, R):
    wl = W.get_workload("llama8b_32k_stack")
    print("workload", wl.name, "R=", R, flush=True)
    layers, prob, sel, k_out, v_out = run_stack(lib, wl, R)
    check_structure_everywhere(wl, prob, sel, R)
    check_gather_everywhere(wl, layers, prob, sel, k_out, v_out, R)
    G = (wl.n_layers + R - 1) // R
    check_sampled_selections(lib, wl, layers, prob, sel, R, [(0, 0, 3), (G // 2, 0, 0), (G - 1, 0, 7)])


def test_stack_128k_keep20(lib, scoring_path):
    """The long-context configuration at its second budget: all 32 layers, keep 20 %, R = 2."""
    if scoring_path == "two_pass":
        pytest.skip("the budget only changes selection and gather; one scoring path is enough at this size")
    wl = W.get_workload("llama8b_128k_stack").with_(keep_pct=20)
    print("workload", wl.name, "20% 32 layers R=2", flush=True)
    layers, prob, sel, k_out, v_out = run_stack(lib, wl, 2)
    check_structure_everywhere(wl, prob, sel, 2)
    check_gather_everywhere(wl, layers, prob, sel, k_out, v_out, 2)
    check_sampled_selections(lib, wl, layers, prob, sel, 2, [(0, 0, 6), (5, 0, 2), (10, 0, 4), (15, 0, 1)])


_ragged_layers = {}


def ragged_layers(n_layers):
    """The first layers of the ragged workload, generated once per session (chunk size, budget and reuse depth
    do not enter the inputs)."""
    if n_layers not in _ragged_layers:
        wl = W.get_workload("ragged_b8").with_(n_layers=n_layers)
        _ragged_layers[n_layers] = [W.make_layer(wl, l, DEV) for l in range(n_layers)]
    return _ragged_layers[n_layers]


@pytest.mark.parametrize("R", [1, 2, 3])
@pytest.mark.parametrize("pct", [10, 20, 30])
@pytest.mark.parametrize("chunk", [5, 10, 20])
def test_ragged_batch_sweep(lib, chunk, pct, R, scoring_path):
    if scoring_path == "two_pass" and R != 2:
        pytest.skip("the two-pass kernels run the R = 2 third of the sweep")
    # batch of 8 ragged sequences (4096..65536 tokens), 28 q / 4 kv heads, packed [sum L][Hkv][d]: all 27
    # (chunk size, budget, reuse depth) combinations of the sweep; 6 of the 28 layers keep a run short, the
    # launch shapes per layer are those of the full stack
    wl = W.get_workload("ragged_b8").with_(chunk=chunk, keep_pct=pct, n_layers=6)
    print("workload", wl.name, f"c={chunk} keep={pct}% R={R} L={wl.seqlens}", flush=True)
    layers, prob, sel, k_out, v_out = run_stack(lib, wl, R, ragged_layers(6))
    check_structure_everywhere(wl, prob, sel, R)
    check_gather_everywhere(wl, layers, prob, sel, k_out, v_out, R)
    short = int(np.argmin(wl.seqlens))
    G = (wl.n_layers + R - 1) // R
    check_sampled_selections(lib, wl, layers, prob, sel, R, [(0, short, 1), (G - 1, (short + 3) % 8, 3)])


def test_ragged_batch_full_28_layers(lib):
    wl = W.get_workload("ragged_b8")
    print("workload", wl.name, "28 layers R=2", flush=True)
    layers, prob, sel, k_out, v_out = run_stack(lib, wl, 2)
    check_structure_everywhere(wl, prob, sel, 2)
    check_gather_everywhere(wl, layers, prob, sel, k_out, v_out, 2)
    check_sampled_selections(lib, wl, layers, prob, sel, 2, [(13, int(np.argmin(wl.seqlens)), 0)])


def test_stack_128k_with_caller_lse(lib, scoring_path):
    """chunkkv_compress_stack_lse at the benchmark's shape (8 of the 32 layers): structure and gather everywhere,
    sampled selections against the oracle's scores from the same log-sum-exps."""
    if scoring_path == "two_pass":
        pytest.skip("the log-sum-exp variant has one implementation; run once")
    wl = W.get_workload("llama8b_128k_stack").with_(n_layers=8)
    R, N = 2, 8
    print("workload", wl.name, "8 layers R=2, caller-supplied log-sum-exps", flush=True)
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl, layers[0])
    # the caller's values: fp32 log-sum-exps from library ops on the device (harness-side input)
    g, w, d, L = wl.group, wl.window, wl.head_dim, wl.seqlens[0]
    P = L - w
    hidden = torch.arange(L, device=DEV)[None, :] > (P + torch.arange(w, device=DEV))[:, None]
    lses = []
    for l in range(N):
        if l % R:
            lses.append(None)
            continue
        out = torch.empty((1, wl.n_q_heads, w), dtype=torch.float32, device=DEV)
        for h in range(wl.n_kv_heads):
            q = layers[l].q[0, h * g:(h + 1) * g].double().reshape(g * w, d)
            s = (q @ layers[l].k[0, h].double().T) / d ** 0.5
            out[0, h * g:(h + 1) * g] = torch.logsumexp(s.view(g, w, L).masked_fill(hidden[None], float("-inf")), dim=2).float()
        lses.append(out)
    G = N // R
    sel_chunk = torch.zeros((G, 1, wl.n_kv_heads, prob.sel_cap), dtype=torch.int32, device=DEV)
    sel_len = torch.zeros_like(sel_chunk)
    sel_count = torch.zeros((G, 1, wl.n_kv_heads), dtype=torch.int32, device=DEV)
    k_out = [torch.zeros(prob.out_elements(), dtype=wl.torch_dtype, device=DEV) for _ in range(N)]
    v_out = [torch.zeros(prob.out_elements(), dtype=wl.torch_dtype, device=DEV) for _ in range(N)]
    ws = torch.empty(lib.chunkkv_workspace_bytes(prob, N, R), dtype=torch.uint8, device=DEV)
    lib.chunkkv_compress_stack_lse(prob, R, [layers[l].q if l % R == 0 else None for l in range(N)],
                                   [x.k for x in layers], [x.v for x in layers], lses, k_out, v_out,
                                   sel_chunk, sel_len, sel_count, ws)
    torch.cuda.synchronize()
    sel = (sel_chunk, sel_len, sel_count)
    check_structure_everywhere(wl, prob, sel, R)
    check_gather_everywhere(wl, layers, prob, sel, k_out, v_out, R)
    nk = int(prob.n_keep[0])
    for (grp, h) in [(0, 2), (3, 7)]:
        li = layers[grp * R]
        q = W.tensor_bits(li.q[0, h * g:(h + 1) * g])
        k = W.tensor_bits(li.k[0, h:h + 1])
        lse = lses[grp * R][0, h * g:(h + 1) * g].double().cpu().numpy()
        o_cs, _ = orc.score_from_lse(q, k, lse, w, wl.chunk)
        got = H.read_selection(prob, *sel, grp)[0][h]
        dd = H.check_selection(got, orc.chunk_topk(o_cs[0], P, wl.chunk, nk), o_cs[0], P, wl.chunk, nk)
        print(f"group {grp} head {h}: {dd} chunks differ inside the tie band", flush=True)


def test_one_million_tokens_single_head(lib, scoring_path):
    """Largest sizes: one kv-head of 1,000,003 tokens (a ragged last tile, block and chunk), 128 window rows.
    Chunk scores against the oracle over the whole length, then selection and gather through the stack call."""
    wl = W.get_workload("llama8b_8k").with_(n_q_heads=4, n_kv_heads=1, seqlens=(1_000_003,), n_spans=(300,), n_layers=1)
    print("workload 1,000,003 tokens, 4 q / 1 kv head, w=32, c=10", scoring_path, flush=True)
    li = W.make_layer(wl, 0, DEV)
    prob = H.make_problem(lib, wl, li)
    cs = torch.zeros((1, 1, prob.score_cap), dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.chunkkv_workspace_bytes(prob), dtype=torch.uint8, device=DEV)
    lib.chunkkv_score(prob, li.q, li.k, cs, None, ws)
    torch.cuda.synchronize()
    q, k, _ = H.seq_arrays(wl, li, 0)
    o_cs, _ = orc.score(q, k, wl.window, wl.chunk)
    err = H.rel_err(cs[0, 0, :o_cs.shape[1]].cpu().numpy(), o_cs[0])
    print(f"max relative score error over {o_cs.shape[1]} chunks: {err:.3e}", flush=True)
    assert err <= H.REL_TOL
    layers, prob, sel, k_out, v_out = run_stack(lib, wl, 1, [li])
    check_structure_everywhere(wl, prob, sel, 1)
    check_gather_everywhere(wl, layers, prob, sel, k_out, v_out, 1)
    P, nk = wl.seqlens[0] - wl.window, int(prob.n_keep[0])
    got = H.read_selection(prob, *sel, 0)[0][0]
    d = H.check_selection(got, orc.chunk_topk(o_cs[0], P, wl.chunk, nk), o_cs[0], P, wl.chunk, nk)
    print(f"{d} chunks differ inside the tie band", flush=True)


def test_hybrid_chunk_sizes_128k(lib, scoring_path):
    """chunkkv_compress_stack_hybrid at the long-context shape: 6 layers, R = 2, chunk sizes 10, 1 and 20 (the
    token-level group has 131008 candidates and 13101 selection entries per head).  Structure and gather for every
    layer and head, sampled selections against the oracle."""
    if scoring_path == "two_pass":
        pytest.skip("chunk size 1 takes the two-pass kernels anyway; run once")
    wl = W.get_workload("llama8b_128k_stack").with_(n_layers=6)
    R, N, chunks = 2, 6, [10, 1, 20]
    print("workload", wl.name, "6 layers R=2 chunk sizes", chunks, flush=True)
    layers = [W.make_layer(wl, l, DEV) for l in range(N)]
    prob = H.make_problem(lib, wl.with_(chunk=1), layers[0])          # capacities for the smallest chunk size
    G, Hk = 3, wl.n_kv_heads
    sel = (torch.zeros((G, 1, Hk, prob.sel_cap), dtype=torch.int32, device=DEV),
           torch.zeros((G, 1, Hk, prob.sel_cap), dtype=torch.int32, device=DEV),
           torch.zeros((G, 1, Hk), dtype=torch.int32, device=DEV))
    k_out = [torch.zeros(prob.out_elements(), dtype=wl.torch_dtype, device=DEV) for _ in range(N)]
    v_out = [torch.zeros(prob.out_elements(), dtype=wl.torch_dtype, device=DEV) for _ in range(N)]
    ws = torch.empty(lib.chunkkv_workspace_bytes_hybrid(prob, N, R, chunks), dtype=torch.uint8, device=DEV)
    lib.chunkkv_compress_stack_hybrid(prob, R, chunks, [layers[l].q if l % R == 0 else None for l in range(N)],
                                      [x.k for x in layers], [x.v for x in layers], None, k_out, v_out, *sel, ws)
    torch.cuda.synchronize()
    for grp, c in enumerate(chunks):
        wl_g = wl.with_(chunk=c, n_layers=R)
        sel_g = tuple(t[grp:grp + 1] for t in sel)
        check_structure_everywhere(wl_g, prob, sel_g, R)
        check_gather_everywhere(wl_g, layers[grp * R:(grp + 1) * R], prob, sel_g, k_out[grp * R:(grp + 1) * R],
                                v_out[grp * R:(grp + 1) * R], R)
        n = check_sampled_selections(lib, wl_g, layers[grp * R:(grp + 1) * R], prob, sel_g, R, [(0, 0, (3 * grp + 1) % 8)])
        print(f"group {grp} (c={c}): {n} chunks differ inside the tie band", flush=True)


def test_quality_metrics_128k(lib, scoring_path):
    """chunkkv_quality_metrics on one full-size layer (131072 tokens, 32 / 8 heads, keep 10 %) against the oracle."""
    if scoring_path == "two_pass":
        pytest.skip("the metrics do not depend on the scoring path; run once")
    wl = W.get_workload("llama8b_128k_stack").with_(n_layers=1)
    layers, prob, sel, k_out, v_out = run_stack(lib, wl, 1)
    li = layers[0]
    q_dec = li.q[:, :, -1, :].contiguous()
    l1 = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
    cos = torch.full((1, wl.n_q_heads), -1.0, dtype=torch.float32, device=DEV)
    qws = torch.empty(lib.chunkkv_quality_workspace_bytes(prob), dtype=torch.uint8, device=DEV)
    lib.chunkkv_quality_metrics(prob, None, q_dec, li.k, li.v, k_out[0], v_out[0], l1, cos, qws)
    torch.cuda.synchronize()
    got = H.read_selection(prob, *sel, 0)
    _, k, v = H.seq_arrays(wl, li, 0)
    kept = [orc.kept_token_indices(got[0][h][0], got[0][h][1], wl.seqlens[0], wl.window, wl.chunk) for h in range(wl.n_kv_heads)]
    l1_ref = orc.kv_l1_loss(k, v, kept)
    cos_ref = orc.attention_cosine(W.tensor_bits(q_dec[0]), k, kept)
    print(f"L1 loss {float(l1[0]):.6f} (oracle {l1_ref:.6f}); cosine mean {float(cos.mean()):.6f} (oracle {cos_ref.mean():.6f})",
          flush=True)
    assert abs(float(l1[0]) - l1_ref) <= 1e-6
    assert np.all(np.abs(cos[0].cpu().numpy() - cos_ref) <= 1e-4 * cos_ref)
