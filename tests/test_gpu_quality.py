"""GPU parity of chunkkv_quality_metrics (KV-cache L1 loss and attention cosine similarity of a compressed
layer against the full one, Appendix A.1) against the CPU oracle, through the C ABI.

The compressed cache is produced by the library's own stack call; the oracle gets the kept token indices of
the selection the GPU made, so the comparison isolates the metrics.  Bars: L1 loss within 1e-6 absolute
(fp32 partial sums of about a thousand rows, fp64 above that), cosine within 1e-4 relative (it is
exp((lse_kept - lse_all) / 2) of two fp32 log-sum-exps); measured: 4e-8 and 7e-7.
Parity unpinned against the paper's own table: its numbers come from real model activations."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import chunkkv_oracle as orc
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
L1_TOL = 1e-6
COS_TOL = 1e-4

CASES = {
    "bf16_4k_10pct": W.get_workload("llama8b_32k_stack").with_(seqlens=(4096,), n_spans=(20,), n_layers=1),
    "bf16_w64_30pct": W.get_workload("llama8b_128k_stack").with_(seqlens=(3000,), n_spans=(9,), n_layers=1, keep_pct=30),
    "f16_g6": W.get_workload("llama8b_8k").with_(dtype="f16", n_q_heads=12, n_kv_heads=2, seqlens=(2222,), n_spans=(5,)),
    "f32_tiny": W.get_workload("tiny"),
    "ragged_bf16_c5": W.get_workload("ragged_b8").with_(seqlens=(1500, 640, 2304, 97), n_spans=(7, 3, 11, 0), n_layers=1,
                                                        chunk=5, keep_pct=30),
    "bf16_b19_sliced": W.get_workload("ragged_b8").with_(seqlens=tuple(90 + 53 * i for i in range(19)), n_spans=(1,) * 19,
                                                         n_layers=1, keep_pct=20),
    "bf16_nhd": W.get_workload("llama8b_8k").with_(n_q_heads=6, n_kv_heads=2, seqlens=(4100,), n_spans=(9,), layout="nhd"),
}


def run_case(lib, wl, flags=0, keep_all=False):
    li = W.make_layer(wl, 0, DEV)
    n_keep = [L - wl.window for L in wl.seqlens] if keep_all else None
    prob = H.make_problem(lib, wl, li, n_keep=n_keep, flags=flags)
    B, Hk = wl.batch, wl.n_kv_heads
    sel = (torch.zeros((1, B, Hk, prob.sel_cap), dtype=torch.int32, device=DEV),
           torch.zeros((1, B, Hk, prob.sel_cap), dtype=torch.int32, device=DEV),
           torch.zeros((1, B, Hk), dtype=torch.int32, device=DEV))
    k_out = torch.zeros(prob.out_elements(), dtype=li.k.dtype, device=DEV)
    v_out = torch.zeros_like(k_out)
    ws = torch.empty(lib.chunkkv_workspace_bytes(prob, 1, 1), dtype=torch.uint8, device=DEV)
    lib.chunkkv_compress_stack(prob, 1, [li.q], [li.k], [li.v], [k_out], [v_out], *sel, ws)
    q_dec = li.q[:, :, -1, :].contiguous()
    kv_len = None
    if flags & lib.FLAG_WHOLE_CHUNKS:
        # tokens per (sequence, kv-head): the kept chunks' lengths plus the window
        lens = sel[1][0].cpu().numpy()
        cnt = sel[2][0].cpu().numpy()
        kv_np = np.array([[int(lens[b, h, :cnt[b, h]].sum()) + wl.window for h in range(Hk)] for b in range(B)], dtype=np.int32)
        kv_len = torch.from_numpy(kv_np).to(DEV)
    l1 = torch.full((B,), -1.0, dtype=torch.float32, device=DEV)
    cos = torch.full((B, wl.n_q_heads), -1.0, dtype=torch.float32, device=DEV)
    n_ws = lib.chunkkv_quality_workspace_bytes(prob)
    assert n_ws > 0
    qws = torch.full((n_ws,), 0xCD, dtype=torch.uint8, device=DEV)   # nothing in it has to be initialised
    lib.chunkkv_quality_metrics(prob, kv_len, q_dec, li.k, li.v, k_out, v_out, l1, cos, qws)
    torch.cuda.synchronize()
    got = H.read_selection(prob, *sel, 0)
    return li, prob, got, q_dec, l1.cpu().numpy(), cos.cpu().numpy()


def check_against_oracle(wl, li, prob, got, q_dec, l1, cos):
    worst_l1 = worst_cos = 0.0
    for b in range(wl.batch):
        _, k, v = H.seq_arrays(wl, li, b)
        kept = [orc.kept_token_indices(got[b][h][0], got[b][h][1], wl.seqlens[b], wl.window, wl.chunk) for h in range(wl.n_kv_heads)]
        l1_ref = orc.kv_l1_loss(k, v, kept)
        cos_ref = orc.attention_cosine(W.tensor_bits(q_dec[b]), k, kept)
        worst_l1 = max(worst_l1, abs(float(l1[b]) - l1_ref))
        worst_cos = max(worst_cos, float(np.max(np.abs(cos[b] - cos_ref) / cos_ref)))
        assert abs(float(l1[b]) - l1_ref) <= L1_TOL, (b, l1[b], l1_ref)
        assert np.all(np.abs(cos[b] - cos_ref) <= COS_TOL * cos_ref), (b, cos[b], cos_ref)
    print(f"worst |l1 - oracle| = {worst_l1:.2e}, worst cosine rel. error = {worst_cos:.2e}")


@pytest.mark.parametrize("case", list(CASES))
def test_quality_metrics_match_oracle(lib, case):
    wl = CASES[case]
    print(f"case={case}", flush=True)
    li, prob, got, q_dec, l1, cos = run_case(lib, wl)
    check_against_oracle(wl, li, prob, got, q_dec, l1, cos)
    assert np.all((l1 > 0) & (l1 < 1)) and np.all((cos > 0) & (cos <= 1.0 + 1e-6))


def test_quality_metrics_whole_chunk_mode(lib):
    # Algorithm 3 as printed keeps floor(n_keep / c) whole chunks: the caches hold fewer tokens than their
    # capacity and kv_len says how many
    wl = CASES["ragged_bf16_c5"].with_(chunk=7)
    li, prob, got, q_dec, l1, cos = run_case(lib, wl, flags=lib.FLAG_WHOLE_CHUNKS)
    check_against_oracle(wl, li, prob, got, q_dec, l1, cos)


def test_keep_everything_is_lossless(lib):
    wl = W.get_workload("llama8b_8k").with_(seqlens=(1111,), n_spans=(3,), n_layers=1)
    _, _, _, _, l1, cos = run_case(lib, wl, keep_all=True)
    assert np.all(np.abs(l1) <= 1e-6)
    assert np.all(np.abs(cos - 1.0) <= 1e-5)
