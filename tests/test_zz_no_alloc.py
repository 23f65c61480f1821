"""chunkkv_decode_attention_static (the entry point for callers that cannot allocate: its partial results live
in a device-resident array of the library) against chunkkv_decode_attention (caller's workspace), through
the C ABI.

Both run the same kernels with the same key-range split, so outputs and log-sum-exps must be bit-identical.
Two calls in a row share the array, the second with a smaller input: stale partial results of the first call
must not leak into it.  A problem that needs more than the array holds is refused."""
import numpy as np
import pytest
import torch

import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _decode_both(lib, wl, seed_layer):
    li = W.make_layer(wl, seed_layer, DEV)
    prob = H.make_problem(lib, wl, li)
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    q = li.q[:, :, -1, :].contiguous()
    ws = torch.empty(lib.chunkkv_decode_workspace_bytes(prob, False), dtype=torch.uint8, device=DEV)
    out_ref = torch.full((B, Hq, d), 3.0, dtype=torch.float32, device=DEV)
    lse_ref = torch.full((B, Hq), 3.0, dtype=torch.float32, device=DEV)
    lib.chunkkv_decode_attention(prob, False, None, q, li.k, li.v, out_ref, lse_ref, ws)
    out = torch.full((B, Hq, d), 5.0, dtype=torch.float32, device=DEV)
    lse = torch.full((B, Hq), 5.0, dtype=torch.float32, device=DEV)
    lib.chunkkv_decode_attention_static(prob, False, None, q, li.k, li.v, out, lse)
    torch.cuda.synchronize()
    return out, lse, out_ref, lse_ref


def test_static_scratch_decode_matches_workspace_call_twice(lib):
    big = W.get_workload("llama8b_8k").with_(seqlens=(8192,), n_spans=(20,))
    small = W.get_workload("llama8b_8k").with_(n_q_heads=8, n_kv_heads=2, seqlens=(777,), n_spans=(3,))
    for i, wl in enumerate((big, small)):
        print(f"call {i}: L={wl.seqlens} Hq={wl.n_q_heads}", flush=True)
        out, lse, out_ref, lse_ref = _decode_both(lib, wl, i)
        assert torch.isfinite(out).all() and torch.isfinite(lse).all()
        assert torch.equal(out, out_ref), float((out - out_ref).abs().max())
        assert torch.equal(lse, lse_ref)
    # ragged batch with 7 query heads per kv-head, then again the small case
    ragged = W.get_workload("ragged_b8").with_(seqlens=(2049, 517, 33), n_spans=(10, 2, 0), n_layers=1)
    for i, wl in enumerate((ragged, small)):
        out, lse, out_ref, lse_ref = _decode_both(lib, wl, 2 + i)
        assert torch.equal(out, out_ref) and torch.equal(lse, lse_ref)


def test_static_scratch_decode_rejects_oversized_problem(lib):
    # 64 sequences x 32 query heads: the partial results of the key ranges exceed the 8 MiB array
    wl = W.get_workload("llama8b_8k").with_(seqlens=(40000,) * 64, n_spans=(0,) * 64)
    row = wl.head_dim
    prob = lib.Problem(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk, lib.BF16, list(wl.seqlens),
                       [0] * 64, [b * wl.n_kv_heads * 40000 * row for b in range(64)], 40000 * row, row)
    assert lib.chunkkv_decode_workspace_bytes(prob, False) > (8 << 20)
    dummy = torch.zeros(64, dtype=torch.float32, device=DEV)
    with pytest.raises(lib.ChunkKVError) as e:
        # rejected by the size check before any pointer is followed
        lib.chunkkv_decode_attention_static(prob, False, None, dummy, dummy, dummy, dummy, None)
    assert e.value.status == 4
