"""The seeded generator: shapes, layout description, determinism, recipe."""
import numpy as np
import torch

import workloads as wlmod
from workloads import synth


def test_tiny_shapes_and_determinism():
    wl = wlmod.get_workload("tiny")
    a = wlmod.make_layer(wl, 0)
    b = wlmod.make_layer(wl, 0)
    assert a.q.shape == (1, 4, 16, 64) and a.k.shape == (1, 2, 512, 64) and a.v.shape == a.k.shape
    assert a.k.dtype == torch.float32
    assert torch.equal(a.k, b.k) and torch.equal(a.q, b.q) and torch.equal(a.v, b.v)
    assert len(a.spans[0]) == 3 and all(5 <= n <= 20 and 0 <= s <= 496 - n for s, n in a.spans[0])
    assert wlmod.keep_budget(512, 16, 25) == 124


def test_spans_raise_key_query_alignment():
    wl = wlmod.get_workload("tiny")
    li = wlmod.make_layer(wl, 0)
    u = torch.from_numpy(synth.layer_direction(wl, 0))
    proj = (li.k[0, 0] @ u)
    in_span = torch.zeros(512, dtype=torch.bool)
    for s, n in li.spans[0]:
        in_span[s:s + n] = True
    assert proj[in_span].mean() > 1.5 and abs(proj[~in_span].mean()) < 0.3
    assert (li.q[0] @ u).mean() > 1.5


def test_adjacent_layers_share_most_spans():
    wl = wlmod.get_workload("llama8b_32k_stack")
    s0 = set(synth.layer_spans(wl, 0)[0])
    s1 = set(synth.layer_spans(wl, 1)[0])
    assert len(s0) == 160 and 0.6 * 160 <= len(s0 & s1) <= 0.95 * 160


def test_ragged_layout_views():
    wl = wlmod.get_workload("ragged_b8").with_(seqlens=(70, 45, 64), n_spans=(1, 1, 1), n_layers=1)
    li = wlmod.make_layer(wl, 0)
    assert li.k.shape == (179, 4, 128) and li.k.dtype == torch.bfloat16
    assert li.kv_stride_head == 128 and li.kv_stride_tok == 4 * 128
    assert li.kv_base == (0, 70 * 512, 115 * 512)
    v1 = li.seq_view(li.k, 1, 4, 128)
    assert v1.shape == (4, 45, 128) and torch.equal(v1[2, 7], li.k[70 + 7, 2])
    bits = wlmod.tensor_bits(li.k)
    assert bits.dtype == np.uint16
    assert np.array_equal(wlmod.bf16_bits_to_f64(bits), li.k.double().numpy())


def test_fp16_layers_widen_exactly():
    wl = wlmod.get_workload("llama8b_8k").with_(dtype="f16", seqlens=(100,), n_spans=(1,), n_layers=1)
    li = wlmod.make_layer(wl, 0)
    assert li.k.dtype == torch.float16 and li.q.dtype == torch.float16 and wl.elem_bytes == 2
    bits = wlmod.tensor_bits(li.k)
    assert bits.dtype == np.float16 and np.array_equal(bits.astype(np.float64), li.k.double().numpy())
    # same draw as the bf16 workload before rounding: both round one fp32 tensor
    lb = wlmod.make_layer(wl.with_(dtype="bf16"), 0)
    assert float((li.k.float() - lb.k.float()).abs().max()) < 0.05


def test_real_ragged_lengths_in_range():
    wl = wlmod.get_workload("ragged_b8")
    assert wl.batch == 8 and all(4096 <= L <= 65536 for L in wl.seqlens)
