"""Seeded synthetic KV-cache workloads shared by the tests, the oracle checks and bench.py.

This package only *draws inputs* (Gaussian Q/K/V with planted salient spans) and
describes their memory layout.  It contains none of the compression method's
arithmetic: no scoring, no selection, no gather.
"""
from .synth import (  # noqa: F401
    Workload,
    LayerInputs,
    WORKLOADS,
    get_workload,
    make_layer,
    keep_budget,
    bf16_bits_to_f64,
    tensor_bits,
)
