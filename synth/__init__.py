"""Seeded synthetic inputs for the AirCache hot path.

This package is shared by the CPU oracle's tests, the HIP parity tests, the
smoke check and the benchmark.  It holds input generation only: shapes, token
segmentation, random tensors and their rounding to the storage dtype.  None of
the method's arithmetic (attention, scores, budgets, selection) lives here.
"""
from .configs import CONFIGS, Workload, get_workload  # noqa: F401
from .generate import (  # noqa: F401
    LayerInputs,
    bf16_bits_to_f64,
    decode_inputs,
    f32_to_bf16_bits,
    layer_inputs,
    salient_fraction,
    salient_mask,
    storage_to_f64,
)
