"""Seeded synthetic inputs (weights, activations, upstream gradients) for the decoder-stage tests.

This package holds no arithmetic of the decoder layer itself: only a counter-based random
generator, the bf16 <-> fp32 format conversion and the public parameter layout.  It is the only
code that both the CPU oracle's tests and the HIP library's tests may draw inputs from.
"""
from .gen import (  # noqa: F401
    TID_GAMMA1, TID_WQKV, TID_WO, TID_GAMMA2, TID_WGU, TID_WD, TID_X, TID_DY,
    StageShape, CONFIGS, mix64, normal, f32_to_bf16_bits, bf16_bits_to_f32, round_to_storage,
    param_layout, layer_param_elems, make_params, make_x, make_dy, split_params, plan_sweep,
    EndsShape, ENDS_CONFIGS, ends_param_layout, make_ends_params, split_ends_params, make_tokens, make_targets, to_device,
)
