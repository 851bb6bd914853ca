"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package draws random tensors and index patterns only.  It contains none of the
method's arithmetic (no router, no plan, no dispatch, no FFN, no SRU): anything the
method computes is computed either by ``oracle/`` or by the HIP library, never here.
"""
from .workloads import (  # noqa: F401
    CONFIGS,
    F32,
    BF16,
    normal_tensor,
    bf16_bits,
    bf16_to_f32,
    f32_to_storage,
    storage_to_f64,
    zipf_weights,
    moe_layer_inputs,
    planted_layer_inputs,
    planted_ids_hot_zipf,
    mix_ids,
    sru_inputs,
    config_inputs,
)
