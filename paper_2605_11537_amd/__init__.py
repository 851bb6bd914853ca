"""MI355X (gfx950) library for the top-1 MoE layer forward with predictor-driven dynamic
expert replication: HIP kernels behind a C ABI (``include/moe_mpmc.h``) and a thin ctypes
binding on torch tensors."""
from .binding import (  # noqa: F401
    EXPORTS,
    LAYOUT_PACKED,
    LAYOUT_PLAIN,
    LIB_PATH,
    MOE_BF16,
    MOE_F32,
    SCHEDULE_EXPERTS,
    SCHEDULE_SLOTS,
    MoeError,
    MoeLayer,
    MoePipeline,
    SruWeights,
    lib,
    moe_combine,
    moe_dispatch,
    moe_expert_ffn,
    moe_pack_weights,
    moe_route,
    replica_plan,
    sru_predict,
    set_ffn_timing_events,
)
