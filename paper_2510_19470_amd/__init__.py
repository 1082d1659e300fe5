"""MI355X-native MoE hot path: Python binding over the C-ABI library libmoe_hip.so.

Every step of the path runs in the HIP kernels behind `include/moe.h`; this package
only marshals arguments (torch tensors -> raw device pointers, current stream)."""
from .binding import (  # noqa: F401
    MOE_BF16, MOE_F32, MOE_FFN_AUTO, MOE_FFN_VALU, MoEConfigC, MoEError, MoEContext,
    library_path, load_library, moe_combine, moe_combine_bwd, moe_create, moe_destroy,
    moe_dispatch, moe_dispatch_routed, moe_dispatch_noalloc, DispatchOut, moe_dispatch_bwd, moe_expert_ffn, moe_expert_ffn_bwd, moe_route,
    moe_route_logits, moe_set_ffn_path, moe_set_placement, moe_strerror, moe_profile_ffn, moe_profile_ffn_launches,
    moe_profile_ffn_read, moe_plan_location, moe_plan_comm_type, moe_plan_comm_frequency,
    moe_plan_expert_dest_rank, moe_plan_model, moe_sr_keep_count, moe_sr_encode, moe_sr_decode,
    moe_route_bwd, MoEPipeline, moe_measure_copy, moe_measure_mfma,
)
