"""MI355X-native MoE prefill block (router, top-k, grouping, grouped SwiGLU expert FFN,
combine) behind a C ABI; see include/moe_prefill.h
(and include/moe_sched.h for the host-only scheduling round).  This package is the thin Python
binding: it marshals torch device tensors into the library's entry points and does no
arithmetic of its own.  Importing it does not load the library; the first call does, and
raises if libmoeprefill.so has not been built (python -m paper_2605_02960_amd.build)."""
from .binding import (  # noqa: F401
    MoEConfig, MoETaps, MoEError, DTYPE_F32, DTYPE_BF16, DTYPE_FP8_E4M3, FLAG_Y_F32,
    CALL_ROUTE, CALL_PERMUTE, CALL_GROUPED_FFN, CALL_COMBINE, CALL_PREFILL_LAYER,
    KERNEL_ROUTER_GEMM, KERNEL_TOPK, KERNEL_PERMUTE, KERNEL_GATE_UP, KERNEL_DOWN, KERNEL_COMBINE,
    KERNEL_NAMES, moe_set_profile_events, moe_init_device,
    lib, lib_path, moe_abi_version, moe_status_string, moe_workspace_bytes,
    moe_quantize_rows_e4m3, moe_route, moe_permute, moe_permute_noalloc, moe_grouped_ffn, moe_combine,
    moe_prefill_layer, make_config, EXPORTED_SYMBOLS, HipEvents, MoEStreamLayer,
    moe_layer_weight_bytes, moe_prefill_layers_streamed, moe_layer_flops_per_token,
    moe_saturation_threshold_flops, moe_calibrated_threshold_flops, moe_resolve_threshold,
    MoECostModel, moe_sched_create, moe_sched_destroy, moe_sched_hash_blocks, moe_sched_round,
    moe_sched_blocks_stored, moe_sched_blocks_evicted, moe_sched_table_size, moe_sched_tokens_executed,
)
