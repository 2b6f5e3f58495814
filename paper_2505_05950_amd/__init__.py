"""MI355X-native FloE decode path: compressed sparse expert FFN (quantized up GEMV, threshold
selection, gathered gate/down GEMVs, top-k combine) behind a C ABI (include/floe.h).

`paper_2505_05950_amd.binding` marshals torch tensors into that ABI; every step runs in the HIP
library.  There is no host fallback: loading fails loudly when the library has not been built.
"""
from .binding import (  # noqa: F401
    FloeError, Expert, Layer, lib_path, load,
    floe_quantize_expert, floe_up_gemv, floe_select_channels, floe_gate_down_sparse,
    floe_expert_ffn_sparse, floe_expert_workspace_bytes, floe_layer_build_table, floe_layer_table_bytes,
    floe_layer_workspace_bytes, floe_moe_layer_decode, floe_moe_layer_decode_static, STATIC_SCRATCH_BYTES,
    floe_moe_layer_decode_offloaded, floe_moe_layer_prefetch,
    floe_moe_layer_decode_prefetched, Prefetch, MissPath, PREFETCH_STAT_DTYPE, floe_stage_channels, floe_status_string,
    words_per_channel, SLOT_STAT_DTYPE, floe_profile_kernel, KERNEL_IDS, floe_tuning, TUNE_UNION_KERNELS, TUNE_STAGE_WORKGROUPS, TUNE_GROUPED_GEMV, TUNE_FUSED_TASKS,
    ChannelCache, floe_channel_cache_load, floe_moe_layer_decode_cached,
    floe_expert_ffn_sparsified, SPARSIFY_UP, SPARSIFY_GATE, SPARSIFY_DOWN,
)
