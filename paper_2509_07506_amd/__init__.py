"""MI355X (gfx950) implementation of the three serving operators of arxiv 2509.07506, Table 1.

The work is done by hand-written HIP kernels behind a C ABI (``include/astra.h``,
``libastra_hip.so``); this package is a thin ``ctypes`` binding with the same names.  There is no
fallback path: if the library is not built or cannot be loaded, every call raises.
"""
from .binding import (  # noqa: F401
    ASTRA_BF16,
    ASTRA_ERR_VARIANT,
    ASTRA_F16,
    ASTRA_VARIANT_LDS_TREE_REDUCTION,
    ASTRA_VARIANT_LIBM_EXP_DIVIDE,
    ASTRA_VARIANT_SCALAR_LOADS,
    ASTRA_VARIANT_TUNED,
    ASTRA_VARIANT_UNHOISTED_WEIGHTS,
    AstraError,
    LaunchInfo,
    astra_ablation_fused_add_rmsnorm,
    astra_ablation_merge_attn_states_lse,
    astra_ablation_silu_and_mul,
    astra_fused_add_rmsnorm,
    astra_merge_attn_states_lse,
    astra_merge_attn_states_lse_kway,
    astra_plan_fused_add_rmsnorm,
    astra_plan_merge_attn_states_lse,
    astra_plan_silu_and_mul,
    astra_plan_xcd_chunked,
    astra_silu_and_mul,
    astra_status_string,
    astra_stream_copy,
    fused_add_rmsnorm,
    library_path,
    load_library,
    merge_attn_states_lse,
    merge_attn_states_lse_kway,
    silu_and_mul,
    stream_copy,
)
