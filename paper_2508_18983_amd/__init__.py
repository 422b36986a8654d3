"""MI355X-native SMoE offloaded-MoE decode path: HIP library + thin binding."""
from .binding import (  # noqa: F401
    MoeCfg, MoeBuffers, MoeTrace, MoeStats, MoeProfile, MoePrefetchInfo, SmoeError, Trace,
    load_library, library_path,
    moe_cache_init, moe_decode_layer, moe_decode_layer_static, moe_prefetch_layer, moe_prefetch_last, moe_cpu_assist_costs, moe_cache_stats, moe_cache_residency,
    moe_cache_reset, moe_cache_destroy, moe_profile_enable, moe_profile_read,
    moe_last_hip_error, moe_calib_copy, moe_host_alloc, moe_host_free, moe_select_alpha, PROF_KINDS,
)
