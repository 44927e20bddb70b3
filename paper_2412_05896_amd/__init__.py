"""MI355X-native decode hot path of XKV (arXiv 2412.05896).

A thin ctypes binding over libxkv.so, the C-ABI library declared in
include/xkv.h.  Every step of the path runs in the library's HIP kernels (or, for
the budget allocator, its host C++); this package only marshals arguments.
PyTorch supplies device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    XKV_ALLOC_TARGET_RAVG,
    XKV_ALLOC_TOTAL_SIZE,
    XKV_CFG_ATTEND_PATH,
    XKV_CFG_FUSED_SPIN_LIMIT,
    XkvCache,
    XkvError,
    load,
    status_string,
    xkv_allocate_budgets,
    xkv_allocate_budgets_device,
    xkv_allocate_device_workspace_bytes,
    xkv_average_allocations,
    xkv_cache_importance,
    xkv_configure,
    xkv_decode_attend_score,
    xkv_decode_step,
    xkv_decode_attend_score_noalloc,
    xkv_evict_compact,
    xkv_fused_status,
    xkv_prefill_evict,
    xkv_prefill_evict_lse,
    xkv_prefill_workspace_bytes,
    xkv_probe_stream_read,
    xkv_profile_enable,
    xkv_profile_read,
    xkv_repack,
    xkv_window_importance,
    xkv_window_importance_lse,
    xkv_workspace_bytes,
)
