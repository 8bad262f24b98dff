"""MI355X-native mixed append-prefill + decode paged attention (libppd) -- thin Python binding.

The functions here carry the names of the C ABI in include/ppd.h and only marshal arguments; every step
of the path runs in the HIP kernels of libppd.so.  There is no CPU fallback: loading fails loudly when
the library has not been built (`python -m paper_2603_13358_amd.build`).
"""
from .binding import (PPDError, Context, WorkItem, PlanStats, Shape, lib_path, load_library, ppd_create,
                      ppd_destroy, ppd_device_error_flags, ppd_get_plan_stats, ppd_kv_append, ppd_kv_land, ppd_transfer_delay_s, ppd_last_error, ppd_last_kernel_ms, ppd_timed_kernels_ms,
                      ppd_mixed_attention, ppd_mixed_attention_static, ppd_plan_build, ppd_route_cell, ppd_route_decide, ppd_route_decide_batch, ppd_route_score, ppd_route_table_build,
                      ppd_set_option, ppd_set_kv_format, PPD_KV_BF16, PPD_KV_FP8_E4M3, ppd_version)

__all__ = ["PPDError", "Context", "WorkItem", "PlanStats", "Shape", "lib_path", "load_library", "ppd_create",
           "ppd_destroy", "ppd_device_error_flags", "ppd_get_plan_stats", "ppd_kv_append", "ppd_kv_land", "ppd_transfer_delay_s", "ppd_last_error", "ppd_last_kernel_ms", "ppd_timed_kernels_ms",
           "ppd_mixed_attention", "ppd_mixed_attention_static", "ppd_plan_build", "ppd_route_cell", "ppd_route_decide", "ppd_route_decide_batch", "ppd_route_score", "ppd_route_table_build",
           "ppd_set_option", "ppd_set_kv_format", "PPD_KV_BF16", "PPD_KV_FP8_E4M3", "ppd_version"]
