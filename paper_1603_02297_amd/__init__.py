"""MI355X-native tensor transposition B[Pi(i)] <- alpha*A[i] + beta*B[Pi(i)] (arXiv 1603.02297, Eq. 1).

The product is libttc.so (C ABI in include/ttc.h, HIP kernels for gfx950); this package is its
thin ctypes binding plus the seeded workload table used by tests and the benchmark.
"""
from .binding import *  # noqa: F401,F403
from .binding import (TtcError, lib, ttc_execute, ttc_last_status, ttc_plan_candidate_count, ttc_plan_create, ttc_plan_create_ex,
                      ttc_plan_destroy, ttc_plan_get_info, ttc_plan_select_candidate, ttc_plan_tune, ttc_plan_tune_pairs,
                      ttc_status_string, ttc_time_ceiling, ttc_time_execute, ttc_debug_emulate_map,
                      ttc_plan_cache_store, ttc_plan_cache_lookup, ttc_plan_set_streaming,
                      ttc_plan_set_tile_mapping)
