"""MI355X-native k-LPM scheduling step (match / select / commit) over a GPU-resident radix tree.

The package is a binding of the C ABI declared in ``include/klpm.h``; all compute runs in the HIP
library ``libklpm.so`` built from ``csrc/``.
"""
from .binding import (  # noqa: F401
    AdaptConfig, AdaptStats, Config, DeviceArrivals, DeviceQueries, DeviceQueue, KlpmError, Stats, Tree, EXPORTS, KLPM_K_INFINITY, KLPM_SELECT_FIFO, STATS_BYTES,
    alloc_aligned, make_config, stats_from_tensor,
    kLPM_arena_bytes, kLPM_build_tree, kLPM_commit, kLPM_commit_matched, kLPM_destroy, kLPM_match, kLPM_queue_advance, kLPM_queue_advance_timed,
    kLPM_queue_gather, kLPM_read_stats, kLPM_probe_read, kLPM_score_hit_rate, kLPM_select, kLPM_select_static, KLPM_SELECT_STATIC_MAX_N, KLPM_ELIMIT, kLPM_select_dynamic, kLPM_select_dynamic_workspace_bytes, kLPM_select_workspace_bytes, kLPM_tie_keys, kLPM_set_budget, kLPM_set_protect, kLPM_reserve_clock, kLPM_batch_token_budget, kLPM_kv_slots, kLPM_gather_slots,
    kLPM_snapshot, kLPM_adapt_state_bytes, kLPM_adapt_init, kLPM_adapt_k, kLPM_adapt_observe, kLPM_adapt_read,
)
from .pipeline import AdaptiveK, Scheduler, OnlineRun, TimedRun, size_config  # noqa: F401
