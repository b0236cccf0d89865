// Host-side internals shared by the translation units of the library.
#pragma once

#include "klpm.h"
#include "klpm_device.hpp"

struct kLPM_tree {
    kLPM_config cfg;
    klpm::TreeView tv;
    klpm::CommitWs ws;
    void *arena;
    size_t arena_bytes;
    int64_t budget;
    int64_t protect;    // most recently admitted prompts whose paths eviction must leave alone
    uint64_t clock_ub;  // host-side upper bound of the logical clock (sizes the eviction key)
    uint64_t clock_reserve;  // admissions the caller may enqueue without this host code seeing them
    int depth_bits;     // bits needed for a depth value (<= max_prompt_len)
};

namespace klpm {

// Enqueue the match kernel. `sel` (device, may be NULL) redirects wave w to query sel[w]; `n_dev`
// (device, may be NULL) caps the number of active waves at run time. Returns 0 or KLPM_EHIP.
int launch_match(const TreeView &tv, const QView &q, const int32_t *sel, const int32_t *n_dev, int32_t n_cap,
                 int honor_skip, int32_t *out_len, int32_t *out_node, hipStream_t stream);

// Enqueue one whole commit (insert + evict) on the stream.  hint_len/hint_node (both or neither):
// queue-wide match results on the current tree, indexed like q, that replace the commit's own match.
int commit_pipeline(kLPM_tree *t, const QView &q, const int32_t *batch_idx, const int32_t *n_selected,
                    int32_t batch_cap, int64_t budget, int64_t protect, kLPM_stats *stats_out, hipStream_t stream,
                    const int32_t *hint_len = nullptr, const int32_t *hint_node = nullptr);

// The two total orders behind Algorithm 1's picks, as built by the sorting path of the selection:
// queue indices in oldest-first order (arrival, index) and in longest-match order (-score, [tie key,]
// arrival, index), and every query's position in each.  The arrays live in the caller's workspace.
struct SelectOrders {
    const uint32_t *order_a, *order_l, *rank_a, *rank_l;
    const int32_t *violated;  // NULL, or DEVICE [1]: non-zero when a promise about the queue did not hold
};
size_t select_sort_workspace_bytes(int32_t n);
int build_select_orders(const uint64_t *arrival, const int32_t *score, const uint32_t *tie_key, int32_t n,
                        const int32_t *n_live, bool want_l, void *workspace, size_t workspace_bytes,
                        hipStream_t stream, SelectOrders *out, bool arrival_ordered = false, int32_t max_score = 0);

inline int check_launch() { return hipGetLastError() == hipSuccess ? KLPM_OK : KLPM_EHIP; }

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace klpm
