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
    uint64_t clock_ub;  // host-side upper bound of the logical clock (sizes the eviction key)
    int depth_bits;     // bits needed for a depth value (<= max_prompt_len)
};

namespace klpm {

// Enqueue the match kernel. `sel` (device, may be NULL) redirects wave w to query sel[w]; `n_dev`
// (device, may be NULL) caps the number of active waves at run time. Returns 0 or KLPM_EHIP.
int launch_match(const TreeView &tv, const QView &q, const int32_t *sel, const int32_t *n_dev, int32_t n_cap,
                 int honor_skip, int32_t *out_len, int32_t *out_node, hipStream_t stream);

// Enqueue one whole commit (insert + evict) on the stream.
int commit_pipeline(kLPM_tree *t, const QView &q, const int32_t *batch_idx, const int32_t *n_selected,
                    int32_t batch_cap, int64_t budget, kLPM_stats *stats_out, hipStream_t stream);

inline int check_launch() { return hipGetLastError() == hipSuccess ? KLPM_OK : KLPM_EHIP; }

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace klpm
