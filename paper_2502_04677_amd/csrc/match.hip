// Batched prefix match: one wavefront per waiting query walks the flattened radix tree.
//
// For query x the kernel computes m = max over cached strings y of overlap(x, y) (Sec. 1.2,
// Notation), i.e. the depth reached by walking x down the tree with partial edge matches counted.
// At a node boundary one child-table slot is read (it carries the child's edge span); along an
// edge the 64 lanes read query and edge tokens in coalesced rows, a ballot of the mismatching
// lanes plus a count-trailing-zeros gives the first difference.
#include "klpm_internal.hpp"

namespace klpm {

// ADMITTED = false: the queue-wide match (wave w handles query w).
// ADMITTED = true : the match of the admitted prompts inside commit (wave w handles query sel[w],
//                   the count comes from device memory, a commit that must be abandoned matches nothing).
template <bool ADMITTED>
__device__ __forceinline__ void match_body(const TreeView &tv, const QView &q, const int32_t *__restrict__ sel,
                                           const int32_t *__restrict__ n_dev, int32_t n_cap,
                                           int32_t *__restrict__ out_len, int32_t *__restrict__ out_node) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t w = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    int32_t n = n_cap;
    if (ADMITTED) {
        uint32_t err;
        n = commit_gate(tv, n_dev, n_cap, &err);  // the plan kernel records the reason of a refusal
    } else {
        n = uni(live_count(n, q.n_live));
    }
    if (w >= n) return;
    int32_t qi = ADMITTED ? uni(sel[w]) : (int32_t)w;
    bool bad = (qi < 0 || qi >= (ADMITTED ? uni(live_count(q.n, q.n_live)) : q.n));
    int64_t off = 0;
    int32_t L = 0;
    if (!bad) {
        off = uni64(q.off[qi]);
        L = uni(q.len[qi]);
        bad = (off < 0 || L < 1 || L > tv.max_prompt_len || off + (int64_t)L > q.n_tokens);
    }
    if (bad) {
        if (lane == 0) {
            out_len[w] = -1;
            if (out_node) out_node[w] = kRoot;
            atomicOr(&tv.st->device_error, 4u /* KLPM_DEV_BAD_INPUT */);
        }
        return;
    }
    const int32_t *__restrict__ x = q.tokens + off;
    const int32_t *__restrict__ pool = tv.pool;
    int32_t cur = kRoot, last = kRoot, d = 0;
    while (d < L) {
        int32_t tok = uni(x[d]);
        int32_t c, el;
        int64_t eo;
        if (slot_find(tv.slots, tv.slot_mask, make_key(cur, tok), c, el, eo) < 0) break;
        int32_t lim = el < L - d ? el : L - d;
        int32_t j = wave_common_prefix(x + d, pool + eo, lim, lane);
        d += j;
        last = c;
        if (j < el) break;  // diverged from the edge, or the prompt ended inside it
        cur = c;
    }
    if (lane == 0) {
        out_len[w] = d;
        if (out_node) out_node[w] = last;
    }
}

__global__ __launch_bounds__(256) void k_match(TreeView tv, QView q, int32_t n, int32_t *__restrict__ out_len,
                                               int32_t *__restrict__ out_node) {
    match_body<false>(tv, q, nullptr, nullptr, n, out_len, out_node);
}

__global__ __launch_bounds__(256) void k_match_admitted(TreeView tv, QView q, const int32_t *__restrict__ sel,
                                                        const int32_t *__restrict__ n_dev, int32_t n_cap,
                                                        int32_t *__restrict__ out_len,
                                                        int32_t *__restrict__ out_node) {
    match_body<true>(tv, q, sel, n_dev, n_cap, out_len, out_node);
}

int launch_match(const TreeView &tv, const QView &q, const int32_t *sel, const int32_t *n_dev, int32_t n_cap,
                 int honor_skip, int32_t *out_len, int32_t *out_node, hipStream_t stream) {
    if (n_cap <= 0) return 0;
    const int waves_per_block = 4;
    unsigned blocks = (unsigned)((n_cap + waves_per_block - 1) / waves_per_block);
    if (sel && n_dev && honor_skip) {
        hipLaunchKernelGGL(k_match_admitted, dim3(blocks), dim3(waves_per_block * kWave), 0, stream, tv, q, sel, n_dev,
                           n_cap, out_len, out_node);
    } else {
        hipLaunchKernelGGL(k_match, dim3(blocks), dim3(waves_per_block * kWave), 0, stream, tv, q, n_cap, out_len,
                           out_node);
    }
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

}  // namespace klpm
