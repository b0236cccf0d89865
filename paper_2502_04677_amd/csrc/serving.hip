// Serving-side steps around the scheduling path: the dynamic batch size under a prefill token budget
// (Sec. 2.1: dynamic batch size with a fixed memory pool) and the cache slots of a batch's matched
// prefixes (what the prefix cache hands to attention: RadixAttention, Sec. 1).
#include "klpm_internal.hpp"

namespace klpm {

constexpr int kCutThreads = 1024;

// Keep the longest prefix of the picks whose uncached tokens fit the budget (the first pick always
// stays), and rewind the k-cycle by the picks handed back.
__global__ __launch_bounds__(kCutThreads) void k_batch_token_budget(QView q, const int32_t *__restrict__ match_len,
                                                                    const int32_t *__restrict__ batch_idx,
                                                                    int32_t *__restrict__ n_selected, int32_t batch_cap,
                                                                    int64_t token_budget, KArg ka,
                                                                    uint32_t *__restrict__ phase_inout) {
    const uint32_t k = ka.get();
    __shared__ int64_t part[kCutThreads / kWave];
    __shared__ int32_t s_keep;
    const int tid = threadIdx.x;
    int32_t nb = *n_selected;
    nb = nb < 0 ? 0 : (nb > batch_cap ? batch_cap : nb);
    const int32_t n_q = live_count(q.n, q.n_live);
    if (tid == 0) s_keep = nb;
    // contiguous runs of picks per thread, one scan over the per-thread sums
    const int32_t per = (nb + kCutThreads - 1) / kCutThreads;
    const int32_t lo = tid * per < nb ? tid * per : nb;
    const int32_t hi = lo + per < nb ? lo + per : nb;
    int64_t mine = 0;
    for (int32_t j = lo; j < hi; ++j) {
        const int32_t i = batch_idx[j];
        if (i >= 0 && i < n_q) {
            int32_t m = match_len[i];
            m = m < 0 ? 0 : m;
            const int32_t len = q.len[i];
            if (len > m) mine += (int64_t)(len - m);
        }
    }
    int64_t all;
    int64_t run = block_inclusive_scan<int64_t, kCutThreads>(mine, part, tid, all) - mine;
    for (int32_t j = lo; j < hi; ++j) {
        const int32_t i = batch_idx[j];
        if (i >= 0 && i < n_q) {
            int32_t m = match_len[i];
            m = m < 0 ? 0 : m;
            const int32_t len = q.len[i];
            if (len > m) run += (int64_t)(len - m);
        }
        if (j > 0 && run > token_budget) { atomicMin(&s_keep, j); break; }  // costs are non-negative: first overflow
    }
    __syncthreads();
    if (tid == 0) {
        const int32_t keep = s_keep;
        if (keep < nb) {
            *n_selected = keep;
            const bool lpm_only = (k == 0u || k == 0xFFFFFFFFu);
            if (!lpm_only) {
                const uint32_t back = (uint32_t)((uint64_t)(uint32_t)(nb - keep) % k);
                const uint32_t ph = *phase_inout % k;
                *phase_inout = (ph + k - back) % k;
            }
        }
    }
}

// One wavefront per admitted prompt walks its matched prefix and writes, for every matched token,
// the pool position that holds it (the slot of that token's cache entry).
__global__ __launch_bounds__(256) void k_kv_slots(TreeView tv, QView q, const int32_t *__restrict__ batch_idx,
                                                  const int32_t *__restrict__ n_selected, int32_t batch_cap,
                                                  int32_t stride, int32_t *__restrict__ n_matched,
                                                  int64_t *__restrict__ slots) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t w = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    int32_t nb = uni(*n_selected);
    nb = nb < 0 ? 0 : (nb > batch_cap ? batch_cap : nb);
    if (w >= batch_cap) return;
    if (w >= nb) {
        if (lane == 0) n_matched[w] = 0;
        return;
    }
    const int32_t qi = uni(batch_idx[w]);
    bool bad = qi < 0 || qi >= uni(live_count(q.n, q.n_live));
    int64_t off = 0;
    int32_t L = 0;
    if (!bad) {
        off = uni64(q.off[qi]);
        L = uni(q.len[qi]);
        bad = off < 0 || L < 1 || L > tv.max_prompt_len || off + (int64_t)L > q.n_tokens;
    }
    if (bad) {
        if (lane == 0) {
            n_matched[w] = -1;
            atomicOr(&tv.st->device_error, 4u /* KLPM_DEV_BAD_INPUT */);
        }
        return;
    }
    if (L > stride) L = stride;  // never write past the row
    const int32_t *__restrict__ x = q.tokens + off;
    int64_t *__restrict__ row = slots + w * (int64_t)stride;
    int32_t cur = kRoot, d = 0;
    while (d < L) {
        int32_t c, el;
        int64_t eo;
        if (slot_find(tv.slots, tv.slot_mask, make_key(cur, uni(x[d])), c, el, eo) < 0) break;
        const int32_t lim = el < L - d ? el : L - d;
        const int32_t j = wave_common_prefix(x + d, tv.pool + eo, lim, lane);
        for (int32_t t = lane; t < j; t += kWave) row[d + t] = eo + t;
        d += j;
        if (j < el) break;
        cur = c;
    }
    if (lane == 0) n_matched[w] = d;
}

__global__ __launch_bounds__(256) void k_gather_slots(TreeView tv, const int64_t *__restrict__ slots, int64_t n,
                                                      int64_t pool_total, int32_t *__restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t s = slots[i];
    out[i] = (s >= 0 && s < pool_total) ? tv.pool[s] : -1;
}

}  // namespace klpm

using namespace klpm;

extern "C" int kLPM_batch_token_budget(const kLPM_queries *q, const int32_t *match_len, const int32_t *batch_idx,
                                       int32_t *n_selected, int32_t batch_cap, int64_t token_budget, uint32_t k,
                                       const uint32_t *k_dev, uint32_t *phase_inout, kLPM_stream stream) {
    if (!q || q->n < 0 || batch_cap < 0 || token_budget < 0 || !n_selected || !phase_inout) return KLPM_EINVAL;
    if (batch_cap > 0 && (!batch_idx || !match_len || !q->len)) return KLPM_EINVAL;
    QView qv;
    qv.tokens = q->tokens; qv.off = q->off; qv.len = q->len; qv.n_tokens = q->n_tokens; qv.n = q->n; qv.n_live = q->n_live;
    hipLaunchKernelGGL(k_batch_token_budget, dim3(1), dim3(kCutThreads), 0, (hipStream_t)stream, qv, match_len, batch_idx,
                       n_selected, batch_cap, token_budget, KArg{k, k_dev}, phase_inout);
    return check_launch();
}

extern "C" int kLPM_kv_slots(kLPM_tree *tree, const kLPM_queries *q, const int32_t *batch_idx, const int32_t *n_selected,
                             int32_t batch_cap, int32_t stride, int32_t *n_matched, int64_t *slots, kLPM_stream stream) {
    if (!tree || !q || q->n < 0 || q->n_tokens < 0 || batch_cap < 0 || stride < 1 || !n_selected) return KLPM_EINVAL;
    if (batch_cap == 0) return KLPM_OK;
    if (!batch_idx || !n_matched || !slots || !q->tokens || !q->off || !q->len) return KLPM_EINVAL;
    QView qv;
    qv.tokens = q->tokens; qv.off = q->off; qv.len = q->len; qv.n_tokens = q->n_tokens; qv.n = q->n; qv.n_live = q->n_live;
    const int waves = 4;
    hipLaunchKernelGGL(k_kv_slots, dim3((unsigned)((batch_cap + waves - 1) / waves)), dim3(waves * kWave), 0,
                       (hipStream_t)stream, tree->tv, qv, batch_idx, n_selected, batch_cap, stride, n_matched, slots);
    return check_launch();
}

extern "C" int kLPM_gather_slots(kLPM_tree *tree, const int64_t *slots, int64_t n, int32_t *tokens_out, kLPM_stream stream) {
    if (!tree || n < 0) return KLPM_EINVAL;
    if (n == 0) return KLPM_OK;
    if (!slots || !tokens_out) return KLPM_EINVAL;
    hipLaunchKernelGGL(k_gather_slots, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, tree->tv, slots,
                       n, 2 * tree->cfg.pool_tokens, tokens_out);
    return check_launch();
}
