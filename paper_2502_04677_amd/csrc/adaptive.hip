// Adaptive k: an epsilon-greedy bandit over a caller's list of k values whose state lives in device
// memory, so that a scheduling loop never reads anything back: selections read the current k from
// the state, one small kernel per step books the TTFT of the queries that step admitted.
// (Sec. 4.2 names a multi-armed bandit as a way to set k and leaves the method open.)
#include "klpm_internal.hpp"

namespace klpm {

constexpr uint32_t kAdaptTag = 0x6B4C504Du;  // third counter word of the bandit's draws
constexpr uint32_t kAdaptMagic = 0x41444150u;

struct AdaptState {
    uint32_t k;  // first word: the k of the current arm, what kLPM_select reads through k_dev
    uint32_t magic;
    int32_t arm, n_arms, window, steps;
    uint32_t error, pad;
    uint64_t explore, seed, pulls, cur_max;
    int64_t cur_n;
    uint32_t arms[KLPM_ADAPT_MAX_ARMS];
    uint64_t count[KLPM_ADAPT_MAX_ARMS];
    uint64_t cost[KLPM_ADAPT_MAX_ARMS];
};

// Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11), all four output words.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// cost_a / count_a < cost_b / count_b, exactly (128-bit cross products; counts are positive)
__device__ __forceinline__ bool mean_less(uint64_t cost_a, uint64_t count_a, uint64_t cost_b, uint64_t count_b) {
    const uint64_t l_hi = __umul64hi(cost_a, count_b), l_lo = cost_a * count_b;
    const uint64_t r_hi = __umul64hi(cost_b, count_a), r_lo = cost_b * count_a;
    return l_hi < r_hi || (l_hi == r_hi && l_lo < r_lo);
}

__device__ int32_t next_arm(const AdaptState *s) {
    const int32_t A = s->n_arms;
    for (int32_t a = 0; a < A; ++a)
        if (s->count[a] == 0) return a;  // every arm once before anything is compared
    uint32_t w[4];
    philox4x32_10((uint32_t)s->pulls, (uint32_t)(s->pulls >> 32), kAdaptTag, 0u, (uint32_t)s->seed,
                  (uint32_t)(s->seed >> 32), w);
    if ((uint64_t)w[0] < s->explore) return (int32_t)(w[1] % (uint32_t)A);
    int32_t best = 0;
    for (int32_t a = 1; a < A; ++a)
        if (mean_less(s->cost[a], s->count[a], s->cost[best], s->count[best])) best = a;
    return best;
}

__global__ __launch_bounds__(kWave) void k_adapt_init(AdaptState *s, kLPM_adapt_config cfg) {
    const int t = threadIdx.x;
    if (t < KLPM_ADAPT_MAX_ARMS) {
        s->arms[t] = t < cfg.n_arms ? cfg.arms[t] : 0u;
        s->count[t] = 0;
        s->cost[t] = 0;
    }
    if (t == 0) {
        s->k = cfg.arms[0];
        s->magic = kAdaptMagic;
        s->arm = 0;
        s->n_arms = cfg.n_arms;
        s->window = cfg.window;
        s->steps = 0;
        s->error = 0;
        s->pad = 0;
        s->explore = cfg.explore;
        s->seed = cfg.seed;
        s->pulls = 0;
        s->cur_max = 0;
        s->cur_n = 0;
    }
}

// One scheduling step has finished: fold the TTFT of the queries it admitted into the running
// window; at the end of a window that admitted somebody, book the pull and choose the next arm.
__global__ __launch_bounds__(256) void k_adapt_observe(AdaptState *s, const int32_t *__restrict__ served_id,
                                                       const int32_t *__restrict__ served_n, int32_t served_cap,
                                                       const int32_t *__restrict__ batch_idx,
                                                       const int32_t *__restrict__ n_selected, int32_t batch_cap,
                                                       const int64_t *__restrict__ ttft, int32_t n_ttft) {
    __shared__ unsigned long long s_max;
    __shared__ int32_t s_cnt;
    __shared__ uint32_t s_err;
    const int tid = threadIdx.x;
    if (tid == 0) { s_max = 0; s_cnt = 0; s_err = 0; }
    __syncthreads();
    if (s->magic != kAdaptMagic) {  // never initialised: leave the memory alone
        return;
    }
    int32_t nb = n_selected ? *n_selected : 0;
    nb = nb < 0 ? 0 : nb;
    if (nb > batch_cap) { nb = batch_cap; if (tid == 0) atomicOr(&s_err, 8u /* KLPM_DEV_BATCH_OVERFLOW */); }
    int32_t n_q = served_n ? *served_n : 0;
    n_q = n_q < 0 ? 0 : (n_q > served_cap ? served_cap : n_q);
    unsigned long long mx = 0;
    int32_t cnt = 0;
    for (int32_t j = tid; j < nb; j += blockDim.x) {
        const int32_t qi = batch_idx[j];
        bool ok = qi >= 0 && qi < n_q;
        int64_t t = -1;
        if (ok) {
            const int32_t id = served_id[qi];
            ok = id >= 0 && id < n_ttft;
            if (ok) t = ttft[id];
        }
        if (ok && t >= 0) {
            mx = (unsigned long long)t > mx ? (unsigned long long)t : mx;
            ++cnt;
        } else {
            atomicOr(&s_err, 4u /* KLPM_DEV_BAD_INPUT */);
        }
    }
    if (cnt) { atomicMax(&s_max, mx); atomicAdd(&s_cnt, cnt); }
    __syncthreads();
    if (tid != 0) return;
    if (s_err) s->error |= s_err;
    if (s_max > s->cur_max) s->cur_max = s_max;
    s->cur_n += s_cnt;
    if (++s->steps < s->window) return;
    s->steps = 0;
    if (s->cur_n > 0) {
        s->count[s->arm] += 1;
        s->cost[s->arm] += s->cur_max;
        s->pulls += 1;
        s->arm = next_arm(s);
        s->k = s->arms[s->arm];
    }
    s->cur_max = 0;
    s->cur_n = 0;
}

}  // namespace klpm

using namespace klpm;

extern "C" int kLPM_adapt_state_bytes(size_t *out_bytes) {
    if (!out_bytes) return KLPM_EINVAL;
    *out_bytes = align_up(sizeof(AdaptState), 256);
    return KLPM_OK;
}

extern "C" int kLPM_adapt_init(void *state, size_t state_bytes, const kLPM_adapt_config *cfg, kLPM_stream stream) {
    if (!state || !cfg || ((uintptr_t)state & 7u) || state_bytes < sizeof(AdaptState)) return KLPM_EINVAL;
    if (cfg->n_arms < 1 || cfg->n_arms > KLPM_ADAPT_MAX_ARMS || cfg->window < 1 || cfg->explore > (1ull << 32))
        return KLPM_EINVAL;
    hipLaunchKernelGGL(k_adapt_init, dim3(1), dim3(kWave), 0, (hipStream_t)stream, (AdaptState *)state, *cfg);
    return check_launch();
}

extern "C" int kLPM_adapt_k(void *state, const uint32_t **k_dev) {
    if (!state || !k_dev) return KLPM_EINVAL;
    *k_dev = &((AdaptState *)state)->k;
    return KLPM_OK;
}

extern "C" int kLPM_adapt_observe(void *state, const kLPM_queue *served, const int32_t *batch_idx,
                                  const int32_t *n_selected, int32_t batch_cap, const int64_t *ttft, int32_t n_ttft,
                                  kLPM_stream stream) {
    if (!state || !served || !served->n || served->cap < 0 || batch_cap < 0 || n_ttft < 0 || !n_selected)
        return KLPM_EINVAL;
    if (batch_cap > 0 && (!batch_idx || !ttft || !served->id)) return KLPM_EINVAL;
    hipLaunchKernelGGL(k_adapt_observe, dim3(1), dim3(256), 0, (hipStream_t)stream, (AdaptState *)state, served->id,
                       served->n, served->cap, batch_idx, n_selected, batch_cap, ttft, n_ttft);
    return check_launch();
}

extern "C" int kLPM_adapt_read(void *state, kLPM_adapt_stats *host_out, kLPM_stream stream) {
    if (!state || !host_out) return KLPM_EINVAL;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return KLPM_EHIP;
    AdaptState s;
    if (hipMemcpy(&s, state, sizeof(s), hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    if (s.magic != kAdaptMagic) return KLPM_EINVAL;
    for (int a = 0; a < KLPM_ADAPT_MAX_ARMS; ++a) {
        host_out->count[a] = s.count[a];
        host_out->cost[a] = s.cost[a];
    }
    host_out->pulls = s.pulls;
    host_out->arm = s.arm;
    host_out->k = s.k;
    host_out->steps_in_window = s.steps;
    host_out->device_error = s.error;
    return KLPM_OK;
}
