// k-LPM batch selection (Algorithm 1 of the paper, cut into bins of B as in Sec. 2.1).
//
// Slot j of the batch is an "oldest query" pick when (phase + j) mod k == 0 and a "longest
// prefix-cache hit" pick otherwise.  Both kinds of pick take the first not-yet-picked entry of a
// fixed total order:
//   A = queue sorted by (arrival, index)            -- the oldest-first order
//   L = queue sorted by (-match_len, arrival, index) -- the longest-match order
// so the kernel sorts once (stable LSD radix sort; L is a stable sort of A by match length) and
// then walks the two orders with two cursors.  After the cursors have consumed A[0,ia) and L[0,il)
// the picked set is exactly {rank_A < ia} U {rank_L < il}, which gives an O(1) "already picked"
// test and lets one wavefront resolve a whole k-cycle with two ballots.
#include "klpm_internal.hpp"

namespace klpm {

constexpr int kSortThreads = 256;
constexpr int kSortItems = 8;
constexpr int kSortTile = kSortThreads * kSortItems;          // 2048 keys per block
constexpr int kSortWaveTile = kWave * kSortItems;             // 512 contiguous keys per wave
constexpr int kScanThreads = 1024;

struct SelectWs {
    uint64_t *key_a, *key_b;
    uint32_t *val_a, *val_b, *val_c;
    uint32_t *rank_a, *rank_l;
    uint32_t *hist;
    int32_t *skip;
};

__global__ __launch_bounds__(256) void k_sel_init(const uint64_t *__restrict__ arrival, int32_t n,
                                                  uint64_t *__restrict__ key, uint32_t *__restrict__ val) {
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        key[i] = arrival[i];
        val[i] = (uint32_t)i;
    }
}

// keys for the longest-match order, laid out in oldest-first order so that a stable sort on the
// match length alone yields (-match_len, arrival, index)
__global__ __launch_bounds__(256) void k_sel_lkeys(const uint32_t *__restrict__ order_a,
                                                   const int32_t *__restrict__ match_len, int32_t n,
                                                   uint64_t *__restrict__ key, uint32_t *__restrict__ val) {
    int32_t r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n) {
        uint32_t i = order_a[r];
        int32_t m = match_len[i];
        if (m < 0) m = 0;
        key[r] = (uint64_t)(0x7FFFFFFFu - (uint32_t)m);
        val[r] = i;
    }
}

__global__ __launch_bounds__(256) void k_sel_ranks(const uint32_t *__restrict__ order_a,
                                                   const uint32_t *__restrict__ order_l, int32_t n,
                                                   uint32_t *__restrict__ rank_a, uint32_t *__restrict__ rank_l) {
    int32_t r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n) {
        rank_a[order_a[r]] = (uint32_t)r;
        rank_l[order_l[r]] = (uint32_t)r;
    }
}

// ---- stable LSD radix sort, 8-bit digits: histogram / scan / scatter per pass ----
__global__ __launch_bounds__(kSortThreads) void k_rs_hist(const uint64_t *__restrict__ key, int32_t n, int shift,
                                                          uint32_t *__restrict__ hist, int32_t nblk) {
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    int64_t base = (int64_t)blockIdx.x * kSortTile;
    for (int r = 0; r < kSortItems; ++r) {
        int64_t i = base + r * kSortThreads + threadIdx.x;
        if (i < n) atomicAdd(&h[(uint32_t)(key[i] >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];
}

// exclusive scan of the digit-major table hist[256][nblk]; also flags a pass in which every key
// has the same digit (the scatter then degenerates to a copy)
__global__ __launch_bounds__(kScanThreads) void k_rs_scan(uint32_t *__restrict__ hist, int32_t nblk, int32_t n,
                                                          int32_t *__restrict__ skip) {
    __shared__ uint32_t part[kScanThreads];
    const int tid = threadIdx.x;
    const int64_t total = 256ll * nblk;
    const int64_t chunk = (total + kScanThreads - 1) / kScanThreads;
    const int64_t lo = tid * chunk;
    const int64_t hi = (lo + chunk < total) ? lo + chunk : total;
    uint32_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += hist[i];
    part[tid] = s;
    if (tid == 0) *skip = 0;
    __syncthreads();
    // Hillis-Steele inclusive scan over the 1024 partial sums
    for (int d = 1; d < kScanThreads; d <<= 1) {
        uint32_t v = (tid >= d) ? part[tid - d] : 0u;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    uint32_t run = part[tid] - s;  // exclusive prefix of this thread's chunk
    for (int64_t i = lo; i < hi; ++i) {
        uint32_t c = hist[i];
        hist[i] = run;
        run += c;
    }
    __syncthreads();
    if (tid < 256) {
        uint32_t begin = hist[(int64_t)tid * nblk];
        uint32_t end = (tid == 255) ? (uint32_t)n : hist[(int64_t)(tid + 1) * nblk];
        if (end - begin == (uint32_t)n) *skip = 1;
    }
}

__global__ __launch_bounds__(kSortThreads) void k_rs_scatter(const uint64_t *__restrict__ key_in,
                                                             const uint32_t *__restrict__ val_in,
                                                             uint64_t *__restrict__ key_out,
                                                             uint32_t *__restrict__ val_out, int32_t n, int shift,
                                                             const uint32_t *__restrict__ hist, int32_t nblk,
                                                             const int32_t *__restrict__ skip) {
    __shared__ uint32_t wcount[kSortThreads / kWave][256];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wv = tid / kWave;
    const int64_t wave_base = (int64_t)blockIdx.x * kSortTile + (int64_t)wv * kSortWaveTile;
    if (*skip) {
        for (int r = 0; r < kSortItems; ++r) {
            int64_t i = wave_base + r * kWave + lane;
            if (i < n) {
                key_out[i] = key_in[i];
                val_out[i] = val_in[i];
            }
        }
        return;
    }
    for (int w = 0; w < kSortThreads / kWave; ++w) wcount[w][tid] = 0;
    __syncthreads();
    uint64_t k[kSortItems];
    uint32_t v[kSortItems];
    uint32_t rank[kSortItems];
    for (int r = 0; r < kSortItems; ++r) {
        int64_t i = wave_base + r * kWave + lane;
        bool valid = i < n;
        k[r] = valid ? key_in[i] : ~0ull;
        v[r] = valid ? val_in[i] : 0u;
        uint32_t dg = (uint32_t)(k[r] >> shift) & 255u;
        // lanes of this row holding the same digit
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < 8; ++b) {
            bool bit = (dg >> b) & 1u;
            uint64_t bb = __ballot(bit);
            peers &= bit ? bb : ~bb;
        }
        uint32_t prior = wcount[wv][dg];
        rank[r] = prior + (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        if (valid && (peers & ((1ull << lane) - 1ull)) == 0ull) wcount[wv][dg] = prior + (uint32_t)__popcll(peers);
        // the row's leader has written before the next row's reads are issued (same wave, in order)
    }
    __syncthreads();
    {
        uint32_t run = hist[(int64_t)tid * nblk + blockIdx.x];
        for (int w = 0; w < kSortThreads / kWave; ++w) {
            uint32_t c = wcount[w][tid];
            wcount[w][tid] = run;
            run += c;
        }
    }
    __syncthreads();
    for (int r = 0; r < kSortItems; ++r) {
        int64_t i = wave_base + r * kWave + lane;
        if (i < n) {
            uint32_t dg = (uint32_t)(k[r] >> shift) & 255u;
            uint32_t pos = wcount[wv][dg] + rank[r];
            if (pos < (uint32_t)n) {
                key_out[pos] = k[r];
                val_out[pos] = v[r];
            }
        }
    }
}

// sorts (key, val) by bits [0, 8*passes) of key; result ends in (key_in, val_in) when `passes` is
// even, else in (key_out, val_out). Returns which one through `result_in_first`.
static int radix_sort(uint64_t *k0, uint32_t *v0, uint64_t *k1, uint32_t *v1, int32_t n, int passes, SelectWs &ws,
                      hipStream_t stream, bool *result_in_first) {
    int32_t nblk = (n + kSortTile - 1) / kSortTile;
    uint64_t *ki = k0, *ko = k1;
    uint32_t *vi = v0, *vo = v1;
    for (int p = 0; p < passes; ++p) {
        hipLaunchKernelGGL(k_rs_hist, dim3(nblk), dim3(kSortThreads), 0, stream, ki, n, 8 * p, ws.hist, nblk);
        hipLaunchKernelGGL(k_rs_scan, dim3(1), dim3(kScanThreads), 0, stream, ws.hist, nblk, n, ws.skip);
        hipLaunchKernelGGL(k_rs_scatter, dim3(nblk), dim3(kSortThreads), 0, stream, ki, vi, ko, vo, n, 8 * p,
                           ws.hist, nblk, ws.skip);
        uint64_t *tk = ki; ki = ko; ko = tk;
        uint32_t *tv = vi; vi = vo; vo = tv;
    }
    *result_in_first = (ki == k0);
    return check_launch();
}

// ---- the two-cursor walk over the oldest-first and longest-match orders ----
constexpr int kStage = 4096;  // entries of each order staged in LDS

__global__ __launch_bounds__(kWave) void k_sel_walk(const uint32_t *__restrict__ order_a,
                                                    const uint32_t *__restrict__ order_l,
                                                    const uint32_t *__restrict__ rank_a,
                                                    const uint32_t *__restrict__ rank_l, int32_t n, uint32_t k,
                                                    int32_t batch, uint32_t *__restrict__ phase_inout,
                                                    int32_t *__restrict__ batch_idx,
                                                    int32_t *__restrict__ n_selected) {
    // a_in_l[r] = rank in L of the r-th oldest query, l_in_a[r] = rank in A of the r-th longest match
    __shared__ uint32_t s_a_in_l[kStage];
    __shared__ uint32_t s_l_in_a[kStage];
    const int lane = threadIdx.x;
    const int32_t nb = batch < n ? batch : n;
    const bool lpm_only = (k == 0u || k == 0xFFFFFFFFu);
    const uint32_t phase = lpm_only ? 0u : (*phase_inout % k);
    if (lane == 0) {
        *n_selected = nb;
        *phase_inout = lpm_only ? 0u : (uint32_t)(((uint64_t)phase + (uint64_t)nb) % k);
    }
    if (nb <= 0) return;
    if (lpm_only || k == 1u) {  // a single order: the batch is its first nb entries
        const uint32_t *ord = lpm_only ? order_l : order_a;
        for (int32_t j = lane; j < nb; j += kWave) batch_idx[j] = (int32_t)ord[j];
        return;
    }
    const int32_t staged = nb < kStage ? nb : kStage;  // cursors never pass nb
    for (int32_t r = lane; r < staged; r += kWave) {
        s_a_in_l[r] = rank_l[order_a[r]];
        s_l_in_a[r] = rank_a[order_l[r]];
    }
    __syncthreads();
    int32_t ia = 0, il = 0, j = 0;
    while (j < nb) {
        // number of consecutive slots of the same kind starting at slot j
        uint32_t pos = (uint32_t)(((uint64_t)phase + (uint64_t)j) % k);
        bool oldest = (pos == 0u);
        int32_t want = oldest ? 1 : (int32_t)((k - pos) < (uint32_t)(nb - j) ? (k - pos) : (uint32_t)(nb - j));
        if (want > nb - j) want = nb - j;
        // take `want` unpicked entries from the chosen order, 64 candidates per round
        while (want > 0) {
            int32_t cur = oldest ? ia : il;
            int32_t r = cur + lane;
            bool cand = false;
            if (r < n) {
                uint32_t other = oldest ? (r < staged ? s_a_in_l[r] : rank_l[order_a[r]])
                                        : (r < staged ? s_l_in_a[r] : rank_a[order_l[r]]);
                cand = oldest ? (other >= (uint32_t)il) : (other >= (uint32_t)ia);
            }
            uint64_t mask = __ballot(cand);
            int32_t avail = (int32_t)__popcll(mask);
            int32_t take = avail < want ? avail : want;
            int32_t my = (int32_t)__popcll(mask & ((1ull << lane) - 1ull));
            if (cand && my < take) batch_idx[j + my] = (int32_t)(oldest ? order_a[r] : order_l[r]);
            int32_t adv;
            if (take == avail && take < want) {
                adv = kWave;  // window exhausted, keep looking further along the order
            } else {
                // advance just past the last entry taken: position of the take-th set bit
                uint64_t m2 = mask;
                for (int32_t t = 1; t < take; ++t) m2 &= m2 - 1ull;
                adv = (int32_t)__builtin_ctzll(m2) + 1;
            }
            if (oldest) ia += adv; else il += adv;
            j += take;
            want -= take;
            if ((oldest ? ia : il) >= n && want > 0) { want = 0; j = nb; }  // cannot happen: nb <= n
        }
    }
}

static void carve(SelectWs &ws, char *base, int32_t n, size_t *used) {
    size_t o = 0;
    auto take = [&](size_t bytes) { void *p = base ? base + o : nullptr; o += align_up(bytes, 256); return p; };
    int32_t nblk = (n + kSortTile - 1) / kSortTile;
    if (nblk < 1) nblk = 1;
    size_t nn = (size_t)(n > 0 ? n : 1);
    ws.key_a = (uint64_t *)take(nn * 8);
    ws.key_b = (uint64_t *)take(nn * 8);
    ws.val_a = (uint32_t *)take(nn * 4);
    ws.val_b = (uint32_t *)take(nn * 4);
    ws.val_c = (uint32_t *)take(nn * 4);
    ws.rank_a = (uint32_t *)take(nn * 4);
    ws.rank_l = (uint32_t *)take(nn * 4);
    ws.hist = (uint32_t *)take((size_t)256 * nblk * 4);
    ws.skip = (int32_t *)take(256);
    *used = o;
}

}  // namespace klpm

using namespace klpm;

extern "C" int kLPM_select_workspace_bytes(int32_t n, size_t *out_bytes) {
    if (n < 0 || !out_bytes) return KLPM_EINVAL;
    SelectWs ws;
    carve(ws, nullptr, n, out_bytes);
    return KLPM_OK;
}

extern "C" int kLPM_select(const uint64_t *arrival, const int32_t *match_len, int32_t n, uint32_t k, int32_t batch,
                           uint32_t *phase_inout, int32_t *batch_idx, int32_t *n_selected, void *workspace,
                           size_t workspace_bytes, kLPM_stream stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (n < 0 || batch < 0 || !phase_inout || !n_selected) return KLPM_EINVAL;
    if (n > 0 && (!arrival || !match_len)) return KLPM_EINVAL;
    if (n > 0 && batch > 0 && !batch_idx) return KLPM_EINVAL;
    SelectWs ws;
    size_t need = 0;
    carve(ws, (char *)workspace, n, &need);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return KLPM_EARENA;
    const uint32_t *order_a = ws.val_a, *order_l = ws.val_a;
    if (n > 0 && batch > 0) {
        unsigned g = (unsigned)((n + 255) / 256);
        hipLaunchKernelGGL(k_sel_init, dim3(g), dim3(256), 0, stream, arrival, n, ws.key_a, ws.val_a);
        bool first = true;
        int rc = radix_sort(ws.key_a, ws.val_a, ws.key_b, ws.val_b, n, 8, ws, stream, &first);
        if (rc) return rc;
        order_a = first ? ws.val_a : ws.val_b;  // 8 passes: back in the first buffer
        if (k != 1u) {
            // stable sort of the oldest-first order by descending match length
            uint32_t *spare = first ? ws.val_b : ws.val_a;
            hipLaunchKernelGGL(k_sel_lkeys, dim3(g), dim3(256), 0, stream, order_a, match_len, n, ws.key_a, ws.val_c);
            bool lfirst = true;
            rc = radix_sort(ws.key_a, ws.val_c, ws.key_b, spare, n, 4, ws, stream, &lfirst);
            if (rc) return rc;
            order_l = lfirst ? ws.val_c : spare;
            hipLaunchKernelGGL(k_sel_ranks, dim3(g), dim3(256), 0, stream, order_a, order_l, n, ws.rank_a, ws.rank_l);
        }
    }
    hipLaunchKernelGGL(k_sel_walk, dim3(1), dim3(kWave), 0, stream, order_a, order_l, ws.rank_a, ws.rank_l, n, k,
                       batch, phase_inout, batch_idx, n_selected);
    return check_launch();
}
