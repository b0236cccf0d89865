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
#include <mutex>

#include "klpm_internal.hpp"
#include "lds_sort.hpp"
#include "wave_ops.hpp"

namespace klpm {

constexpr int kSortThreads = 256;
constexpr int kSortItems = 8;
constexpr int kSortTile = kSortThreads * kSortItems;          // 2048 keys per block
constexpr int kSortWaveTile = kWave * kSortItems;             // 512 contiguous keys per wave
constexpr int kScanThreads = 1024;

// The queue length as the kernels get it: the host-side count (which sizes the launches) and the
// optional device-side count that cuts it down.
struct LiveN {
    int32_t n;
    const int32_t *live;
    __device__ __forceinline__ int32_t get() const { return live_count(n, live); }
};

struct SelectWs {
    uint64_t *key_a, *key_b;
    uint32_t *val_a, *val_b, *val_c;
    uint32_t *rank_a, *rank_l;
    uint32_t *hist;
    int32_t *skip;
    int32_t *viol;
};

__global__ __launch_bounds__(256) void k_sel_init(const uint64_t *__restrict__ arrival, LiveN nn,
                                                  uint64_t *__restrict__ key, uint32_t *__restrict__ val) {
    const int32_t n = nn.get();
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        key[i] = arrival[i];
        val[i] = (uint32_t)i;
    }
}

// keys for the longest-match order, laid out in oldest-first order so that a stable sort on the
// match length alone yields (-match_len, arrival, index)
// (with tie keys: (-match_len, tie key, arrival, index); the tie key goes below the inverted length)
__global__ __launch_bounds__(256) void k_sel_lkeys(const uint32_t *__restrict__ order_a,
                                                   const int32_t *__restrict__ match_len,
                                                   const uint32_t *__restrict__ tie_key, LiveN nn,
                                                   uint64_t *__restrict__ key, uint32_t *__restrict__ val) {
    const int32_t n = nn.get();
    int32_t r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n) {
        uint32_t i = order_a[r];
        int32_t m = match_len[i];
        if (m < 0) m = 0;
        uint64_t inv = (uint64_t)(0x7FFFFFFFu - (uint32_t)m);
        key[r] = tie_key ? ((inv << 32) | (uint64_t)tie_key[i]) : inv;
        val[r] = i;
    }
}

__global__ void k_sel_zero_flag(int32_t *__restrict__ viol) {
    if (threadIdx.x < 2) viol[threadIdx.x] = 0;
}
__global__ __launch_bounds__(256) void k_sel_rank_l(const uint32_t *__restrict__ order_l, LiveN nn,
                                                    uint32_t *__restrict__ rank_l) {
    const int32_t n = nn.get();
    const int32_t r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n) rank_l[order_l[r]] = (uint32_t)r;
}
// A queue promised to be in arrival order: the oldest-first order is the index order, and the keys of
// the longest-match order, max_score - score, are laid out in it.  The promise and the bound are checked.
__global__ __launch_bounds__(256) void k_sel_fifo_keys(const uint64_t *__restrict__ arrival,
                                                       const int32_t *__restrict__ score, LiveN nn, int32_t max_score,
                                                       uint64_t *__restrict__ key, uint32_t *__restrict__ val,
                                                       uint32_t *__restrict__ order_a, uint32_t *__restrict__ rank_a,
                                                       int32_t *__restrict__ viol) {
    const int32_t n = nn.get();
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int32_t m = score[i];
    if (m < 0) m = 0;
    const bool bad = m > max_score || (i + 1 < n && arrival[i] > arrival[i + 1]);
    key[i] = (uint64_t)(uint32_t)(max_score - (bad ? max_score : m));
    val[i] = (uint32_t)i;
    order_a[i] = (uint32_t)i;
    rank_a[i] = (uint32_t)i;
    if (bad) viol[1] = 1;
}

__global__ __launch_bounds__(256) void k_sel_ranks(const uint32_t *__restrict__ order_a,
                                                   const uint32_t *__restrict__ order_l, LiveN nn,
                                                   uint32_t *__restrict__ rank_a, uint32_t *__restrict__ rank_l) {
    const int32_t n = nn.get();
    int32_t r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n) {
        rank_a[order_a[r]] = (uint32_t)r;
        rank_l[order_l[r]] = (uint32_t)r;
    }
}

// ---- both orders of a short queue in one workgroup ----
// Up to kSmallOrdersN entries: two sorts in LDS on two-word keys, (arrival, index) for the
// oldest-first order and (inverted score | tie key, oldest-first rank) for the longest-match order,
// instead of the ~40 launches of the radix sorts below.
constexpr int kSmallOrdersN = 4096;
constexpr int kSmallOrdersThreads = 1024;

__device__ __forceinline__ void sort_pairs(uint64_t *hi, uint32_t *lo, int32_t np2, int tid) {
    sort_lds<kSmallOrdersThreads, kSmallOrdersN / kSmallOrdersThreads, true>(hi, lo, np2, tid);
}

__global__ __launch_bounds__(kSmallOrdersThreads) void k_orders_small(const uint64_t *__restrict__ arrival,
                                                                      const int32_t *__restrict__ score,
                                                                      const uint32_t *__restrict__ tie_key, LiveN nn,
                                                                      int want_l, uint32_t *__restrict__ order_a,
                                                                      uint32_t *__restrict__ order_l,
                                                                      uint32_t *__restrict__ rank_a,
                                                                      uint32_t *__restrict__ rank_l) {
    __shared__ uint64_t hi[kSmallOrdersN];
    __shared__ uint32_t lo[kSmallOrdersN];
    __shared__ uint32_t oa[kSmallOrdersN];
    int32_t n = nn.get();
    n = n < kSmallOrdersN ? n : kSmallOrdersN;
    const int tid = threadIdx.x;
    int32_t np2 = 1;
    while (np2 < n) np2 <<= 1;
    for (int32_t i = tid; i < np2; i += kSmallOrdersThreads) {
        hi[i] = i < n ? arrival[i] : ~0ull;
        lo[i] = i < n ? (uint32_t)i : 0xFFFFFFFFu;
    }
    __syncthreads();
    sort_pairs(hi, lo, np2, tid);
    for (int32_t r = tid; r < n; r += kSmallOrdersThreads) {
        const uint32_t i = lo[r];
        oa[r] = i;
        order_a[r] = i;
        rank_a[i] = (uint32_t)r;
    }
    if (!want_l) return;
    __syncthreads();
    // longest-match keys in oldest-first order; the second word (that rank) settles equal keys by
    // arrival, then index
    for (int32_t r = tid; r < np2; r += kSmallOrdersThreads) {
        uint64_t key = ~0ull;
        if (r < n) {
            const uint32_t i = oa[r];
            int32_t m = score[i];
            if (m < 0) m = 0;
            const uint64_t inv = (uint64_t)(0x7FFFFFFFu - (uint32_t)m);
            key = tie_key ? ((inv << 32) | (uint64_t)tie_key[i]) : inv;
        }
        hi[r] = key;
        lo[r] = r < n ? (uint32_t)r : 0xFFFFFFFFu;
    }
    __syncthreads();
    sort_pairs(hi, lo, np2, tid);
    for (int32_t p = tid; p < n; p += kSmallOrdersThreads) {
        const uint32_t i = oa[lo[p]];
        order_l[p] = i;
        rank_l[i] = (uint32_t)p;
    }
}

// ---- stable LSD radix sort, 8-bit digits: histogram / scan / scatter per pass ----
__global__ __launch_bounds__(kSortThreads) void k_rs_hist(const uint64_t *__restrict__ key, LiveN nn, int shift,
                                                          uint32_t *__restrict__ hist, int32_t nblk) {
    const int32_t n = nn.get();
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
__global__ __launch_bounds__(kScanThreads) void k_rs_scan(uint32_t *__restrict__ hist, int32_t nblk, LiveN nn,
                                                          int32_t *__restrict__ skip) {
    const int32_t n = nn.get();
    __shared__ uint32_t part[kScanThreads / kWave];
    const int tid = threadIdx.x;
    const int64_t total = 256ll * nblk;
    const int64_t chunk = (total + kScanThreads - 1) / kScanThreads;
    const int64_t lo = tid * chunk;
    const int64_t hi = (lo + chunk < total) ? lo + chunk : total;
    // (counts are read eight at a time, all requested before any is added up: a loop that uses each
    // value at once pays a memory round trip per entry; the first eight are kept for the second sweep)
    constexpr int kU = 8;
    uint32_t head[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) head[u] = lo + u < hi ? hist[lo + u] : 0u;
    uint32_t s = 0;
#pragma unroll
    for (int u = 0; u < kU; ++u) s += head[u];
    for (int64_t i0 = lo + kU; i0 < hi; i0 += kU) {
        uint32_t v[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) v[u] = i0 + u < hi ? hist[i0 + u] : 0u;
#pragma unroll
        for (int u = 0; u < kU; ++u) s += v[u];
    }
    if (tid == 0) *skip = 0;
    uint32_t all;
    const uint32_t incl = block_inclusive_scan<uint32_t, kScanThreads>(s, part, tid, all);
    uint32_t run = incl - s;  // exclusive prefix of this thread's chunk
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        if (lo + u < hi) hist[lo + u] = run;
        run += head[u];
    }
    for (int64_t i0 = lo + kU; i0 < hi; i0 += kU) {
        uint32_t v[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) v[u] = i0 + u < hi ? hist[i0 + u] : 0u;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (i0 + u < hi) hist[i0 + u] = run;
            run += v[u];
        }
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
                                                             uint32_t *__restrict__ val_out, LiveN nn, int shift,
                                                             const uint32_t *__restrict__ hist, int32_t nblk,
                                                             const int32_t *__restrict__ skip) {
    const int32_t n = nn.get();
    __shared__ uint32_t wcount[kSortThreads / kWave][256];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wv = tid / kWave;
    const int64_t wave_base = (int64_t)blockIdx.x * kSortTile + (int64_t)wv * kSortWaveTile;
    // everything this thread reads is requested up front, together with the skip flag
    const int32_t skip_pass = *skip;
    const uint32_t run0 = hist[(int64_t)tid * nblk + blockIdx.x];
    uint64_t k[kSortItems];
    uint32_t v[kSortItems];
    uint32_t rank[kSortItems];
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        int64_t i = wave_base + r * kWave + lane;
        bool valid = i < n;
        k[r] = valid ? key_in[i] : ~0ull;
        v[r] = valid ? val_in[i] : 0u;
    }
    if (skip_pass) {
#pragma unroll
        for (int r = 0; r < kSortItems; ++r) {
            int64_t i = wave_base + r * kWave + lane;
            if (i < n) {
                key_out[i] = k[r];
                val_out[i] = v[r];
            }
        }
        return;
    }
    for (int w = 0; w < kSortThreads / kWave; ++w) wcount[w][tid] = 0;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        int64_t i = wave_base + r * kWave + lane;
        bool valid = i < n;
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
        uint32_t run = run0;
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
static int radix_sort(uint64_t *k0, uint32_t *v0, uint64_t *k1, uint32_t *v1, LiveN nn, int passes, SelectWs &ws,
                      hipStream_t stream, bool *result_in_first) {
    const LiveN n = nn;
    int32_t nblk = (nn.n + kSortTile - 1) / kSortTile;
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
// Acc gives, for a position r < n_valid of either order: the queue index stored there
// (a_elem / l_elem) and the position of that same query in the other order (a_in_l / l_in_a; any
// value >= nb stands for "not among the first nb of the other order").  One wavefront runs it.
template <class Acc>
struct TwoCursorWalk {
    // Each order is looked at through a window of 64 consecutive entries held in registers (lane =
    // entry); a window is read again once the cursor has moved kReload entries into it, so a pick
    // costs ballots and scalar arithmetic, not a round trip to LDS or memory.
    static constexpr int32_t kReload = 16;
    const Acc &acc;
    const int32_t n_valid, nb;
    const uint32_t k, km1;
    int32_t *__restrict__ const batch_idx;
    const int lane;
    const uint64_t below;
    int32_t ia = 0, il = 0, j = 0;
    int32_t wa = -kWave, wl = -kWave;  // first entry of each window (a load is due at the start)
    uint32_t a_oth = 0, a_elv = 0, l_oth = 0, l_elv = 0;
    bool a_ok = false, l_ok = false;

    __device__ __forceinline__ TwoCursorWalk(const Acc &acc_, int32_t n_valid_, int32_t nb_, uint32_t k_,
                                             int32_t *__restrict__ batch_idx_, int lane_)
        : acc(acc_), n_valid(n_valid_), nb(nb_), k(k_), km1(k_ - 1u), batch_idx(batch_idx_), lane(lane_),
          below((1ull << lane_) - 1ull) {}

    __device__ __forceinline__ void reload() {
        if (ia - wa >= kReload) {
            wa = ia;
            a_ok = wa + lane < n_valid;
            a_oth = a_ok ? acc.a_in_l(wa + lane) : 0u;
            a_elv = a_ok ? acc.a_elem(wa + lane) : 0u;
        }
        if (il - wl >= kReload) {
            wl = il;
            l_ok = wl + lane < n_valid;
            l_oth = l_ok ? acc.l_in_a(wl + lane) : 0u;
            l_elv = l_ok ? acc.l_elem(wl + lane) : 0u;
        }
    }
    // after consuming A[0,ia) and L[0,il) the picked set is {pos_A < ia} U {pos_L < il}
    __device__ __forceinline__ bool cand_a() const { return a_ok && wa + lane >= ia && a_oth >= (uint32_t)il; }
    __device__ __forceinline__ bool cand_l(int32_t ia_now) const {
        return l_ok && wl + lane >= il && l_oth >= (uint32_t)ia_now;
    }

    // Several whole cycles at once (at the start of a cycle, nb - j >= k, k - 1 <= 64), as many as
    // the two orders do not interfere inside the windows.  Returns the number of cycles taken.
    __device__ __forceinline__ int32_t bulk() {
        const bool ca = cand_a(), cl = cand_l(ia);
        const uint64_t mask_a = __ballot(ca), mask_l = __ballot(cl);
        const int32_t my_a = (int32_t)__popcll(mask_a & below), my_l = (int32_t)__popcll(mask_l & below);
        const int32_t n_a = (int32_t)__popcll(mask_a), n_l = (int32_t)__popcll(mask_l);
        int32_t c = n_a;
        if ((int32_t)((uint32_t)n_l / km1) < c) c = (int32_t)((uint32_t)n_l / km1);
        if ((int32_t)((uint32_t)(nb - j) / k) < c) c = (int32_t)((uint32_t)(nb - j) / k);
        if (c <= 0) return 0;
        {
            // an oldest pick that also lies in the consumed stretch of the longest-match order (or the
            // other way round) makes the two streams interact: only the cycles before the first such
            // pick are taken at once (a shorter stretch cannot create new clashes)
            const int32_t take_l = c * (int32_t)km1;
            const int32_t ia_end = wa + (int32_t)__builtin_ctzll(__ballot(ca && my_a == c - 1)) + 1;
            const int32_t il_end = wl + (int32_t)__builtin_ctzll(__ballot(cl && my_l == take_l - 1)) + 1;
            const uint64_t clash_a = __ballot(ca && my_a < c && a_oth < (uint32_t)il_end);
            const uint64_t clash_l = __ballot(cl && my_l < take_l && l_oth < (uint32_t)ia_end);
            if (clash_a) {
                const int32_t before = (int32_t)__popcll(mask_a & ((1ull << __builtin_ctzll(clash_a)) - 1ull));
                c = before < c ? before : c;
            }
            if (clash_l) {
                const int32_t before = (int32_t)((uint32_t)__popcll(mask_l & ((1ull << __builtin_ctzll(clash_l)) - 1ull)) / km1);
                c = before < c ? before : c;
            }
        }
        if (c <= 0) return 0;
        const int32_t take_l = c * (int32_t)km1;
        if (ca && my_a < c) batch_idx[j + my_a * (int32_t)k] = (int32_t)a_elv;
        if (cl && my_l < take_l) {
            const uint32_t cyc = (uint32_t)my_l / km1;
            const uint32_t within = (uint32_t)my_l - cyc * km1;
            batch_idx[j + (int32_t)(cyc * k + 1u + within)] = (int32_t)l_elv;
        }
        ia = wa + (int32_t)__builtin_ctzll(__ballot(ca && my_a == c - 1)) + 1;
        il = wl + (int32_t)__builtin_ctzll(__ballot(cl && my_l == take_l - 1)) + 1;
        j += c * (int32_t)k;
        return c;
    }

    // One whole cycle in straight-line code (same preconditions): the oldest pick, then the k-1
    // longest-match picks among what is left.  False when a window does not hold all of it.
    __device__ __forceinline__ bool cycle() {
        const uint64_t mask_a = __ballot(cand_a());
        if (!mask_a) return false;
        const int fa = (int)__builtin_ctzll(mask_a);
        const int32_t ia_next = wa + fa + 1;
        const bool cl = cand_l(ia_next);
        const uint64_t mask_l = __ballot(cl);
        if ((uint32_t)__popcll(mask_l) < km1) return false;
        const int32_t my_l = (int32_t)__popcll(mask_l & below);
        if (lane == fa) batch_idx[j] = (int32_t)a_elv;
        if (cl && my_l < (int32_t)km1) batch_idx[j + 1 + my_l] = (int32_t)l_elv;
        il = wl + (int32_t)__builtin_ctzll(__ballot(cl && my_l == (int32_t)km1 - 1)) + 1;
        ia = ia_next;
        j += (int32_t)k;
        return true;
    }

    // One run at cycle position pos: a single oldest pick, or the longest-match picks up to the next
    // oldest pick, as far as the window reaches.  Returns the picks made.
    __device__ __forceinline__ int32_t run(uint32_t pos) {
        const bool oldest = (pos == 0u);
        const uint32_t len = oldest ? 1u : (k - pos);
        const int32_t want = (int32_t)(len < (uint32_t)(nb - j) ? len : (uint32_t)(nb - j));
        const bool cand = oldest ? cand_a() : cand_l(ia);
        const uint64_t mask = __ballot(cand);
        const int32_t my = (int32_t)__popcll(mask & below);
        const int32_t avail = (int32_t)__popcll(mask);
        const int32_t take = avail < want ? avail : want;
        if (cand && my < take) batch_idx[j + my] = (int32_t)(oldest ? a_elv : l_elv);
        int32_t next = (oldest ? wa : wl) + kWave;  // window exhausted: go on behind it
        if (take == want) next = (oldest ? wa : wl) + (int32_t)__builtin_ctzll(__ballot(cand && my == take - 1)) + 1;
        if (oldest) ia = next; else il = next;
        j += take;
        if (take < want && next >= n_valid) j = nb;  // unreachable while nb <= n_valid
        return take;
    }
};

template <class Acc>
__device__ __forceinline__ void two_cursor_walk(const Acc &acc, int32_t n_valid, int32_t nb, uint32_t k, uint32_t phase,
                                                int32_t *__restrict__ batch_idx, int lane) {
    if (k == 1u) {  // oldest picks only: the first nb entries of that order
        for (int32_t t = lane; t < nb; t += kWave) batch_idx[t] = (int32_t)acc.a_elem(t);
        return;
    }
    TwoCursorWalk<Acc> w(acc, n_valid, nb, k, batch_idx, lane);
    uint32_t pos = phase;  // (phase + j) mod k, kept incrementally; phase < k on entry
    int burst = 1;
    while (w.j < nb) {
        if (pos == 0u && w.km1 <= (uint32_t)kWave) {
            // whole cycles: in bulk while that works; after an attempt that found a clash at once, a
            // few cycles one by one (clashes come in stretches, e.g. when most of the queue is
            // admitted, and a failed attempt costs as much as a cycle), then in bulk again
            const int32_t j0 = w.j;
            while ((uint32_t)(nb - w.j) >= k) {
                w.reload();
                if (w.bulk() == 0) break;
                burst = 1;
            }
            for (int t = 0; t < burst && (uint32_t)(nb - w.j) >= k; ++t) {
                w.reload();
                if (!w.cycle()) break;
            }
            burst = burst < 16 ? 2 * burst : 16;  // an isolated clash costs one single cycle, a stretch 1, 2, 4, 8, 16, 16 ...
            if (w.j != j0) continue;
        }
        w.reload();
        pos += (uint32_t)w.run(pos);
        if (pos >= k) pos -= k;
    }
}

// ---- the same walk by a whole workgroup ----
// Slot j of the batch is an oldest-first slot iff (phase + j) mod k = 0.  Were no query within reach of
// both cursors, the t-th oldest-first slot would take A[t] and the u-th longest-match slot L[u], all
// at once.  A query that both cursors can reach (a "dual": position i in A and p in L, both inside the
// stretches the cursors can cover) goes to whichever cursor arrives first and is stepped over by the
// other; every position behind a stepped-over one moves one slot forward.  Duals are few when the queue
// is much longer than the batch, and their fates are settled one by one in order of time: with the fates
// settled so far, a dual's arrival times are upper bounds (more may still be stepped over before it),
// and the earliest of all those bounds is exact - everything stepped over before that moment is already
// settled.  More than 64 duals: the one-wavefront walk does the batch instead.
struct WalkSlots {
    uint32_t k, km1, r0;  // r0: the first oldest-first slot
    __device__ __forceinline__ uint64_t slot_a(uint32_t t) const { return (uint64_t)r0 + (uint64_t)t * k; }
    __device__ __forceinline__ uint64_t slot_l(uint32_t u) const {
        if (u < r0) return u;
        const uint32_t v = u - r0;
        const uint32_t c = v / km1;
        return (uint64_t)r0 + (uint64_t)c * k + 1u + (uint64_t)(v - c * km1);
    }
};

constexpr int kWalkDuals = 64;
constexpr int kWalkScratch = 8 + 4 * kWalkDuals;  // words of LDS the workgroup walk needs

// Every thread of the workgroup calls it (behind a barrier after the writes acc reads); same arguments
// and result as two_cursor_walk.
template <class Acc, int THREADS>
__device__ __forceinline__ void two_cursor_block(const Acc &acc, int32_t n_valid, int32_t nb, uint32_t k, uint32_t phase,
                                                 int32_t *__restrict__ batch_idx, int tid, int32_t *s_w) {
    if (k == 1u) {
        for (int32_t t = tid; t < nb; t += THREADS) batch_idx[t] = (int32_t)acc.a_elem(t);
        return;
    }
    const int lane = tid & (kWave - 1);
    const WalkSlots ws{k, k - 1u, (k - phase) % k};
    const int32_t cnt_a = (uint32_t)nb > ws.r0 ? (int32_t)(((uint64_t)((uint32_t)nb - ws.r0) + k - 1u) / k) : 0;
    const int32_t cnt_l = nb - cnt_a;
    int32_t *du_i = s_w + 8, *du_p = du_i + kWalkDuals, *skip_a = du_p + kWalkDuals, *skip_l = skip_a + kWalkDuals;
    if (tid < 8) s_w[tid] = 0;
    __syncthreads();
    // queries among the first nb of both orders
    int32_t mine = 0;
    for (int32_t i = tid; i < nb; i += THREADS) mine += acc.a_in_l(i) < (uint32_t)nb ? 1 : 0;
    mine = wave_sum(mine);
    if (lane == 0 && mine) atomicAdd(&s_w[0], mine);
    __syncthreads();
    const int32_t n_dual = s_w[0];
    // ... and inside the stretch either cursor can cover (its slots plus what it may step over)
    for (int32_t i = tid; i < nb; i += THREADS) {
        const uint32_t p = acc.a_in_l(i);
        if (p < (uint32_t)nb && i < cnt_a + n_dual && (int32_t)p < cnt_l + n_dual) {
            const int32_t at = atomicAdd(&s_w[1], 1);
            if (at < kWalkDuals) {
                du_i[at] = i;
                du_p[at] = (int32_t)p;
            }
        }
    }
    __syncthreads();
    const int32_t n_both = s_w[1];
    if (n_both > kWalkDuals) {
        if (tid < kWave) two_cursor_walk(acc, n_valid, nb, k, phase, batch_idx, tid);
        return;
    }
    if (n_both > 0 && tid < kWave) {
        const int32_t di = lane < n_both ? du_i[lane] : 0, dp = lane < n_both ? du_p[lane] : 0;
        uint64_t i_less = 0, p_less = 0;
        for (int r = 0; r < n_both; ++r) {
            const int32_t oi = __shfl(di, r), op = __shfl(dp, r);
            if (oi < di) i_less |= 1ull << r;
            if (op < dp) p_less |= 1ull << r;
        }
        uint64_t und = n_both == 64 ? ~0ull : ((1ull << n_both) - 1ull), to_a = 0, to_l = 0;
        while (und) {
            const uint32_t st_a = (uint32_t)__popcll(to_l & i_less), st_l = (uint32_t)__popcll(to_a & p_less);
            const uint64_t ta = ws.slot_a((uint32_t)di - st_a), tl = ws.slot_l((uint32_t)dp - st_l);
            const uint64_t t64 = ta < tl ? ta : tl;
            const uint32_t t = ((und >> lane) & 1ull) ? (t64 < 0xFFFFFFFFull ? (uint32_t)t64 : 0xFFFFFFFFu) : 0xFFFFFFFFu;
            uint32_t tmin = t;
#pragma unroll
            for (int d = 32; d > 0; d >>= 1) {
                const uint32_t o = (uint32_t)__shfl_xor((int)tmin, d);
                tmin = o < tmin ? o : tmin;
            }
            if (tmin >= (uint32_t)nb) break;  // nobody else is reached inside the batch
            const int who = (int)__builtin_ctzll(__ballot(t == tmin));
            if (__shfl((int)(ta < tl), who)) to_a |= 1ull << who; else to_l |= 1ull << who;
            und &= ~(1ull << who);
        }
        const uint64_t below = (1ull << lane) - 1ull;
        if ((to_l >> lane) & 1ull) skip_a[__popcll(to_l & below)] = di;
        if ((to_a >> lane) & 1ull) skip_l[__popcll(to_a & below)] = dp;
        if (lane == 0) {
            s_w[2] = (int32_t)__popcll(to_l);
            s_w[3] = (int32_t)__popcll(to_a);
        }
    }
    __syncthreads();
    const int32_t n_sa = s_w[2], n_sl = s_w[3];
    for (int32_t r = tid; r < nb; r += THREADS) {
        if (r < cnt_a + n_sa) {
            int32_t before = 0;
            bool skipped = false;
            for (int q = 0; q < n_sa; ++q) {
                const int32_t v = skip_a[q];
                before += v < r ? 1 : 0;
                skipped |= v == r;
            }
            const uint64_t slot = ws.slot_a((uint32_t)(r - before));
            if (!skipped && slot < (uint64_t)nb) batch_idx[slot] = (int32_t)acc.a_elem(r);
        }
        if (r < cnt_l + n_sl) {
            int32_t before = 0;
            bool skipped = false;
            for (int q = 0; q < n_sl; ++q) {
                const int32_t v = skip_l[q];
                before += v < r ? 1 : 0;
                skipped |= v == r;
            }
            const uint64_t slot = ws.slot_l((uint32_t)(r - before));
            if (!skipped && slot < (uint64_t)nb) batch_idx[slot] = (int32_t)acc.l_elem(r);
        }
    }
}

constexpr int kStage = 4096;  // entries of each order staged in LDS

struct StagedAcc {
    const uint32_t *order_a, *order_l, *rank_a, *rank_l;  // global
    const uint32_t *s_a_elem, *s_l_elem, *s_a_in_l, *s_l_in_a;  // LDS copies of the first `staged` entries
    int32_t staged;
    __device__ __forceinline__ uint32_t a_elem(int32_t r) const { return r < staged ? s_a_elem[r] : order_a[r]; }
    __device__ __forceinline__ uint32_t l_elem(int32_t r) const { return r < staged ? s_l_elem[r] : order_l[r]; }
    __device__ __forceinline__ uint32_t a_in_l(int32_t r) const { return r < staged ? s_a_in_l[r] : rank_l[order_a[r]]; }
    __device__ __forceinline__ uint32_t l_in_a(int32_t r) const { return r < staged ? s_l_in_a[r] : rank_a[order_l[r]]; }
};

__global__ __launch_bounds__(256) void k_sel_walk(const uint32_t *__restrict__ order_a,
                                                  const uint32_t *__restrict__ order_l,
                                                  const uint32_t *__restrict__ rank_a,
                                                  const uint32_t *__restrict__ rank_l, LiveN nn, KArg ka,
                                                  int32_t batch, uint32_t *__restrict__ phase_inout,
                                                  int32_t *__restrict__ batch_idx,
                                                  int32_t *__restrict__ n_selected) {
    const int32_t n = nn.get();
    const uint32_t k = ka.get();
    __shared__ uint32_t s_a_elem[kStage], s_l_elem[kStage], s_a_in_l[kStage], s_l_in_a[kStage];
    const int tid = threadIdx.x;
    const int32_t nb = batch < n ? batch : n;
    const bool lpm_only = (k == 0u || k == 0xFFFFFFFFu);
    const uint32_t phase = lpm_only ? 0u : (*phase_inout % k);
    __syncthreads();  // every thread has read the phase before it is rewritten
    if (tid == 0) {
        *n_selected = nb;
        *phase_inout = lpm_only ? 0u : (uint32_t)(((uint64_t)phase + (uint64_t)nb) % k);
    }
    if (nb <= 0) return;
    if (lpm_only || k == 1u) {  // a single order: the batch is its first nb entries
        const uint32_t *ord = lpm_only ? order_l : order_a;
        for (int32_t j = tid; j < nb; j += blockDim.x) batch_idx[j] = (int32_t)ord[j];
        return;
    }
    const int32_t staged = nb < kStage ? nb : kStage;  // the cursors never pass nb
    for (int32_t r = tid; r < staged; r += blockDim.x) {
        uint32_t ea = order_a[r], el = order_l[r];
        s_a_elem[r] = ea;
        s_l_elem[r] = el;
        s_a_in_l[r] = rank_l[ea];
        s_l_in_a[r] = rank_a[el];
    }
    __syncthreads();
    if (tid >= kWave) return;
    StagedAcc acc{order_a, order_l, rank_a, rank_l, s_a_elem, s_l_elem, s_a_in_l, s_l_in_a, staged};
    two_cursor_walk(acc, n, nb, k, phase, batch_idx, tid);
}

// ---- single-kernel selection for a queue kept in arrival order ----
// When arrival[] is non-decreasing in the queue index, the oldest-first order is the index order
// and the longest-match order is (-match_len, index).  One workgroup then finds the nb-th largest
// match length by a few histogram sweeps over match_len, gathers the nb winners of the
// longest-match order, sorts them in LDS and runs the two-cursor walk, all in one launch.
constexpr int kFifoThreads = 1024;
constexpr int kFqSingleBlockN = 8192;  // queues up to this length take the single-workgroup kernel (longer ones: the kernels further down)
constexpr int kFifoMaxBatch = 4096;
constexpr int kFifoBins = 2048;

struct FifoAcc {
    const uint32_t *l_elem_, *a_in_l_;
    __device__ __forceinline__ uint32_t a_elem(int32_t r) const { return (uint32_t)r; }
    __device__ __forceinline__ uint32_t l_elem(int32_t r) const { return l_elem_[r]; }
    __device__ __forceinline__ uint32_t a_in_l(int32_t r) const { return a_in_l_[r]; }
    __device__ __forceinline__ uint32_t l_in_a(int32_t r) const { return l_elem_[r]; }
};

__global__ __launch_bounds__(kFifoThreads) void k_select_fifo(const uint64_t *__restrict__ arrival,
                                                               const int32_t *__restrict__ match_len, LiveN nn,
                                                               KArg ka, int32_t batch,
                                                               uint32_t *__restrict__ phase_inout,
                                                               int32_t *__restrict__ batch_idx,
                                                               int32_t *__restrict__ n_selected) {
    const int32_t n = nn.get();
    const uint32_t k = ka.get();
    __shared__ uint32_t hist[kFifoBins];
    __shared__ uint64_t cand[kFifoMaxBatch];
    __shared__ uint32_t l_elem[kFifoMaxBatch];
    __shared__ uint32_t a_in_l[kFifoMaxBatch];
    __shared__ int32_t s_walk[kWalkScratch];
    __shared__ int32_t sbuf[kFifoThreads];
    __shared__ int32_t s_flag, s_max, s_bin, s_above, s_count;
    const int tid = threadIdx.x;
    const int32_t nb = batch < n ? batch : n;
    const bool lpm_only = (k == 0u || k == 0xFFFFFFFFu);
    const uint32_t phase = lpm_only ? 0u : (*phase_inout % k);
    if (tid == 0) { s_flag = 0; s_max = 0; s_count = 0; }
    __syncthreads();
    if (nb <= 0) {
        if (tid == 0) { *n_selected = 0; *phase_inout = phase; }
        return;
    }
    // The queue (at most kFqSingleBlockN entries) is read once: every thread keeps kOwn consecutive
    // entries' match lengths in registers for the whole kernel (index order = thread order), so that
    // everything behind this round trip runs on registers and LDS.  Arrival order check and the
    // largest match length come with it.
    constexpr int kOwn = kFqSingleBlockN / kFifoThreads;
    int32_t mv[kOwn];
    {
        uint64_t t[kOwn + 1];
        const int32_t first = tid * kOwn;
#pragma unroll
        for (int r = 0; r < kOwn; ++r) {
            const int32_t i = first + r;
            const int32_t ic = i < n ? i : n - 1;
            mv[r] = match_len[ic];
            t[r] = arrival[ic];
        }
        t[kOwn] = arrival[first + kOwn < n ? first + kOwn : n - 1];
        int32_t mx = 0;
        bool viol = false;
#pragma unroll
        for (int r = 0; r < kOwn; ++r) {
            mv[r] = (first + r < n) ? (mv[r] < 0 ? 0 : mv[r]) : -1;  // (-1: no entry)
            mx = mv[r] > mx ? mv[r] : mx;
            viol |= first + r + 1 < n && t[r] > t[r + 1];
        }
        if (viol) atomicOr(&s_flag, 1);
        mx = wave_max(mx);
        if ((tid & (kWave - 1)) == 0) atomicMax(&s_max, mx);
    }
    __syncthreads();
    if (s_flag) {  // the caller's promise does not hold: select nothing, say so
        if (tid == 0) *n_selected = -1;
        return;
    }
    if (tid == 0) {
        *n_selected = nb;
        *phase_inout = lpm_only ? 0u : (uint32_t)(((uint64_t)phase + (uint64_t)nb) % k);
    }
    if (k == 1u) {  // FCFS on an arrival-ordered queue: its first nb entries
        for (int32_t j = tid; j < nb; j += kFifoThreads) batch_idx[j] = j;
        return;
    }
    if (nb == 1) {
        // one query per step (Def. 2 as it stands): the head of the queue, or the first query that
        // holds the largest match length found above
        if (!lpm_only && phase == 0u) {
            if (tid == 0) batch_idx[0] = 0;
            return;
        }
        if (tid == 0) s_bin = n;
        __syncthreads();
        const int32_t best = s_max;
        int32_t first = n;
#pragma unroll
        for (int r = kOwn - 1; r >= 0; --r)
            if (mv[r] == best) first = tid * kOwn + r;
        if (first < n) atomicMin(&s_bin, first);
        __syncthreads();
        if (tid == 0) batch_idx[0] = s_bin;
        return;
    }
    // the entries that can be picked: all of a short queue of which a good part is admitted (sorting
    // them all is then cheaper than the threshold search), else the nb best by match length
    int32_t n_cand = nb;
    if (n <= kFifoMaxBatch && ((int64_t)nb * 8 >= n || n <= 256)) {
        n_cand = n;
#pragma unroll
        for (int r = 0; r < kOwn; ++r) {
            const int32_t i = tid * kOwn + r;
            if (mv[r] >= 0) cand[i] = ((uint64_t)(0x7FFFFFFFu - (uint32_t)mv[r]) << 32) | (uint64_t)(uint32_t)i;
        }
    } else {
        // the nb-th largest match length m*, found digit by digit (11 bits per pass over the registers)
        int mbits = 0;
        while (mbits < 31 && (s_max >> mbits) != 0) ++mbits;
        int32_t fixed_hi = 0;      // value of the bits above `shift` already decided
        int32_t need = nb;         // winners still to be found among elements matching fixed_hi
        int shift = mbits;         // bits [shift, mbits) are decided
        while (shift > 0) {
            const int width = shift < 11 ? shift : 11;
            const int nshift = shift - width;
            for (int i = tid; i < kFifoBins; i += kFifoThreads) hist[i] = 0;
            __syncthreads();
#pragma unroll
            for (int r = 0; r < kOwn; ++r) {
                const int32_t m = mv[r];
                const bool in = m >= 0 && (m >> shift) == fixed_hi;
                const int32_t bin = (m >> nshift) & ((1 << width) - 1);
                // lanes that share the first active lane's bin are added once (scores cluster and same-address
                // LDS atomics serialise)
                const uint64_t act = __ballot(in);
                if (act) {
                    const int32_t lead = __shfl(bin, (int)__builtin_ctzll(act));
                    const uint64_t same = __ballot(in && bin == lead);
                    if (in && bin == lead) {
                        if ((tid & (kWave - 1)) == (int)__builtin_ctzll(same)) atomicAdd(&hist[bin], (uint32_t)__popcll(same));
                    } else if (in) {
                        atomicAdd(&hist[bin], 1u);
                    }
                }
            }
            __syncthreads();
            // suffix counts over the bins, top down: thread t owns bins 2t and 2t+1 counted from the top
            const int nbins = 1 << width;
            int b0 = nbins - 1 - 2 * tid, b1 = nbins - 2 - 2 * tid;
            int32_t c0 = (b0 >= 0) ? (int32_t)hist[b0] : 0;
            int32_t c1 = (b1 >= 0) ? (int32_t)hist[b1] : 0;
            int32_t all_bins;
            int32_t incl = block_inclusive_scan<int32_t, kFifoThreads>(c0 + c1, sbuf, tid, all_bins);
            int32_t before = incl - c0 - c1;  // elements in bins above b0
            if (b0 >= 0 && before < need && before + c0 >= need) { s_bin = b0; s_above = before; }
            if (b1 >= 0 && before + c0 < need && before + c0 + c1 >= need) { s_bin = b1; s_above = before + c0; }
            __syncthreads();
            fixed_hi = (fixed_hi << width) | s_bin;
            need -= s_above;
            shift = nshift;
            __syncthreads();
        }
        const int32_t m_star = fixed_hi;  // count(m > m*) = nb - need < nb <= count(m >= m*)
        // gather: every query above m*, and the first `need` queries (by index) equal to m*: a scan
        // over the threads' counts of equal entries gives their index order
        int32_t eq = 0;
#pragma unroll
        for (int r = 0; r < kOwn; ++r) eq += mv[r] == m_star ? 1 : 0;
        int32_t eq_all;
        int32_t rank = block_inclusive_scan<int32_t, kFifoThreads>(eq, sbuf, tid, eq_all) - eq;
#pragma unroll
        for (int r = 0; r < kOwn; ++r) {
            const int32_t m = mv[r];
            const bool is_eq = m == m_star;
            if (m > m_star || (is_eq && rank < need)) {
                const int32_t at = atomicAdd(&s_count, 1);
                if (at < kFifoMaxBatch)
                    cand[at] = ((uint64_t)(0x7FFFFFFFu - (uint32_t)m) << 32) | (uint64_t)(uint32_t)(tid * kOwn + r);
            }
            rank += is_eq ? 1 : 0;
        }
        __syncthreads();
    }
    __syncthreads();
    // sort them by (-match_len, index), padded to the next power of two
    int32_t np2 = 1;
    while (np2 < n_cand) np2 <<= 1;
    for (int32_t i = n_cand + tid; i < np2; i += kFifoThreads) cand[i] = ~0ull;
    __syncthreads();
    sort_lds<kFifoThreads, kFifoMaxBatch / kFifoThreads, false>(cand, nullptr, np2, tid);
    for (int32_t p = tid; p < nb; p += kFifoThreads) {
        l_elem[p] = (uint32_t)cand[p];
        a_in_l[p] = 0xFFFFFFFFu;
    }
    __syncthreads();
    if (lpm_only) {
        for (int32_t j = tid; j < nb; j += kFifoThreads) batch_idx[j] = (int32_t)l_elem[j];
        return;
    }
    for (int32_t p = tid; p < nb; p += kFifoThreads) {
        uint32_t e = l_elem[p];
        if (e < (uint32_t)nb) a_in_l[e] = (uint32_t)p;  // the e-th oldest query sits at position p of L
    }
    __syncthreads();
    FifoAcc acc{l_elem, a_in_l};
    two_cursor_block<FifoAcc, kFifoThreads>(acc, nb, nb, k, phase, batch_idx, tid, s_walk);
}

// ---- the same selection for long arrival-ordered queues: short multi-workgroup kernels ----
// One compute unit sweeping a 65,536-entry queue is bound by its own LDS-atomic and load rates, so
// long queues are histogrammed, counted and gathered by many workgroups (1,024 entries each) and only
// the final sort + walk over the nb winners runs in one workgroup.
constexpr int kFqThreads = 1024;
constexpr int kFqMinTile = 4096;    // queue entries per workgroup, at least
constexpr int kFqMaxWg = 32;        // workgroups of the sweeps, at most (each owns one row of suffix counts)
constexpr int kFqLevelBits = 14;    // bits of match length resolved per histogram kernel (prompts of up to 16,383 tokens: one level)
constexpr int kFqBins = 1 << kFqLevelBits;
constexpr int kFqRow = kFqBins + 64;   // words per row of suffix counts (bins 0 .. nbins, the last one zero)
constexpr int kFqMaxLevels = 5;     // 31 bits of score (+ 32 bits of tie key) at most

// What the longest-match picks maximise, as one unsigned number ("goodness"): the score, or with
// tie keys (score, inverted tie key) - a smaller tie key wins among equal scores.
template <bool TIE>
struct FqKey;
template <>
struct FqKey<false> {
    using G = uint32_t;
    const int32_t *__restrict__ score;
    __device__ __forceinline__ G at(int32_t i, int32_t &m) const {
        m = score[i];
        m = m < 0 ? 0 : m;
        return (uint32_t)m;
    }
};
template <>
struct FqKey<true> {
    using G = uint64_t;
    const int32_t *__restrict__ score;
    const uint32_t *__restrict__ tie;
    __device__ __forceinline__ G at(int32_t i, int32_t &m) const {
        m = score[i];
        m = m < 0 ? 0 : m;
        return ((uint64_t)(uint32_t)m << 32) | (uint64_t)(0xFFFFFFFFu - tie[i]);
    }
};

// Nothing in the workspace has to hold a particular value when a selection starts, and no two
// workgroups ever add into the same word: every workgroup owns one row of suffix counts (entries of
// its stretch of the queue whose digit is >= bin), one state record and one flag.  The digit of the
// nb-th largest goodness at a level is the largest bin whose column sum over the rows reaches the
// number still needed; every workgroup finds it for itself at the start of the next kernel (two
// rounds of independent loads), so there is no shared histogram to clear, no atomic on a shared
// bin and no "last workgroup" between the levels.
struct FqWgState {
    uint64_t fixed_hi;  // digits decided before the level whose rows are current (written from level 1 on)
    int32_t need;       // winners still to be found among the entries that share fixed_hi
    int32_t gt;         // this workgroup's entries above fixed_hi at the levels already closed
    int32_t viol;       // level 0: arrival order broken in this stretch, or a score above the caller's bound
    int32_t flag;       // gather kernel: this workgroup's winners are written (cleared by the histogram kernels)
    int32_t pad[2];
};

struct FqWs {
    FqWgState *wg;       // [kFqMaxWg]
    uint32_t *rows[2];   // [n_wg][kFqRow] suffix counts, by parity of the level
    uint32_t *coarse[2]; // [n_wg][kFqThreads] every per-th suffix count of a row (per = ceil(nbins / 1024)), side by side
    uint64_t *cand;      // [kFifoMaxBatch] winners as inverted goodness (no tie keys: with the index below it)
    uint32_t *cand_idx;  // [kFifoMaxBatch] with tie keys: the winners' indices
};

struct FqDigit {
    int32_t digit;  // largest bin whose suffix count over all rows is >= need
    int32_t above;  // entries in the bins above it
    int32_t base;   // first bin of the second round
};
// After fq_search, row g's suffix counts at the bins base + q (q = 0 .. per) of the second round sit at
// s_a[kFqFine + 32 q + g] (until s_a is written again): the counts at the digit and above it need no
// further load.
constexpr int kFqFine = 64;
__device__ __forceinline__ int32_t fq_fine(const int32_t *s_a, const FqDigit &d, int off, int g) {
    return s_a[kFqFine + 32 * (d.digit - d.base + off) + g];
}

// Every thread of the workgroup calls it (THREADS = kFqThreads); s_a holds kFqThreads + 1 words, s_b 32.
// Column sums of suffix counts fall from bin to bin, so the digit lies behind the last of 1,024
// evenly spaced probes that still reaches `need`; a second round looks at the bins between that
// probe and the next.
__device__ __forceinline__ FqDigit fq_search(const uint32_t *__restrict__ rows, const uint32_t *__restrict__ coarse,
                                            int n_wg, int nbins, int32_t need, int32_t *s_a, int32_t *s_b, int tid) {
    const int per = (nbins + kFqThreads - 1) / kFqThreads;  // <= 16
    const int p = tid * per;
    int32_t s = -1;
    if (p < nbins) {
        // (all loads of a chunk are issued before the first is added)
        s = 0;
        for (int g0 = 0; g0 < n_wg; g0 += 16) {
            uint32_t v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = (g0 + u < n_wg) ? coarse[(size_t)(g0 + u) * kFqThreads + tid] : 0u;
#pragma unroll
            for (int u = 0; u < 16; ++u) s += (int32_t)v[u];
        }
    }
    __syncthreads();  // (the arrays may still be read from an earlier call)
    s_a[tid] = s;
    if (tid == 0) {
        s_a[kFqThreads] = -1;
        s_b[0] = 0;
        s_b[1] = 0;
        s_b[2] = 0;
    }
    __syncthreads();
    if (s >= need && s_a[tid + 1] < need) s_b[0] = p;  // one thread: the sums fall and the first reaches need
    __syncthreads();
    const int base = s_b[0];
    __syncthreads();
    // the bins base .. base + per: one load per thread (bin = tid / 32, row = tid mod 32), summed in LDS
    if (tid <= per) s_a[tid] = 0;
    __syncthreads();
    {
        const int q = tid >> 5, g = tid & 31;
        static_assert(kFqMaxWg <= 32 && (kFqBins / kFqThreads + 1) * 32 <= kFqThreads, "one load per thread");
        static_assert(kFqFine + 32 * (kFqBins / kFqThreads + 1) <= kFqThreads, "room for the second round's counts");
        if (q <= per) {
            uint32_t v = 0;
            if (g < n_wg && base + q <= nbins) v = rows[(size_t)g * kFqRow + base + q];  // (bin nbins holds zeros)
            if (v) atomicAdd(&s_a[q], (int32_t)v);
            s_a[kFqFine + 32 * q + g] = (int32_t)v;
        }
    }
    __syncthreads();
    if (tid < per && base + tid < nbins && s_a[tid] >= need && s_a[tid + 1] < need) {
        s_b[1] = base + tid;
        s_b[2] = s_a[tid + 1];
    }
    __syncthreads();
    FqDigit d{s_b[1], s_b[2], base};
    if (d.digit < base) d.digit = base;  // (only when no bin qualified: rows of a refused call)
    return d;
}

// The state a kernel starts from: after one level nothing has been decided yet.
__device__ __forceinline__ void fq_prev_state(const FqWs &ws, int levels_done, int32_t nb, uint64_t &fixed_hi,
                                              int32_t &need, int32_t &gt) {
    fixed_hi = 0;
    need = nb;
    gt = 0;
    if (levels_done >= 2) {
        const FqWgState *st = &ws.wg[blockIdx.x];
        fixed_hi = st->fixed_hi;
        need = st->need;
        gt = st->gt;
    }
}

// Suffix counts of one digit (up to 14 bits) of the goodness values that share the digits fixed so far, one
// row per workgroup; level 0 also checks the arrival order and the caller's bound on the scores.
// `tile` = queue entries per workgroup (a multiple of the workgroup size), `nbins` = bins of this
// level, `prev_nbins` / `prev_width` = those of the level before.
template <bool TIE>
__global__ __launch_bounds__(kFqThreads) void k_fq_hist(const uint64_t *__restrict__ arrival, FqKey<TIE> key, LiveN nn,
                                                       int32_t batch, int32_t max_match, int level, int shift, int width,
                                                       int nbins, int prev_nbins, int prev_width, int32_t tile,
                                                       int order_only, FqWs ws) {
    using G = typename FqKey<TIE>::G;
    const int32_t n = nn.get();
    __shared__ uint32_t h[kFqBins + 1];
    __shared__ int32_t s_a[kFqThreads + 1];
    __shared__ int32_t s_b[32];
    __shared__ int32_t part[kFqThreads / kWave];
    __shared__ int32_t s_viol;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int n_wg = (int)gridDim.x, b = (int)blockIdx.x;
    const int32_t nb = batch < n ? batch : n;
    if (tid == 0) {
        s_viol = 0;
        ws.wg[b].flag = 0;
    }
    G fixed_hi = 0;
    if (level > 0) {
        if (nb <= 0) return;  // (an empty queue: nothing is looked at by the kernels behind this one)
        uint64_t f;
        int32_t need, gt;
        fq_prev_state(ws, level, nb, f, need, gt);
        const uint32_t *prev = ws.rows[(level - 1) & 1];
        const FqDigit d = fq_search(prev, ws.coarse[(level - 1) & 1], n_wg, prev_nbins, need, s_a, s_b, tid);
        f = (f << prev_width) | (uint64_t)(uint32_t)d.digit;
        fixed_hi = (G)f;
        if (tid == 0) {
            FqWgState *st = &ws.wg[b];
            st->fixed_hi = f;
            st->need = need - d.above;
            st->gt = gt + fq_fine(s_a, d, 1, b);
        }
    }
    for (int i = tid; i <= nbins; i += kFqThreads) h[i] = 0;
    __syncthreads();
    const int32_t base = b * tile;
    bool viol = false;
    constexpr int kRows = 4;  // rows of the stretch whose loads are issued together
    for (int32_t r0 = 0; r0 < tile; r0 += kRows * kFqThreads) {
        if (base + r0 >= n) break;  // (uniform)
        G gv[kRows];
        int32_t mv[kRows];
        uint64_t a0[kRows], a1[kRows];
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
            const int32_t i = base + r0 + u * kFqThreads + tid;
            const bool in = r0 + u * kFqThreads < tile && i < n;
            mv[u] = 0;
            gv[u] = in ? key.at(i, mv[u]) : (G)0;
            a0[u] = (level == 0 && in) ? arrival[i] : 0ull;
            a1[u] = (level == 0 && in && i + 1 < n) ? arrival[i + 1] : ~0ull;
        }
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
            const int32_t i = base + r0 + u * kFqThreads + tid;
            bool in = r0 + u * kFqThreads < tile && i < n;
            const G g = gv[u];
            if (level == 0 && in) {
                viol |= mv[u] > max_match;
                viol |= a0[u] > a1[u];
            }
            if (order_only) continue;
            in = in && (level == 0 || (g >> (shift + width)) == fixed_hi);  // (level > 0: shift + width < bits of G)
            const int32_t bin = (int32_t)((g >> shift) & (G)((1 << width) - 1));
            // lanes that share the first active lane's bin are added once (scores cluster and same-address
            // LDS atomics serialise)
            const uint64_t act = __ballot(in);
            if (act) {
                const int32_t lead = __shfl(bin, (int)__builtin_ctzll(act));
                const uint64_t same = __ballot(in && bin == lead);
                if (in && bin == lead) {
                    if (lane == (int)__builtin_ctzll(same)) atomicAdd(&h[bin], (uint32_t)__popcll(same));
                } else if (in) {
                    atomicAdd(&h[bin], 1u);
                }
            }
        }
    }
    if (level == 0) {
        if (viol) atomicOr(&s_viol, 1);
        __syncthreads();
        if (tid == 0) ws.wg[b].viol = s_viol;
    }
    if (order_only) return;
    __syncthreads();
    // suffix counts in place: thread t owns a run of bins counted from the top
    const int per = (nbins + kFqThreads - 1) / kFqThreads;
    constexpr int kMaxPer = kFqBins / kFqThreads;
    int32_t c[kMaxPer];
    int32_t mine = 0;
#pragma unroll
    for (int q = 0; q < kMaxPer; ++q) {
        const int bin = nbins - 1 - (tid * per + q);
        c[q] = (q < per && bin >= 0) ? (int32_t)h[bin] : 0;
        mine += c[q];
    }
    int32_t all;
    int32_t run = block_inclusive_scan<int32_t, kFqThreads>(mine, part, tid, all) - mine;  // entries in higher bins
#pragma unroll
    for (int q = 0; q < kMaxPer; ++q) {
        const int bin = nbins - 1 - (tid * per + q);
        if (q < per && bin >= 0) {
            run += c[q];
            h[bin] = (uint32_t)run;
        }
    }
    __syncthreads();
    uint32_t *row = ws.rows[level & 1] + (size_t)b * kFqRow;
    for (int i = tid; i <= nbins; i += kFqThreads) row[i] = h[i];
    ws.coarse[level & 1][(size_t)b * kFqThreads + tid] = (tid * per < nbins) ? h[tid * per] : 0u;
}

struct FqLds {
    uint64_t *cand;    // [kFifoMaxBatch]
    uint32_t *l_elem;  // [kFifoMaxBatch]
    uint32_t *a_in_l;  // [kFifoMaxBatch]
    int32_t *walk;     // [kWalkScratch]
};

// The longest-match order of the nb winners - sorted here by (-score, [tie key,] index) in LDS, or, with
// `placed`, read as the gather kernel placed it - and the walk over both orders.  Run by one whole
// workgroup once every winner is written.
template <bool TIE>
__device__ __forceinline__ void fq_finish(int32_t n, uint32_t k, uint32_t phase_in, int32_t violated, int32_t batch,
                                          bool placed, const FqWs &ws, const FqLds &lds,
                                          uint32_t *__restrict__ phase_inout, int32_t *__restrict__ batch_idx,
                                          int32_t *__restrict__ n_selected) {
    uint64_t *cand = lds.cand;
    uint32_t *l_elem = lds.l_elem, *a_in_l = lds.a_in_l;
    int32_t *s_walk = lds.walk;
    const int tid = threadIdx.x;
    constexpr int kPer = kFifoMaxBatch / kFifoThreads;
    const int32_t nb = batch < n ? batch : n;
    const bool lpm_only = (k == 0u || k == 0xFFFFFFFFu);
    const uint32_t phase = lpm_only ? 0u : (phase_in % k);
    if (violated) {  // the caller's promise does not hold: select nothing, say so
        if (tid == 0) *n_selected = -1;
        return;
    }
    if (tid == 0) {
        *n_selected = nb;
        *phase_inout = lpm_only ? 0u : (uint32_t)(((uint64_t)phase + (uint64_t)nb) % k);
    }
    if (placed) {
#pragma unroll
        for (int c = 0; c < kPer; ++c) {
            const int32_t i = tid + c * kFifoThreads;
            if (i < nb) {
                l_elem[i] = ws.cand_idx[i];
                a_in_l[i] = 0xFFFFFFFFu;
            }
        }
    } else {
        int32_t np2 = 1;
        while (np2 < nb) np2 <<= 1;
#pragma unroll
        for (int c = 0; c < kPer; ++c) {
            const int32_t i = tid + c * kFifoThreads;
            if (i < np2) {
                cand[i] = (i < nb) ? ws.cand[i] : ~0ull;
                if (TIE) l_elem[i] = (i < nb) ? ws.cand_idx[i] : 0xFFFFFFFFu;  // second key word: the index
            }
        }
        __syncthreads();
        sort_lds<kFifoThreads, kFifoMaxBatch / kFifoThreads, TIE>(cand, l_elem, np2, tid);
        for (int32_t p = tid; p < nb; p += kFifoThreads) {
            if (!TIE) l_elem[p] = (uint32_t)cand[p];
            a_in_l[p] = 0xFFFFFFFFu;
        }
    }
    __syncthreads();
    if (lpm_only) {
        for (int32_t j = tid; j < nb; j += kFifoThreads) batch_idx[j] = (int32_t)l_elem[j];
        return;
    }
    for (int32_t p = tid; p < nb; p += kFifoThreads) {
        uint32_t e = l_elem[p];
        if (e < (uint32_t)nb) a_in_l[e] = (uint32_t)p;  // the e-th oldest query sits at position p of L
    }
    __syncthreads();
    FifoAcc acc{l_elem, a_in_l};
    two_cursor_block<FifoAcc, kFifoThreads>(acc, nb, nb, k, phase, batch_idx, tid, s_walk);
}

// Winners = every entry above g* and the first `need` entries (by index) equal to g*; written in index
// order at positions given by prefix counts over the rows (no atomics).  A workgroup that finds every
// flag set after raising its own runs the final sort and walk: the one whose flag went up last does,
// and if two see it at once both write the same batch.
// When one level resolved the whole score (no tie keys), the rows of suffix counts also give every
// winner its place in the longest-match order, and the final sort is not needed: a workgroup sorts its
// own winners (a few dozen, on registers), and the winner at place q of that list, of score m, has in
// front of it in the whole queue the entries of score >= m of the workgroups before (their rows at m:
// equal scores go by index), its own q, and the entries of score > m of the workgroups behind (their
// rows at m + 1).
template <bool TIE>
__global__ __launch_bounds__(kFqThreads) void k_fq_gather(FqKey<TIE> key, LiveN nn, KArg ka, int32_t batch, int levels,
                                                         int width, int nbins, int32_t tile, FqWs ws,
                                                         uint32_t *__restrict__ phase_inout,
                                                         int32_t *__restrict__ batch_idx,
                                                         int32_t *__restrict__ n_selected) {
    using G = typename FqKey<TIE>::G;
    const int32_t n = nn.get();
    const uint32_t k = ka.get();
    const uint32_t phase_in = *phase_inout;  // (read by every workgroup before any flag is up, written after all are)
    __shared__ int32_t s_a[kFqThreads + 1];
    __shared__ int32_t s_b[32];
    __shared__ int32_t s_rank, s_out, s_last, s_viol;
    constexpr int kRows = 4;  // rows of the stretch handled together
    __shared__ int32_t w_eq[kRows][kFqThreads / kWave], w_win[kRows][kFqThreads / kWave];
    __shared__ uint64_t l_cand[kFifoMaxBatch];
    __shared__ uint32_t l_elem[kFifoMaxBatch];
    __shared__ uint32_t l_a_in_l[kFifoMaxBatch];
    __shared__ int32_t l_walk[kWalkScratch];
    const FqLds lds{l_cand, l_elem, l_a_in_l, l_walk};
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave;
    const int n_wg = (int)gridDim.x, b = (int)blockIdx.x;
    const int32_t nb = batch < n ? batch : n;
    const bool placed = !TIE && levels == 1;
    const int32_t base = b * tile;
    // (the first rows of the stretch are requested before the search: they do not depend on it)
    G gv[kRows];
    int32_t mv[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
        const int32_t i = base + u * kFqThreads + tid;
        mv[u] = 0;
        gv[u] = (u * kFqThreads < tile && i < n) ? key.at(i, mv[u]) : (G)0;
    }
    if (nb > 0) {
        uint64_t f;
        int32_t need, gt_unused;
        fq_prev_state(ws, levels, nb, f, need, gt_unused);
        const uint32_t *rows = ws.rows[(levels - 1) & 1];
        const FqDigit d = fq_search(rows, ws.coarse[(levels - 1) & 1], n_wg, nbins, need, s_a, s_b, tid);
        const G g_star = (G)((f << width) | (uint64_t)(uint32_t)d.digit);
        need -= d.above;
        // entries equal to g* and winners in the workgroups before this one
        if (wv == 0) {
            int32_t gt = 0, eq = 0;
            if (lane < n_wg) {
                const int32_t hi = fq_fine(s_a, d, 1, lane);
                gt = (levels >= 2 ? ws.wg[lane].gt : 0) + hi;
                eq = fq_fine(s_a, d, 0, lane) - hi;
            }
            const int32_t gt_before = wave_inclusive_scan(gt, lane) - gt;
            const int32_t eq_before = wave_inclusive_scan(eq, lane) - eq;
            if (lane == b) {
                s_rank = eq_before;
                s_out = gt_before + (eq_before < need ? eq_before : need);
            }
        }
        __syncthreads();
        int32_t rank = s_rank, out = s_out;
        const int32_t out0 = out;
        const uint64_t below = (1ull << lane) - 1ull;
        for (int32_t r0 = 0; r0 < tile; r0 += kRows * kFqThreads) {
            if (base + r0 >= n) break;  // (uniform)
            if (r0 > 0) {
#pragma unroll
                for (int u = 0; u < kRows; ++u) {
                    const int32_t i = base + r0 + u * kFqThreads + tid;
                    mv[u] = 0;
                    gv[u] = (r0 + u * kFqThreads < tile && i < n) ? key.at(i, mv[u]) : (G)0;
                }
            }
            bool in[kRows], is_eq[kRows];
            uint64_t eqmask[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                in[u] = r0 + u * kFqThreads < tile && base + r0 + u * kFqThreads + tid < n;
                is_eq[u] = in[u] && gv[u] == g_star;
                eqmask[u] = __ballot(is_eq[u]);
            }
            __syncthreads();  // (the counts of the rows before are read)
            if (lane == 0) {
#pragma unroll
                for (int u = 0; u < kRows; ++u) w_eq[u][wv] = (int32_t)__popcll(eqmask[u]);
            }
            __syncthreads();
            bool win[kRows];
            uint64_t wmask[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u) {  // rows in turn, inside a row the wavefronts before mine
                int32_t eq_before = 0, eq_row = 0;
                for (int w = 0; w < kFqThreads / kWave; ++w) {
                    const int32_t v = w_eq[u][w];
                    if (w < wv) eq_before += v;
                    eq_row += v;
                }
                const int32_t my_rank = rank + eq_before + (int32_t)__popcll(eqmask[u] & below);
                win[u] = in[u] && (gv[u] > g_star || (is_eq[u] && my_rank < need));
                wmask[u] = __ballot(win[u]);
                rank += eq_row;
            }
            if (lane == 0) {
#pragma unroll
                for (int u = 0; u < kRows; ++u) w_win[u][wv] = (int32_t)__popcll(wmask[u]);
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                int32_t win_before = 0, win_row = 0;
                for (int w = 0; w < kFqThreads / kWave; ++w) {
                    const int32_t v = w_win[u][w];
                    if (w < wv) win_before += v;
                    win_row += v;
                }
                if (win[u]) {
                    const int32_t i = base + r0 + u * kFqThreads + tid;
                    const int32_t at = out + win_before + (int32_t)__popcll(wmask[u] & below);
                    if (at >= 0 && at < kFifoMaxBatch) {
                        if (TIE) {
                            ws.cand[at] = ~(uint64_t)gv[u];
                            ws.cand_idx[at] = (uint32_t)i;
                        } else if (!placed) {
                            ws.cand[at] = ((uint64_t)(0x7FFFFFFFu - (uint32_t)mv[u]) << 32) | (uint64_t)(uint32_t)i;
                        } else {  // (this workgroup's list, in index order; at - out0 < nb)
                            l_cand[at - out0] = ((uint64_t)(0x7FFFFFFFu - (uint32_t)mv[u]) << 32) | (uint64_t)(uint32_t)i;
                        }
                    }
                }
                out += win_row;
            }
        }
        if (placed) {
            int32_t mine = out - out0;  // this workgroup's winners
            if (mine > kFifoMaxBatch) mine = kFifoMaxBatch;
            if (mine < 0) mine = 0;
            int32_t np2 = 1;
            while (np2 < mine) np2 <<= 1;
            __syncthreads();
            for (int32_t i = mine + tid; i < np2; i += kFqThreads) l_cand[i] = ~0ull;
            __syncthreads();
            sort_lds<kFqThreads, kFifoMaxBatch / kFqThreads, false>(l_cand, l_elem, np2, tid);
            int32_t *place = (int32_t *)l_a_in_l;
            for (int32_t q = tid; q < mine; q += kFqThreads) place[q] = q;
            __syncthreads();
            const int32_t pairs = mine * n_wg;
            for (int32_t idx = tid; idx < pairs; idx += kFqThreads) {
                const int32_t q = idx / n_wg, g = idx - q * n_wg;
                const int32_t mm = (int32_t)(0x7FFFFFFFu - (uint32_t)(l_cand[q] >> 32)) + (g < b ? 0 : 1);
                if (g != b && mm <= nbins) {  // (a score beyond the caller's bound has no bin; the call is refused anyway)
                    const uint32_t v = rows[(size_t)g * kFqRow + mm];
                    if (v) atomicAdd(&place[q], (int32_t)v);
                }
            }
            __syncthreads();
            for (int32_t q = tid; q < mine; q += kFqThreads) {
                const int32_t at = place[q];
                if (at >= 0 && at < kFifoMaxBatch) ws.cand_idx[at] = (uint32_t)l_cand[q];
            }
        }
    }
    // raise this workgroup's flag behind its winners, then look at everybody's
    __syncthreads();
    if (wv == 0) {
        if (lane == 0) {
            __threadfence();  // (behind the barrier: covers the whole workgroup's stores)
            __hip_atomic_exchange(&ws.wg[b].flag, 1, __ATOMIC_SEQ_CST, __HIP_MEMORY_SCOPE_AGENT);
            __threadfence();
        }
        int32_t up = 1, v = 0;
        if (lane < n_wg) {
            up = __hip_atomic_load(&ws.wg[lane].flag, __ATOMIC_SEQ_CST, __HIP_MEMORY_SCOPE_AGENT);
            v = ws.wg[lane].viol;
        }
        const bool all_up = __ballot(up == 0) == 0ull;
        const bool any_viol = __ballot(v != 0) != 0ull;
        if (lane == 0) {
            s_last = all_up ? 1 : 0;
            s_viol = any_viol ? 1 : 0;
        }
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    fq_finish<TIE>(n, k, phase_in, s_viol, batch, placed, ws, lds, phase_inout, batch_idx, n_selected);
}

// FCFS on an arrival-ordered queue: its first nb entries (after the order check of the histogram kernel).
__global__ __launch_bounds__(256) void k_fq_fcfs(LiveN nn, int32_t batch, int n_wg, FqWs ws,
                                                 uint32_t *__restrict__ phase_inout, int32_t *__restrict__ batch_idx,
                                                 int32_t *__restrict__ n_selected) {
    const int32_t n = nn.get();
    const int32_t nb = batch < n ? batch : n;
    int32_t violated = 0;
    for (int g = 0; g < n_wg; ++g) violated |= ws.wg[g].viol;
    if (violated) {
        if (blockIdx.x == 0 && threadIdx.x == 0) *n_selected = -1;
        return;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *n_selected = nb;
        *phase_inout = 0u;  // k = 1: every slot is the start of a cycle
    }
    int32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < nb) batch_idx[j] = j;
}

// Workgroups of the sweeps over a queue of n entries and the entries each of them takes.
static void fq_grid(int32_t n, int *n_wg, int32_t *tile) {
    int64_t g = ((int64_t)n + kFqMinTile - 1) / kFqMinTile;
    if (g < 1) g = 1;
    if (g > kFqMaxWg) g = kFqMaxWg;
    int64_t t = ((int64_t)(n > 0 ? n : 1) + g - 1) / g;
    t = (t + kFqThreads - 1) / kFqThreads * kFqThreads;
    *n_wg = (int)g;
    *tile = (int32_t)t;
}

static void carve_fq(FqWs &f, char *base, int32_t n, size_t *used) {
    size_t o = 0;
    auto take = [&](size_t bytes) { void *p = base ? base + o : nullptr; o += align_up(bytes, 256); return p; };
    int n_wg;
    int32_t tile;
    fq_grid(n, &n_wg, &tile);
    f.wg = (FqWgState *)take(sizeof(FqWgState) * kFqMaxWg);
    f.rows[0] = (uint32_t *)take((size_t)n_wg * kFqRow * 4);
    f.rows[1] = (uint32_t *)take((size_t)n_wg * kFqRow * 4);
    f.coarse[0] = (uint32_t *)take((size_t)n_wg * kFqThreads * 4);
    f.coarse[1] = (uint32_t *)take((size_t)n_wg * kFqThreads * 4);
    f.cand = (uint64_t *)take((size_t)kFifoMaxBatch * 8);
    f.cand_idx = (uint32_t *)take((size_t)kFifoMaxBatch * 4);
    *used = o;
}

template <bool TIE>
static int select_fifo_long(const uint64_t *arrival, FqKey<TIE> key, LiveN nn, KArg k, int32_t batch,
                            int32_t max_match, uint32_t *phase_inout, int32_t *batch_idx, int32_t *n_selected,
                            char *workspace, hipStream_t stream) {
    FqWs f;
    size_t used = 0;
    carve_fq(f, workspace, nn.n, &used);
    const LiveN n = nn;
    const int32_t nb = batch < nn.n ? batch : nn.n;  // upper bound of the picks, sizes the FCFS launch
    int n_wg;
    int32_t tile;
    fq_grid(nn.n, &n_wg, &tile);
    int mbits = 0;
    while (mbits < 31 && (max_match >> mbits) != 0) ++mbits;
    if (mbits == 0) mbits = 1;
    const bool fcfs = (!k.dev && k.k == 1u);  // (a k read on the device takes the general kernels)
    int shift = mbits + (TIE ? 32 : 0), level = 0;
    int width = 0, nbins = 0, prev_width = 0, prev_nbins = 0;
    while (shift > 0 && level < kFqMaxLevels) {
        prev_width = width;
        prev_nbins = nbins;
        width = shift < kFqLevelBits ? shift : kFqLevelBits;
        shift -= width;
        // (the top digit only reaches as far as the caller's bound on the scores does)
        nbins = (level == 0 && !TIE && (max_match >> shift) + 1 < (1 << width)) ? (max_match >> shift) + 1 : (1 << width);
        hipLaunchKernelGGL(k_fq_hist<TIE>, dim3(n_wg), dim3(kFqThreads), 0, stream, arrival, key, n, batch, max_match,
                           level, shift, width, nbins, prev_nbins, prev_width, tile, fcfs ? 1 : 0, f);
        ++level;
        if (fcfs) break;  // only the order check of level 0 is needed
    }
    if (fcfs) {
        hipLaunchKernelGGL(k_fq_fcfs, dim3((nb + 255) / 256), dim3(256), 0, stream, n, batch, n_wg, f, phase_inout,
                           batch_idx, n_selected);
        return check_launch();
    }
    hipLaunchKernelGGL(k_fq_gather<TIE>, dim3(n_wg), dim3(kFqThreads), 0, stream, key, n, k, batch, level, width, nbins,
                       tile, f, phase_inout, batch_idx, n_selected);
    return check_launch();
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
    ws.viol = (int32_t *)take(256);
    *used = o;
}

size_t select_sort_workspace_bytes(int32_t n) {
    SelectWs ws;
    size_t need = 0;
    carve(ws, nullptr, n, &need);
    return need;
}

// Both total orders of the queue and each query's position in them (see the head of this file).
// Without `want_l` only the oldest-first order is built (the other pointers then alias it).
int build_select_orders(const uint64_t *arrival, const int32_t *score, const uint32_t *tie_key, int32_t n,
                        const int32_t *n_live, bool want_l, void *workspace, size_t workspace_bytes,
                        hipStream_t stream, SelectOrders *out, bool arrival_ordered, int32_t max_score) {
    SelectWs ws;
    size_t need = 0;
    carve(ws, (char *)workspace, n, &need);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return KLPM_EARENA;
    const LiveN nn{n, n_live};
    const uint32_t *order_a = ws.val_a, *order_l = ws.val_a;
    out->violated = nullptr;
    if (arrival_ordered && want_l && !tie_key && max_score > 0 && n > kSmallOrdersN) {
        // no sort by arrival, and only as many passes over the scores as the bound needs
        int bits = 1;
        while (bits < 31 && (max_score >> bits) != 0) ++bits;
        const unsigned g = (unsigned)((n + 255) / 256);
        hipLaunchKernelGGL(k_sel_zero_flag, dim3(1), dim3(kWave), 0, stream, ws.viol);
        hipLaunchKernelGGL(k_sel_fifo_keys, dim3(g), dim3(256), 0, stream, arrival, score, nn, max_score, ws.key_a, ws.val_c,
                           ws.val_a, ws.rank_a, ws.viol);
        bool lfirst = true;
        int rc = radix_sort(ws.key_a, ws.val_c, ws.key_b, ws.val_b, nn, (bits + 7) / 8, ws, stream, &lfirst);
        if (rc) return rc;
        order_l = lfirst ? ws.val_c : ws.val_b;
        hipLaunchKernelGGL(k_sel_rank_l, dim3(g), dim3(256), 0, stream, order_l, nn, ws.rank_l);
        out->order_a = ws.val_a;
        out->order_l = order_l;
        out->rank_a = ws.rank_a;
        out->rank_l = ws.rank_l;
        out->violated = ws.viol + 1;
        return check_launch();
    }
    if (n > 0 && n <= kSmallOrdersN) {
        hipLaunchKernelGGL(k_orders_small, dim3(1), dim3(kSmallOrdersThreads), 0, stream, arrival, score, tie_key, nn,
                           want_l ? 1 : 0, ws.val_a, ws.val_c, ws.rank_a, ws.rank_l);
        out->order_a = ws.val_a;
        out->order_l = want_l ? ws.val_c : ws.val_a;
        out->rank_a = ws.rank_a;
        out->rank_l = ws.rank_l;
        return check_launch();
    }
    if (n > 0) {
        unsigned g = (unsigned)((n + 255) / 256);
        hipLaunchKernelGGL(k_sel_init, dim3(g), dim3(256), 0, stream, arrival, nn, ws.key_a, ws.val_a);
        bool first = true;
        int rc = radix_sort(ws.key_a, ws.val_a, ws.key_b, ws.val_b, nn, 8, ws, stream, &first);
        if (rc) return rc;
        order_a = first ? ws.val_a : ws.val_b;  // 8 passes: back in the first buffer
        if (want_l) {
            // stable sort of the oldest-first order by descending score (then ascending tie key)
            uint32_t *spare = first ? ws.val_b : ws.val_a;
            hipLaunchKernelGGL(k_sel_lkeys, dim3(g), dim3(256), 0, stream, order_a, score, tie_key, nn, ws.key_a,
                               ws.val_c);
            bool lfirst = true;
            rc = radix_sort(ws.key_a, ws.val_c, ws.key_b, spare, nn, tie_key ? 8 : 4, ws, stream, &lfirst);
            if (rc) return rc;
            order_l = lfirst ? ws.val_c : spare;
            hipLaunchKernelGGL(k_sel_ranks, dim3(g), dim3(256), 0, stream, order_a, order_l, nn, ws.rank_a, ws.rank_l);
        }
    }
    out->order_a = order_a;
    out->order_l = order_l;
    out->rank_a = ws.rank_a;
    out->rank_l = ws.rank_l;
    return check_launch();
}

// ---- score and tie-key variants of Algorithm 1 ----
// Hit rate of Algorithm 1's wording as an integer score: floor(m * 2^bits / |x|).
__global__ __launch_bounds__(256) void k_score_hit_rate(const int32_t *__restrict__ match_len,
                                                        const int32_t *__restrict__ len, LiveN nn, int bits,
                                                        int32_t *__restrict__ score) {
    const int32_t n = nn.get();
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int64_t m = match_len[i], l = len[i];
    m = m < 0 ? 0 : m;
    l = l < 1 ? 1 : l;
    m = m > l ? l : m;
    score[i] = (int32_t)((uint64_t)(m << bits) / (uint64_t)l);
}

// Philox-4x32 with 10 rounds (Salmon et al., SC'11): each round multiplies counter words 0 and 2 by
// two fixed odd constants, crosses the halves over and mixes in the key; the key advances by a Weyl
// constant between rounds.
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                        uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
    }
    return c0;
}

__global__ __launch_bounds__(256) void k_tie_keys(uint64_t seed, uint64_t step, const int32_t *__restrict__ id, LiveN nn,
                                                  uint32_t *__restrict__ tie_key) {
    const int32_t n = nn.get();
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t c0 = id ? (uint32_t)id[i] : (uint32_t)i;
    tie_key[i] = philox4x32_10_word0(c0, 0u, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t)seed, (uint32_t)(seed >> 32));
}

}  // namespace klpm

using namespace klpm;

extern "C" int kLPM_score_hit_rate(const int32_t *match_len, const int32_t *len, int32_t n, const int32_t *n_live,
                                   int32_t scale_bits, int32_t *score, kLPM_stream stream) {
    if (n < 0 || scale_bits < 1 || scale_bits > 30) return KLPM_EINVAL;
    if (n == 0) return KLPM_OK;
    if (!match_len || !len || !score) return KLPM_EINVAL;
    hipLaunchKernelGGL(k_score_hit_rate, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, match_len,
                       len, LiveN{n, n_live}, (int)scale_bits, score);
    return check_launch();
}

extern "C" int kLPM_tie_keys(uint64_t seed, uint64_t step, const int32_t *id, int32_t n, const int32_t *n_live,
                             uint32_t *tie_key, kLPM_stream stream) {
    if (n < 0) return KLPM_EINVAL;
    if (n == 0) return KLPM_OK;
    if (!tie_key) return KLPM_EINVAL;
    hipLaunchKernelGGL(k_tie_keys, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, seed, step, id,
                       LiveN{n, n_live}, tie_key);
    return check_launch();
}

extern "C" int kLPM_select_workspace_bytes(int32_t n, size_t *out_bytes) {
    if (n < 0 || !out_bytes) return KLPM_EINVAL;
    SelectWs ws;
    carve(ws, nullptr, n, out_bytes);
    FqWs f;
    size_t fq = 0;
    carve_fq(f, nullptr, n, &fq);
    if (fq > *out_bytes) *out_bytes = fq;
    return KLPM_OK;
}

// Selects nothing: the count goes to zero, the phase stays (n = 0 or batch = 0).
__global__ void k_sel_none(int32_t *__restrict__ n_selected) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_selected = 0;
}

static int select_impl(const uint64_t *arrival, const int32_t *match_len, const uint32_t *tie_key, int32_t n,
                       const int32_t *n_live, uint32_t k_host, const uint32_t *k_dev, int32_t batch, uint32_t flags,
                       int32_t max_match, uint32_t *phase_inout, int32_t *batch_idx, int32_t *n_selected, void *workspace,
                       size_t workspace_bytes, hipStream_t stream) {
    if (n < 0 || batch < 0 || !phase_inout || !n_selected) return KLPM_EINVAL;
    if (n > 0 && (!arrival || !match_len)) return KLPM_EINVAL;
    if (n > 0 && batch > 0 && !batch_idx) return KLPM_EINVAL;
    if (n == 0 || batch == 0) {  // nothing to select: no workspace is needed either
        hipLaunchKernelGGL(k_sel_none, dim3(1), dim3(kWave), 0, stream, n_selected);
        return check_launch();
    }
    const LiveN nn{n, n_live};
    const KArg k{k_host, k_dev};
    // (with tie keys a short queue goes to the one-workgroup sort of both orders further down)
    const bool fifo = (flags & KLPM_SELECT_FIFO) && (batch < n ? batch : n) <= kFifoMaxBatch;
    if (fifo && tie_key && n > kSmallOrdersN) {
        size_t fq_need = 0;
        FqWs probe;
        carve_fq(probe, nullptr, n, &fq_need);
        if (!workspace || workspace_bytes < fq_need || ((uintptr_t)workspace & 255u)) return KLPM_EARENA;
        return select_fifo_long<true>(arrival, FqKey<true>{match_len, tie_key}, nn, k, batch,
                                      max_match > 0 ? max_match : 0x7FFFFFFF, phase_inout, batch_idx, n_selected,
                                      (char *)workspace, stream);
    }
    if (fifo && !tie_key) {
        if (n <= kFqSingleBlockN) {
            hipLaunchKernelGGL(k_select_fifo, dim3(1), dim3(kFifoThreads), 0, stream, arrival, match_len, nn, k, batch,
                               phase_inout, batch_idx, n_selected);
            return check_launch();
        }
        size_t fq_need = 0;
        FqWs probe;
        carve_fq(probe, nullptr, n, &fq_need);
        if (!workspace || workspace_bytes < fq_need || ((uintptr_t)workspace & 255u)) return KLPM_EARENA;
        return select_fifo_long<false>(arrival, FqKey<false>{match_len}, nn, k, batch,
                                       max_match > 0 ? max_match : 0x7FFFFFFF, phase_inout, batch_idx, n_selected,
                                       (char *)workspace, stream);
    }
    SelectOrders ord;
    int rc = build_select_orders(arrival, match_len, tie_key, n, n_live, k_dev || k_host != 1u, workspace,
                                 workspace_bytes, stream, &ord);
    if (rc) return rc;
    hipLaunchKernelGGL(k_sel_walk, dim3(1), dim3(256), 0, stream, ord.order_a, ord.order_l, ord.rank_a, ord.rank_l, nn, k,
                       batch, phase_inout, batch_idx, n_selected);
    return check_launch();
}

extern "C" int kLPM_select(const uint64_t *arrival, const int32_t *match_len, const uint32_t *tie_key, int32_t n,
                           const int32_t *n_live, uint32_t k_host, const uint32_t *k_dev, int32_t batch, uint32_t flags,
                           int32_t max_match, uint32_t *phase_inout, int32_t *batch_idx, int32_t *n_selected,
                           void *workspace, size_t workspace_bytes, kLPM_stream stream) {
    return select_impl(arrival, match_len, tie_key, n, n_live, k_host, k_dev, batch, flags, max_match, phase_inout,
                       batch_idx, n_selected, workspace, workspace_bytes, (hipStream_t)stream);
}

// ---- selection for callers that cannot allocate ----
// The same selection with its workspace in a file-scope device array instead of caller memory.
// Every GPU holds its own copy of the array (at its own address) from the moment the library is
// loaded there until the process ends; the host-side name of the array is only a handle for
// hipGetSymbolAddress, the kernels get the address that call returns.
namespace klpm {
constexpr size_t kStaticScratchBytes = (size_t)KLPM_SELECT_STATIC_MAX_N * 36 + (1u << 20);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];  // per device, filled on the first call there

// Device address of the current device's copy of `scratch` (NULL and *rc set on failure).
static void *static_scratch(int *rc) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        *rc = KLPM_EHIP;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            *rc = KLPM_EHIP;
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    *rc = KLPM_OK;
    return g_scratch_ptr[dev];
}
}  // namespace klpm

extern "C" int kLPM_select_static(const uint64_t *arrival, const int32_t *match_len, const uint32_t *tie_key, int32_t n,
                                  const int32_t *n_live, uint32_t k_host, const uint32_t *k_dev, int32_t batch,
                                  uint32_t flags, int32_t max_match, uint32_t *phase_inout, int32_t *batch_idx,
                                  int32_t *n_selected, kLPM_stream stream) {
    if (n > KLPM_SELECT_STATIC_MAX_N) return KLPM_ELIMIT;
    size_t need = 0;
    if (n >= 0 && (kLPM_select_workspace_bytes(n, &need) != KLPM_OK || need > kStaticScratchBytes)) return KLPM_ELIMIT;
    int rc = KLPM_OK;
    void *ws = static_scratch(&rc);
    if (!ws) return rc;
    return select_impl(arrival, match_len, tie_key, n, n_live, k_host, k_dev, batch, flags, max_match, phase_inout,
                       batch_idx, n_selected, ws, kStaticScratchBytes, (hipStream_t)stream);
}
