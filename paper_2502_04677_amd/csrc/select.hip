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
constexpr int kFifoMaxBatch = 4096;
constexpr int kFifoBins = 2048;
constexpr int kSweepRows = 16;  // independent loads per thread and trip in the queue sweeps

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
    // sweep 0 (coalesced): arrival order check and the largest match length
    {
        int32_t mx = 0;
        bool viol = false;
        // eight independent rows per trip keep the single workgroup's loads in flight together
        for (int32_t base = 0; base < n; base += kSweepRows * kFifoThreads) {
            int32_t mv[kSweepRows];
            uint64_t t0[kSweepRows], t1[kSweepRows];
#pragma unroll
            for (int r = 0; r < kSweepRows; ++r) {
                int32_t i = base + r * kFifoThreads + tid;
                int32_t ic = i < n ? i : n - 1;
                int32_t in = ic + 1 < n ? ic + 1 : n - 1;
                mv[r] = match_len[ic];
                t0[r] = arrival[ic];
                t1[r] = arrival[in];
            }
#pragma unroll
            for (int r = 0; r < kSweepRows; ++r) {
                mx = mv[r] > mx ? mv[r] : mx;
                viol |= t0[r] > t1[r];
            }
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
        // holds the largest match length found by the sweep above
        if (!lpm_only && phase == 0u) {
            if (tid == 0) batch_idx[0] = 0;
            return;
        }
        if (tid == 0) s_bin = n;
        __syncthreads();
        const int32_t best = s_max;
        int32_t first = n;
        for (int32_t base = 0; base < n; base += kSweepRows * kFifoThreads) {
            int32_t mv[kSweepRows];
#pragma unroll
            for (int r = 0; r < kSweepRows; ++r) {
                int32_t i = base + r * kFifoThreads + tid;
                mv[r] = match_len[i < n ? i : n - 1];
            }
#pragma unroll
            for (int r = 0; r < kSweepRows; ++r) {
                int32_t i = base + r * kFifoThreads + tid;
                if (i < n && (mv[r] < 0 ? 0 : mv[r]) == best && i < first) first = i;
            }
        }
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
        for (int32_t i = tid; i < n; i += kFifoThreads) {
            int32_t m = match_len[i];
            m = m < 0 ? 0 : m;
            cand[i] = ((uint64_t)(0x7FFFFFFFu - (uint32_t)m) << 32) | (uint64_t)(uint32_t)i;
        }
    } else {
        // the nb-th largest match length m*, found digit by digit (11 bits per sweep)
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
            for (int32_t base = 0; base < n; base += kSweepRows * kFifoThreads) {
                int32_t mv[kSweepRows];
#pragma unroll
                for (int r = 0; r < kSweepRows; ++r) {
                    int32_t i = base + r * kFifoThreads + tid;
                    mv[r] = match_len[i < n ? i : n - 1];
                }
#pragma unroll
                for (int r = 0; r < kSweepRows; ++r) {
                    int32_t i = base + r * kFifoThreads + tid;
                    int32_t m = mv[r] < 0 ? 0 : mv[r];
                    if (i < n && (m >> shift) == fixed_hi) atomicAdd(&hist[(m >> nshift) & ((1 << width) - 1)], 1u);
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
        // gather: every query above m*, and the first `need` queries (by index) equal to m*.  Each
        // wavefront owns a contiguous segment of the queue and reads it 64 entries at a time, so the
        // index order of the equal-to-m* queries is a ballot prefix plus the counts of earlier segments.
        {
            const int lane = tid & (kWave - 1);
            const int wv = tid / kWave;
            const int n_wv = kFifoThreads / kWave;
            const int32_t seg = ((n + n_wv - 1) / n_wv + kWave - 1) / kWave * kWave;
            const int32_t lo = (int64_t)wv * seg < n ? wv * seg : n;
            const int32_t hi = lo + seg < n ? lo + seg : n;
            int32_t eq = 0;
            for (int32_t base = lo; base < hi; base += kSweepRows * kWave) {
                int32_t mv[kSweepRows];
#pragma unroll
                for (int r = 0; r < kSweepRows; ++r) {
                    int32_t i = base + r * kWave + lane;
                    mv[r] = match_len[i < hi ? i : hi - 1];
                }
#pragma unroll
                for (int r = 0; r < kSweepRows; ++r) {
                    int32_t i = base + r * kWave + lane;
                    int32_t m = mv[r] < 0 ? 0 : mv[r];
                    eq += (int32_t)__popcll(__ballot(i < hi && m == m_star));
                }
            }
            if (lane == 0) sbuf[wv] = eq;
            __syncthreads();
            int32_t rank = 0;  // equal-to-m* queries in earlier segments
            for (int w2 = 0; w2 < wv; ++w2) rank += sbuf[w2];
            for (int32_t base = lo; base < hi; base += kSweepRows * kWave) {
                int32_t mv[kSweepRows];
#pragma unroll
                for (int r = 0; r < kSweepRows; ++r) {
                    int32_t i = base + r * kWave + lane;
                    mv[r] = match_len[i < hi ? i : hi - 1];
                }
#pragma unroll
                for (int r = 0; r < kSweepRows; ++r) {
                    int32_t i = base + r * kWave + lane;
                    bool in = i < hi;
                    int32_t m = mv[r] < 0 ? 0 : mv[r];
                    bool is_eq = in && m == m_star;
                    uint64_t eqmask = __ballot(is_eq);
                    int32_t my_rank = rank + (int32_t)__popcll(eqmask & ((1ull << lane) - 1ull));
                    bool win = in && (m > m_star || (is_eq && my_rank < need));
                    if (win) {
                        int32_t at = atomicAdd(&s_count, 1);
                        if (at < kFifoMaxBatch)
                            cand[at] = ((uint64_t)(0x7FFFFFFFu - (uint32_t)m) << 32) | (uint64_t)(uint32_t)i;
                    }
                    rank += (int32_t)__popcll(eqmask);
                }
            }
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
    if (tid >= kWave) return;
    FifoAcc acc{l_elem, a_in_l};
    two_cursor_walk(acc, nb, nb, k, phase, batch_idx, tid);
}

// ---- the same selection for long arrival-ordered queues: short multi-workgroup kernels ----
// One compute unit sweeping a 65,536-entry queue is bound by its own LDS-atomic and load rates, so
// long queues are histogrammed, counted and gathered by many workgroups (1,024 entries each) and only
// the final sort + walk over the nb winners runs in one workgroup.
constexpr int kFqThreads = 1024;    // (one entry per thread: what a workgroup spends its time on is the bins)
constexpr int kFqTile = 1024;       // queue entries per workgroup
constexpr int kFqLevelBits = 14;    // bits of match length resolved per histogram kernel (prompts of up to 16,383 tokens: one level)
constexpr int kFqBins = 1 << kFqLevelBits;
constexpr int kFqMaxLevels = 5;     // 31 bits of score (+ 32 bits of tie key) at most
constexpr int kFqSingleBlockN = 8192;  // shorter queues are cheaper in the single-workgroup kernel

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

struct FqMeta {        // zeroed before every call
    uint64_t fixed_hi; // decided high bits of the nb-th largest goodness
    int32_t violated;  // arrival order broken, or a score above the caller's bound
    int32_t need;      // winners still to be found among the entries that share fixed_hi
    int32_t done[kFqMaxLevels + 1];  // finished workgroups per kernel
};

struct FqWs {
    FqMeta *meta;
    uint32_t *hist;      // [kFqMaxLevels][kFqBins]
    int32_t *blockcnt;   // [n_blocks][2]: entries above g*, entries equal to g*
    uint64_t *cand;      // [kFifoMaxBatch] winners as inverted goodness (no tie keys: with the index below it)
    uint32_t *cand_idx;  // [kFifoMaxBatch] with tie keys: the winners' indices
};

__device__ __forceinline__ bool fq_last_block(int32_t *counter) {
    __shared__ int s_last;
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        s_last = (atomicAdd(counter, 1) == (int)gridDim.x - 1) ? 1 : 0;
    }
    __syncthreads();
    if (s_last) __threadfence();
    return s_last != 0;
}

// Histogram of one digit (up to 14 bits) of the goodness values that share the digits fixed so far; level 0
// also checks the arrival order.  The last workgroup to finish fixes the digit of the nb-th largest.
template <bool TIE>
__global__ __launch_bounds__(kFqThreads) void k_fq_hist(const uint64_t *__restrict__ arrival, FqKey<TIE> key, LiveN nn,
                                                       int32_t batch, int32_t max_match, int level, int shift, int width,
                                                       FqWs ws) {
    using G = typename FqKey<TIE>::G;
    const int32_t n = nn.get();
    __shared__ uint32_t h[kFqBins];
    __shared__ int32_t part[kFqThreads / kWave];
    __shared__ int32_t s_viol, s_pick, s_above;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    // (the top digit only reaches as far as the caller's bound on the scores does)
    const int nbins = (level == 0 && !TIE && (max_match >> shift) + 1 < (1 << width)) ? (max_match >> shift) + 1 : (1 << width);
    for (int i = tid; i < nbins; i += kFqThreads) h[i] = 0;
    if (tid == 0) { s_viol = 0; s_pick = 0; s_above = 0; }
    __syncthreads();
    const G fixed_hi = (level == 0) ? (G)0 : (G)ws.meta->fixed_hi;
    const int32_t base = blockIdx.x * kFqTile;
    bool viol = false;
#pragma unroll
    for (int r = 0; r < kFqTile / kFqThreads; ++r) {
        int32_t i = base + r * kFqThreads + tid;
        bool in = i < n;
        int32_t m = 0;
        const G g = in ? key.at(i, m) : (G)0;
        if (level == 0 && in) {
            viol |= m > max_match;
            viol |= (i + 1 < n) && (arrival[i] > arrival[i + 1]);
        }
        in = in && (level == 0 || (g >> (shift + width)) == fixed_hi);  // (level > 0: shift + width < bits of G)
        int32_t bin = (int32_t)((g >> shift) & (G)((1 << width) - 1));
        // lanes that share the first active lane's bin are added once (scores cluster and same-address
        // LDS atomics serialise)
        uint64_t act = __ballot(in);
        if (act) {
            int32_t lead = __shfl(bin, (int)__builtin_ctzll(act));
            uint64_t same = __ballot(in && bin == lead);
            if (in && bin == lead) {
                if (lane == (int)__builtin_ctzll(same)) atomicAdd(&h[bin], (uint32_t)__popcll(same));
            } else if (in) {
                atomicAdd(&h[bin], 1u);
            }
        }
    }
    if (viol) atomicOr(&s_viol, 1);
    __syncthreads();
    if (tid == 0 && s_viol) atomicOr(&ws.meta->violated, 1);
    uint32_t *gh = ws.hist + (size_t)level * kFqBins;
    for (int i = tid; i < nbins; i += kFqThreads) {
        uint32_t c = h[i];
        if (c) atomicAdd(&gh[i], c);
    }
    if (!fq_last_block(&ws.meta->done[level])) return;
    // suffix counts over the bins, top down: thread t owns a contiguous run of bins counted from the top
    const int per = (nbins + kFqThreads - 1) / kFqThreads;
    const int32_t nb = batch < n ? batch : n;
    const int32_t need = (level == 0) ? nb : ws.meta->need;
    // (after the fence of fq_last_block plain loads see the other workgroups' atomics)
    constexpr int kMaxPer = kFqBins / kFqThreads;
    int32_t c[kMaxPer];
    int32_t mine = 0;
#pragma unroll
    for (int q = 0; q < kMaxPer; ++q) {
        int b = nbins - 1 - (tid * per + q);
        c[q] = (q < per && b >= 0) ? (int32_t)gh[b] : 0;
        mine += c[q];
    }
    int32_t all;
    int32_t run = block_inclusive_scan<int32_t, kFqThreads>(mine, part, tid, all) - mine;  // entries in higher bins
#pragma unroll
    for (int q = 0; q < kMaxPer; ++q) {
        int b = nbins - 1 - (tid * per + q);
        if (q < per && b >= 0) {
            if (run < need && run + c[q] >= need) { s_pick = b; s_above = run; }
            run += c[q];
        }
    }
    __syncthreads();
    if (tid == 0) {
        ws.meta->fixed_hi = ((uint64_t)fixed_hi << width) | (uint64_t)(uint32_t)s_pick;
        ws.meta->need = need - s_above;
    }
}

// Per workgroup: how many of its entries lie above g* and how many equal it.
template <bool TIE>
__global__ __launch_bounds__(kFqThreads) void k_fq_count(FqKey<TIE> key, LiveN nn, FqWs ws) {
    using G = typename FqKey<TIE>::G;
    const int32_t n = nn.get();
    __shared__ int32_t s_gt, s_eq;
    const int tid = threadIdx.x;
    if (tid == 0) { s_gt = 0; s_eq = 0; }
    __syncthreads();
    const G g_star = (G)ws.meta->fixed_hi;
    const int32_t base = blockIdx.x * kFqTile;
    int32_t gt = 0, eq = 0;
#pragma unroll
    for (int r = 0; r < kFqTile / kFqThreads; ++r) {
        int32_t i = base + r * kFqThreads + tid;
        int32_t m;
        const bool in = i < n;
        const G g = in ? key.at(i, m) : (G)0;
        gt += (int32_t)__popcll(__ballot(in && g > g_star));
        eq += (int32_t)__popcll(__ballot(in && g == g_star));
    }
    if ((tid & (kWave - 1)) == 0) { atomicAdd(&s_gt, gt); atomicAdd(&s_eq, eq); }
    __syncthreads();
    if (tid == 0) { ws.blockcnt[2 * blockIdx.x] = s_gt; ws.blockcnt[2 * blockIdx.x + 1] = s_eq; }
}

// Winners = every entry above g* and the first `need` entries (by index) equal to g*; written in
// index order at positions given by prefix counts (no atomics).
template <bool TIE>
__global__ __launch_bounds__(kFqThreads) void k_fq_gather(FqKey<TIE> key, LiveN nn, FqWs ws) {
    using G = typename FqKey<TIE>::G;
    const int32_t n = nn.get();
    __shared__ int32_t part[kFqThreads / kWave];
    __shared__ int32_t s_rank, s_out;
    __shared__ int32_t w_eq[kFqThreads / kWave], w_win[kFqThreads / kWave];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave;
    const G g_star = (G)ws.meta->fixed_hi;
    const int32_t need = ws.meta->need;
    // entries equal to g* and winners in the workgroups before this one
    {
        int32_t eq_b = 0, gt_b = 0;
        for (int32_t b = tid; b < (int32_t)blockIdx.x; b += kFqThreads) {
            gt_b += ws.blockcnt[2 * b];
            eq_b += ws.blockcnt[2 * b + 1];
        }
        int32_t eq_all, gt_all;
        block_inclusive_scan<int32_t, kFqThreads>(eq_b, part, tid, eq_all);
        block_inclusive_scan<int32_t, kFqThreads>(gt_b, part, tid, gt_all);
        if (tid == 0) {
            s_rank = eq_all;
            s_out = gt_all + (eq_all < need ? eq_all : need);
        }
        __syncthreads();
    }
    int32_t rank = s_rank, out = s_out;
    const int32_t base = blockIdx.x * kFqTile;
    for (int r = 0; r < kFqTile / kFqThreads; ++r) {
        int32_t i = base + r * kFqThreads + tid;
        bool in = i < n;
        int32_t m = 0;
        const G g = in ? key.at(i, m) : (G)0;
        bool is_eq = in && g == g_star;
        uint64_t eqmask = __ballot(is_eq);
        // this row: counts of the wavefronts before mine
        __syncthreads();
        if (lane == 0) w_eq[wv] = (int32_t)__popcll(eqmask);
        __syncthreads();
        int32_t eq_before = 0, eq_row = 0;
        for (int w = 0; w < kFqThreads / kWave; ++w) {
            if (w < wv) eq_before += w_eq[w];
            eq_row += w_eq[w];
        }
        int32_t my_rank = rank + eq_before + (int32_t)__popcll(eqmask & ((1ull << lane) - 1ull));
        bool win = in && (g > g_star || (is_eq && my_rank < need));
        uint64_t wmask = __ballot(win);
        __syncthreads();
        if (lane == 0) w_win[wv] = (int32_t)__popcll(wmask);
        __syncthreads();
        int32_t win_before = 0, win_row = 0;
        for (int w = 0; w < kFqThreads / kWave; ++w) {
            if (w < wv) win_before += w_win[w];
            win_row += w_win[w];
        }
        if (win) {
            int32_t at = out + win_before + (int32_t)__popcll(wmask & ((1ull << lane) - 1ull));
            if (at >= 0 && at < kFifoMaxBatch) {
                if (TIE) {
                    ws.cand[at] = ~(uint64_t)g;
                    ws.cand_idx[at] = (uint32_t)i;
                } else {
                    ws.cand[at] = ((uint64_t)(0x7FFFFFFFu - (uint32_t)m) << 32) | (uint64_t)(uint32_t)i;
                }
            }
        }
        rank += eq_row;
        out += win_row;
    }
}

// Sort the nb winners by (-score, [tie key,] index) in LDS and run the two-cursor walk.
template <bool TIE>
__global__ __launch_bounds__(kFifoThreads) void k_fq_finish(LiveN nn, KArg ka, int32_t batch, FqWs ws,
                                                            uint32_t *__restrict__ phase_inout,
                                                            int32_t *__restrict__ batch_idx,
                                                            int32_t *__restrict__ n_selected) {
    __shared__ uint64_t cand[kFifoMaxBatch];
    __shared__ uint32_t l_elem[kFifoMaxBatch];
    __shared__ uint32_t a_in_l[kFifoMaxBatch];
    const int tid = threadIdx.x;
    // one round trip: the scalars, the verdict of the order check and this thread's winners (the
    // winner arrays hold kFifoMaxBatch entries whatever nb is; what lies past nb is not used)
    constexpr int kPer = kFifoMaxBatch / kFifoThreads;
    const int32_t n = nn.get();
    const uint32_t k = ka.get();
    const uint32_t phase_in = *phase_inout;
    const int32_t violated = ws.meta->violated;
    uint64_t own[kPer];
    uint32_t own_idx[kPer];
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
        own[c] = ws.cand[tid + c * kFifoThreads];
        own_idx[c] = TIE ? ws.cand_idx[tid + c * kFifoThreads] : 0u;
    }
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
    int32_t np2 = 1;
    while (np2 < nb) np2 <<= 1;
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
        const int32_t i = tid + c * kFifoThreads;
        if (i < np2) {
            cand[i] = (i < nb) ? own[c] : ~0ull;
            if (TIE) l_elem[i] = (i < nb) ? own_idx[c] : 0xFFFFFFFFu;  // second key word: the index
        }
    }
    __syncthreads();
    sort_lds<kFifoThreads, kFifoMaxBatch / kFifoThreads, TIE>(cand, l_elem, np2, tid);
    for (int32_t p = tid; p < nb; p += kFifoThreads) {
        if (!TIE) l_elem[p] = (uint32_t)cand[p];
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
    if (tid >= kWave) return;
    FifoAcc acc{l_elem, a_in_l};
    two_cursor_walk(acc, nb, nb, k, phase, batch_idx, tid);
}

// FCFS on an arrival-ordered queue: its first nb entries (after the order check of the histogram kernel).
__global__ __launch_bounds__(256) void k_fq_fcfs(LiveN nn, int32_t batch, FqWs ws, uint32_t *__restrict__ phase_inout,
                                                 int32_t *__restrict__ batch_idx, int32_t *__restrict__ n_selected) {
    const int32_t n = nn.get();
    const int32_t nb = batch < n ? batch : n;
    if (ws.meta->violated) {
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

// Zeroes the meta block and the histograms (a kernel rather than a memset node, so that the whole
// selection can be captured into a HIP graph and replayed).
__global__ __launch_bounds__(256) void k_fq_zero(uint32_t *__restrict__ p, int32_t n_words) {
    for (int32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += gridDim.x * blockDim.x) p[i] = 0u;
}

static void carve_fq(FqWs &f, char *base, int32_t n, size_t *used) {
    size_t o = 0;
    auto take = [&](size_t bytes) { void *p = base ? base + o : nullptr; o += align_up(bytes, 256); return p; };
    int32_t nblk = (n + kFqTile - 1) / kFqTile;
    if (nblk < 1) nblk = 1;
    f.meta = (FqMeta *)take(sizeof(FqMeta));
    f.hist = (uint32_t *)take((size_t)kFqMaxLevels * kFqBins * 4);
    f.blockcnt = (int32_t *)take((size_t)nblk * 8);
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
    const int32_t nblk = (nn.n + kFqTile - 1) / kFqTile;
    // meta and histograms are contiguous at the start of the workspace
    const int32_t zero_words = (int32_t)(((char *)f.blockcnt - (char *)f.meta) / 4);
    hipLaunchKernelGGL(k_fq_zero, dim3(32), dim3(256), 0, stream, (uint32_t *)f.meta, zero_words);
    int mbits = 0;
    while (mbits < 31 && (max_match >> mbits) != 0) ++mbits;
    if (mbits == 0) mbits = 1;
    const bool fcfs = (!k.dev && k.k == 1u);  // (a k read on the device takes the general kernels)
    int shift = mbits + (TIE ? 32 : 0), level = 0;
    while (shift > 0 && level < kFqMaxLevels) {
        int width = shift < kFqLevelBits ? shift : kFqLevelBits;
        shift -= width;
        hipLaunchKernelGGL(k_fq_hist<TIE>, dim3(nblk), dim3(kFqThreads), 0, stream, arrival, key, n, batch, max_match,
                           level, shift, width, f);
        ++level;
        if (fcfs) break;  // only the order check of level 0 is needed
    }
    if (fcfs) {
        hipLaunchKernelGGL(k_fq_fcfs, dim3((nb + 255) / 256), dim3(256), 0, stream, n, batch, f, phase_inout, batch_idx,
                           n_selected);
        return check_launch();
    }
    hipLaunchKernelGGL(k_fq_count<TIE>, dim3(nblk), dim3(kFqThreads), 0, stream, key, n, f);
    hipLaunchKernelGGL(k_fq_gather<TIE>, dim3(nblk), dim3(kFqThreads), 0, stream, key, n, f);
    hipLaunchKernelGGL(k_fq_finish<TIE>, dim3(1), dim3(kFifoThreads), 0, stream, n, k, batch, f, phase_inout, batch_idx,
                       n_selected);
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
                        hipStream_t stream, SelectOrders *out) {
    SelectWs ws;
    size_t need = 0;
    carve(ws, (char *)workspace, n, &need);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return KLPM_EARENA;
    const LiveN nn{n, n_live};
    const uint32_t *order_a = ws.val_a, *order_l = ws.val_a;
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
