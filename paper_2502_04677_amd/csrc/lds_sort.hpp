// Sort of a short array in LDS by a whole workgroup: runs of 64 entries are sorted on registers
// (a bitonic network whose every partner sits in the same wavefront: cross-lane moves with immediate patterns, no barrier),
// then runs are merged pairwise, every entry finding its place in the merged run by a binary search
// in the partner run.  A 1,024-entry sort is 21 register steps and 4 merge levels (34 dependent LDS
// reads, 9 barriers); the plain bitonic network in LDS it replaces took 55 steps with a barrier each.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace klpm {

// The value of `v` held by the lane whose number differs in bit ST (ST = 1 .. 32): a swizzle with
// an immediate pattern inside each half of the wavefront, a permute through a prepared byte
// address ((lane ^ 32) * 4) across the halves.
template <int ST>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v, int addr32) {
    if constexpr (ST == 32) {
        return (uint32_t)__builtin_amdgcn_ds_bpermute(addr32, (int)v);
    } else {
        return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (ST << 10) | 0x1F);  // and 0x1F, or 0, xor ST
    }
}

// One compare-exchange step of a bitonic network on registers: the entry (k, l) of this lane
// against the one ST lanes away; `up` = this pair is ordered upwards (the lower lane keeps the
// smaller entry).
template <bool HAS_LO, int ST>
__device__ __forceinline__ void lane_step(uint64_t &k, uint32_t &l, int lane, bool up, int addr32) {
    const uint32_t o0 = lane_xor<ST>((uint32_t)k, addr32), o1 = lane_xor<ST>((uint32_t)(k >> 32), addr32);
    const uint64_t ok = ((uint64_t)o1 << 32) | (uint64_t)o0;
    const uint32_t ol = HAS_LO ? lane_xor<ST>(l, addr32) : 0u;
    const bool want_min = ((lane & ST) == 0) == up;
    const bool other_lt = ok < k || (HAS_LO && ok == k && ol < l);
    const bool other_gt = ok > k || (HAS_LO && ok == k && ol > l);
    if (want_min ? other_lt : other_gt) {
        k = ok;
        l = ol;
    }
}
template <bool HAS_LO, int ST>
struct LaneMerge {  // the steps at distances ST, ST/2, .. 1
    static __device__ __forceinline__ void run(uint64_t &k, uint32_t &l, int lane, bool up, int addr32) {
        lane_step<HAS_LO, ST>(k, l, lane, up, addr32);
        if constexpr (ST > 1) LaneMerge<HAS_LO, ST / 2>::run(k, l, lane, up, addr32);
    }
};
// Bitonic sort of every aligned block of `first` lanes (a power of two, at most 64), all blocks
// upwards: blocks of 2, 4, .. SIZE are merged in turn, alternating direction below the last size.
template <bool HAS_LO, int SIZE>
struct LaneSort {
    static __device__ __forceinline__ void run(uint64_t &k, uint32_t &l, int lane, int32_t first, int addr32) {
        if constexpr (SIZE > 2) LaneSort<HAS_LO, SIZE / 2>::run(k, l, lane, first, addr32);
        if (SIZE <= first) LaneMerge<HAS_LO, SIZE / 2>::run(k, l, lane, SIZE == first || (lane & SIZE) == 0, addr32);
    }
};

// Sorts hi[0..np2) ascending (np2 a power of two, at most THREADS * MAX_PER; with HAS_LO by
// (hi, lo), lo moving along; equal entries keep no particular order).  Every thread of the
// workgroup calls it after a barrier behind the writes that filled the arrays; it returns after a
// barrier.
template <int THREADS, int MAX_PER, bool HAS_LO>
__device__ __forceinline__ void sort_lds(uint64_t *hi, uint32_t *lo, int32_t np2, int tid) {
    constexpr int kLanes = 64;
    static_assert(THREADS % kLanes == 0, "whole wavefronts");
    const int32_t first = np2 < kLanes ? np2 : kLanes;
    const int lane = tid & (kLanes - 1);
    const int addr32 = (lane ^ 32) << 2;
    for (int32_t i = tid; i < np2; i += THREADS) {  // (position i sits in lane i mod 64)
        uint64_t k = hi[i];
        uint32_t l = HAS_LO ? lo[i] : 0u;
        LaneSort<HAS_LO, kLanes>::run(k, l, lane, first, addr32);
        hi[i] = k;
        if (HAS_LO) lo[i] = l;
    }
    __syncthreads();
    for (int32_t len = kLanes; len < np2; len <<= 1) {
        uint64_t k[MAX_PER];
        uint32_t l[MAX_PER];
        int32_t dst[MAX_PER];
#pragma unroll
        for (int c = 0; c < MAX_PER; ++c) {
            const int32_t i = tid + c * THREADS;
            dst[c] = -1;
            if (i < np2) {
                k[c] = hi[i];
                l[c] = HAS_LO ? lo[i] : 0u;
                const bool second = (i & len) != 0;          // the entry sits in the second run of its pair
                const int32_t other = (i ^ len) & ~(len - 1);  // start of the partner run
                // partner entries that go before this one: the smaller ones, and for an entry of
                // the second run the equal ones too
                int32_t a = 0, b = len;
                while (a < b) {
                    const int32_t mid = (a + b) >> 1;
                    const uint64_t ok = hi[other + mid];
                    bool before;
                    if (HAS_LO) {
                        const uint32_t ol = lo[other + mid];
                        before = ok < k[c] || (ok == k[c] && (second ? ol <= l[c] : ol < l[c]));
                    } else {
                        before = second ? ok <= k[c] : ok < k[c];
                    }
                    if (before) a = mid + 1; else b = mid;
                }
                dst[c] = (i & ~(2 * len - 1)) + (i & (len - 1)) + a;
            }
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < MAX_PER; ++c) {
            if (dst[c] >= 0) {
                hi[dst[c]] = k[c];
                if (HAS_LO) lo[dst[c]] = l[c];
            }
        }
        __syncthreads();
    }
}

}  // namespace klpm
