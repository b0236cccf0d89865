// Bitonic sort of a short array in LDS by a whole workgroup.
//
// The compare-exchange steps whose partner lies within the wavefront (distance < 64) run on
// registers with cross-lane moves and no barrier; only the steps at distance >= 64 go through LDS
// with a barrier each.  For 1,024 entries that is 15 barriers instead of 55.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace klpm {

// One compare-exchange step of the network for the entry at position i, held in (k, l); the partner
// sits st lanes away (st < 64).  Pairs inside blocks of `size` entries are ordered upwards when bit
// `size` of the position is clear, downwards otherwise.
template <bool HAS_LO>
__device__ __forceinline__ void bitonic_lane_step(uint64_t &k, uint32_t &l, int32_t i, int32_t size, int32_t st) {
    const uint64_t ok = (uint64_t)__shfl_xor((unsigned long long)k, st);
    const uint32_t ol = HAS_LO ? (uint32_t)__shfl_xor((int)l, st) : 0u;
    const bool up = (i & size) == 0;
    const bool lower = (i & st) == 0;
    const bool mine_gt = k > ok || (HAS_LO && k == ok && l > ol);
    const bool other_gt = ok > k || (HAS_LO && ok == k && ol > l);
    const bool a_gt_b = lower ? mine_gt : other_gt;  // a = the lower position of the pair
    if (a_gt_b == up) {
        k = ok;
        l = ol;
    }
}

// Sorts hi[0..np2) ascending (np2 a power of two; with HAS_LO by (hi, lo), lo moving along).  Every
// thread of the workgroup calls it after a barrier behind the writes that filled the arrays; it
// returns after a barrier.
template <int THREADS, bool HAS_LO>
__device__ __forceinline__ void bitonic_sort_lds(uint64_t *hi, uint32_t *lo, int32_t np2, int tid) {
    constexpr int kLanes = 64;
    const int32_t first = np2 < kLanes ? np2 : kLanes;
    // blocks of up to 64 entries: every step stays inside a wavefront
    for (int32_t i = tid; i < np2; i += THREADS) {
        uint64_t k = hi[i];
        uint32_t l = HAS_LO ? lo[i] : 0u;
        for (int32_t size = 2; size <= first; size <<= 1)
            for (int32_t st = size >> 1; st > 0; st >>= 1) bitonic_lane_step<HAS_LO>(k, l, i, size, st);
        hi[i] = k;
        if (HAS_LO) lo[i] = l;
    }
    __syncthreads();
    for (int32_t size = 2 * kLanes; size <= np2; size <<= 1) {
        for (int32_t stride = size >> 1; stride >= kLanes; stride >>= 1) {
            for (int32_t t = tid; t < (np2 >> 1); t += THREADS) {
                const int32_t a = 2 * t - (t & (stride - 1));
                const int32_t b = a + stride;
                const bool up = (a & size) == 0;
                const uint64_t ha = hi[a], hb = hi[b];
                if (HAS_LO) {
                    const uint32_t la = lo[a], lb = lo[b];
                    const bool gt = ha > hb || (ha == hb && la > lb);
                    if (gt == up) { hi[a] = hb; hi[b] = ha; lo[a] = lb; lo[b] = la; }
                } else {
                    if ((ha > hb) == up) { hi[a] = hb; hi[b] = ha; }
                }
            }
            __syncthreads();
        }
        for (int32_t i = tid; i < np2; i += THREADS) {
            uint64_t k = hi[i];
            uint32_t l = HAS_LO ? lo[i] : 0u;
#pragma unroll
            for (int32_t st = kLanes >> 1; st > 0; st >>= 1) bitonic_lane_step<HAS_LO>(k, l, i, size, st);
            hi[i] = k;
            if (HAS_LO) lo[i] = l;
        }
        __syncthreads();
    }
}

}  // namespace klpm
