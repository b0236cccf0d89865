// Reductions across the 64 lanes of a wavefront.  A workgroup that wants one total adds the
// wavefronts' results in LDS: atomics of every thread on one LDS word are served one by one
// (about 5 ns each), so 1,024 threads adding to one counter cost more than the rest of a short kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace klpm {

// Sum over the wavefront; lane 0 holds the result.  Every lane of the wavefront must call it.
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_down(v, d);
    return v;
}
// Maximum over the wavefront; lane 0 holds the result.
template <typename T>
__device__ __forceinline__ T wave_max(T v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const T o = __shfl_down(v, d);
        v = o > v ? o : v;
    }
    return v;
}

}  // namespace klpm
