// A plain streaming read over a buffer: the reference point for what a read-bound kernel can reach
// on this GPU (the match kernel's bandwidth figures are set beside it).
#include "klpm_internal.hpp"

namespace klpm {

__global__ __launch_bounds__(256) void k_probe_read(const uint4 *__restrict__ src, int64_t n_vec,
                                                    unsigned long long *__restrict__ sink) {
    uint32_t acc = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    // four independent 16-byte loads per trip
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n_vec; i += stride) {
        const uint4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    // one word per wavefront leaves the kernel, so the loads cannot be dropped
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) acc ^= (uint32_t)__shfl_xor((int)acc, d);
    if ((threadIdx.x & (kWave - 1)) == 0 && acc == 0xFFFFFFFFu) atomicAdd(sink, 1ull);
}

}  // namespace klpm

using namespace klpm;

extern "C" int kLPM_probe_read(const void *src, size_t bytes, uint64_t *sink, kLPM_stream stream) {
    if (!src || !sink || ((uintptr_t)src & 15u) || bytes < 16) return KLPM_EINVAL;
    const int64_t n_vec = (int64_t)(bytes / 16);
    hipLaunchKernelGGL(k_probe_read, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src, n_vec,
                       (unsigned long long *)sink);
    return check_launch();
}
