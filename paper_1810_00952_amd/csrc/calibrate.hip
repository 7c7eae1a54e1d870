// Measurement aid: what the matrix pipes of this chip deliver when nothing else is in the way.  Every wave runs a
// chain of bf16 MFMAs (32x32x16, fp32 accumulate) on register operands, four independent accumulator tiles per wave
// so that no MFMA waits for the one before it, eight waves per workgroup and two workgroups per CU (four waves per
// SIMD).  No memory traffic apart from one store per lane at the end (which keeps the chain alive for the compiler).
// The rate this kernel reaches is the ceiling the contraction kernels are held against, next to the quoted peak.
#include "device_utils.h"

namespace rl {

__global__ __launch_bounds__(512) void mfma_peak_kernel(float *out, int32_t iters)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const int lane = threadIdx.x & 63;
    u32x4 a = {0x3f803f80u + (uint32_t)lane, 0x3f803f80u, 0x3f003f00u, 0x3e803e80u};
    u32x4 b = {0x3f803f80u, 0x3f003f00u + (uint32_t)lane, 0x3f803f80u, 0x3e803e80u};
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc[i], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
#endif
}

// grid workgroups of 512 threads, each wave issuing 16 * iters MFMAs of 32 x 32 x 16 x 2 flops
hipError_t launch_mfma_peak(float *out, int32_t grid, int32_t iters, hipStream_t s)
{
    if (!out || grid < 1 || iters < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(mfma_peak_kernel, dim3((unsigned)grid), dim3(512), 0, s, out, iters);
    return hipGetLastError();
}

}  // namespace rl
