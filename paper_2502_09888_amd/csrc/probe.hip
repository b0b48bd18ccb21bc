// MFMA-only probe: what bf16 matrix rate does the device sustain at its own clocks?  A measurement
// aid for the roofline of the attention kernels of Climber (arXiv 2502.09888, Eq. (3): Q K^T and
// A V are dense contractions); not a step of the method.
#include "../../include/climber.h"

#include <hip/hip_runtime.h>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__device__ __forceinline__ unsigned mix(unsigned x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// Operands are pseudo-random values of unit scale (all mantissa bits in play) and rotate between
// MFMAs: the sustained clock, and with it the rate, depends on how many operand bits toggle
// (measured: ~1.64 PFLOP/s with such data against ~2.1 PFLOP/s with small-integer operands).
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *sink, int iters)
{
    bf16x8 a[4], b[4];
    for (int v = 0; v < 4; ++v)
        for (int e = 0; e < 8; ++e) {
            const unsigned h1 = mix(threadIdx.x * 64 + v * 8 + e + blockIdx.x * 977), h2 = mix(h1 + 12345);
            a[v][e] = (__bf16)(((h1 & 0xffff) / 65536.f - 0.5f) * 3.4f);
            b[v][e] = (__bf16)(((h2 & 0xffff) / 65536.f - 0.5f) * 3.4f);
        }
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + u) & 3], b[(i + 2 * u + 1) & 3], acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" int climber_probe_mfma(int32_t workgroups, int32_t iters, float *sink, void *stream)
{
    if (!sink) return CLIMBER_ERR_NULL;
    if (workgroups < 1 || workgroups > 65536 || iters < 4 || iters % 4 != 0) return CLIMBER_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream,
                       sink, (int)iters);
    return hipGetLastError() == hipSuccess ? CLIMBER_OK : CLIMBER_ERR_RUNTIME;
}
