// MFMA-only probe: what bf16 matrix rate does the device sustain at its own clocks?  A measurement
// aid for the roofline of the attention kernels of Climber (arXiv 2502.09888, Eq. (3): Q K^T and
// A V are dense contractions); not a step of the method.
#include "../../include/climber.h"

#include <hip/hip_runtime.h>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__global__ __launch_bounds__(256) void mfma_probe_kernel(float *sink, int iters)
{
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((threadIdx.x + e) % 7 - 3);
        b[e] = (__bf16)(0.125f * (float)((threadIdx.x * 3 + e) % 5 - 2));
    }
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
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
    if (workgroups < 1 || workgroups > 65536 || iters < 1) return CLIMBER_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream,
                       sink, (int)iters);
    return hipGetLastError() == hipSuccess ? CLIMBER_OK : CLIMBER_ERR_RUNTIME;
}
