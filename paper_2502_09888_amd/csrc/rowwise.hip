// Row-wise kernels of the layer stack: RMSNorm (fp32 residual stream -> bf16 GEMM operand), also
// straight from the bf16 input embeddings (which it widens into the fp32 stream on the way).
#include "gemm.h"

namespace climber {
namespace {

typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;

// one wavefront per row
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *x, const __bf16 *g, __bf16 *y,
                                                      int64_t rows, int d, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float *xr = x + row * d;
    float ss = 0.f;
    for (int e = lane * 4; e < d; e += 256) {
        const float4 v = *(const float4 *)(xr + e);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    const float r = 1.f / sqrtf(ss / (float)d + eps);
    __bf16 *yr = y + row * d;
    for (int e = lane * 4; e < d; e += 256) {
        const float4 v = *(const float4 *)(xr + e);
        __attribute__((aligned(8))) __bf16 out[4];
        out[0] = (__bf16)(v.x * r * (float)g[e]);
        out[1] = (__bf16)(v.y * r * (float)g[e + 1]);
        out[2] = (__bf16)(v.z * r * (float)g[e + 2]);
        out[3] = (__bf16)(v.w * r * (float)g[e + 3]);
        *(uint2 *)(yr + e) = *(const uint2 *)out;
    }
}

// the same for bf16 input rows, which are also widened into the fp32 residual stream
__global__ __launch_bounds__(256) void rmsnorm_bf16_kernel(const __bf16 *x, const __bf16 *g, __bf16 *y,
                                                           float *x32, int64_t rows, int d, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const __bf16 *xr = x + row * d;
    float ss = 0.f;
    for (int e = lane * 4; e < d; e += 256) {
        const bf16x4 v = *(const bf16x4 *)(xr + e);
        const float4 f = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
        ss += f.x * f.x + f.y * f.y + f.z * f.z + f.w * f.w;
        *(float4 *)(x32 + row * d + e) = f;
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    const float r = 1.f / sqrtf(ss / (float)d + eps);
    __bf16 *yr = y + row * d;
    for (int e = lane * 4; e < d; e += 256) {
        const bf16x4 v = *(const bf16x4 *)(xr + e);
        bf16x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = (__bf16)((float)v[i] * r * (float)g[e + i]);
        *(bf16x4 *)(yr + e) = out;
    }
}

}  // namespace

hipError_t rmsnorm_to_bf16(const float *x, const void *g, void *y, int64_t rows, int d, float eps,
                           hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    if (d % 4 != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rmsnorm_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, x,
                       (const __bf16 *)g, (__bf16 *)y, rows, d, eps);
    return hipGetLastError();
}

hipError_t rmsnorm_from_bf16(const void *x, const void *g, void *y, float *x32, int64_t rows, int d,
                             float eps, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    if (d % 4 != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rmsnorm_bf16_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                       (const __bf16 *)x, (const __bf16 *)g, (__bf16 *)y, x32, rows, d, eps);
    return hipGetLastError();
}

}  // namespace climber
