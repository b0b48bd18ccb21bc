// Row-wise kernels of the layer stack: RMSNorm (fp32 residual stream -> bf16 GEMM operand) and the
// bf16 -> fp32 widening of the input embeddings.
#include "gemm.h"

namespace climber {
namespace {

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

__global__ __launch_bounds__(256) void cast_kernel(const __bf16 *x, float *y, int64_t n8)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        const uint4 raw = ((const uint4 *)x)[i];
        const __bf16 *b = (const __bf16 *)&raw;
        float4 lo = {(float)b[0], (float)b[1], (float)b[2], (float)b[3]};
        float4 hi = {(float)b[4], (float)b[5], (float)b[6], (float)b[7]};
        ((float4 *)y)[2 * i] = lo;
        ((float4 *)y)[2 * i + 1] = hi;
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

hipError_t cast_bf16_to_f32(const void *x, float *y, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    if (n % 8 != 0) return hipErrorInvalidValue;
    const int64_t n8 = n / 8, blocks = (n8 + 255) / 256;
    hipLaunchKernelGGL(cast_kernel, dim3((unsigned)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, s,
                       (const __bf16 *)x, y, n8);
    return hipGetLastError();
}

}  // namespace climber
