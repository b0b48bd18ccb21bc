// Row-wise kernels of the layer stack.  RMSNorm itself is folded into the projections (gemm.h); what
// is left is the preparation of the rows a stack call starts from.
#include "gemm.h"

namespace climber {
namespace {

typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;

// one wavefront per row
// Row preparation for a projection that applies the RMSNorm scale in its epilogue: sum of squares
// of the row into ss[row][0] (the other partial slots are cleared), plus the copy of the row in the
// other precision.  BF16_IN: x bf16 -> x32 fp32;  otherwise: x fp32 -> xb bf16.
template <bool BF16_IN>
__global__ __launch_bounds__(256) void row_prep_kernel(const void *x, void *copy, float *ss, int n_part,
                                                       int64_t rows, int d)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    float acc = 0.f;
    for (int e = lane * 4; e < d; e += 256) {
        float4 f;
        if (BF16_IN) {
            const bf16x4 v = *(const bf16x4 *)((const __bf16 *)x + row * d + e);
            f = float4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
            *(float4 *)((float *)copy + row * d + e) = f;
        } else {
            f = *(const float4 *)((const float *)x + row * d + e);
            bf16x4 o;
            o[0] = (__bf16)f.x; o[1] = (__bf16)f.y; o[2] = (__bf16)f.z; o[3] = (__bf16)f.w;
            *(bf16x4 *)((__bf16 *)copy + row * d + e) = o;
        }
        acc += f.x * f.x + f.y * f.y + f.z * f.z + f.w * f.w;
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane < n_part) ss[row * n_part + lane] = lane == 0 ? acc : 0.f;
}

}  // namespace

hipError_t row_prep_bf16(const void *x, float *x32, float *ss, int n_part, int64_t rows, int d, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    if (d % 4 != 0 || n_part < 1 || n_part > 64) return hipErrorInvalidValue;
    hipLaunchKernelGGL(row_prep_kernel<true>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, x,
                       (void *)x32, ss, n_part, rows, d);
    return hipGetLastError();
}

hipError_t row_prep_f32(const float *x, void *xb, float *ss, int n_part, int64_t rows, int d, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    if (d % 4 != 0 || n_part < 1 || n_part > 64) return hipErrorInvalidValue;
    hipLaunchKernelGGL(row_prep_kernel<false>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                       (const void *)x, xb, ss, n_part, rows, d);
    return hipGetLastError();
}

}  // namespace climber
