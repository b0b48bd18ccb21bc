// GEMM and row-wise kernels of the layer stack (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace climber {

enum { EPI_STORE_BF16 = 0, EPI_GELU_BF16 = 1, EPI_RESID_F32 = 2 };

// W [K][N] bf16 row-major -> MFMA B-operand fragments (same byte size).  K % 16 == 0, N % 32 == 0.
hipError_t pack_weight(const void *w, void *packed, int K, int N, hipStream_t s);

// Several weights in one launch (n <= kMaxPackJobs): job i packs w[i] [K[i]][N[i]] into packed[i].
constexpr int kMaxPackJobs = 16;
struct PackJobs {
    const void *w[kMaxPackJobs];
    void *packed[kMaxPackJobs];
    int K[kMaxPackJobs], N[kMaxPackJobs];
    int n;
};
hipError_t pack_weights(const PackJobs &jobs, hipStream_t s);

// C = A W (+ epilogue).  A: bf16 [M][lda]; w_packed from pack_weight; N % 128 == 0, K % 64 == 0.
// EPI_STORE_BF16 / EPI_GELU_BF16: C is bf16 [M][ldc].  EPI_RESID_F32: C is fp32, C = acc + resid.
hipError_t gemm_bf16(int epi, const void *A, int64_t lda, const void *w_packed, int M, int N, int K,
                     void *C, int64_t ldc, const float *resid, int64_t ldr, hipStream_t s);

// y[r][:] = bf16( x[r][:] / sqrt(mean(x[r]^2) + eps) * g[:] ),  x fp32 [rows][d], g bf16 [d]
hipError_t rmsnorm_to_bf16(const float *x, const void *g, void *y, int64_t rows, int d, float eps,
                           hipStream_t s);
// the same from bf16 rows, which are also widened into the fp32 residual stream x32 (first layer)
hipError_t rmsnorm_from_bf16(const void *x, const void *g, void *y, float *x32, int64_t rows, int d,
                             float eps, hipStream_t s);

}  // namespace climber
