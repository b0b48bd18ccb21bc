// bf16 MFMA GEMM for the projections of the layer stack (f_QKV and f_FFN of Eq. (3), Climber,
// arXiv 2502.09888): C[M][N] = A[M][K] * W[K][N] with fp32 accumulation and a fused epilogue
// (plain bf16 store, residual add into the fp32 stream, erf-GELU).
//
// W is first repacked (pack_weight) into B-operand fragments of v_mfma_f32_32x32x16_bf16:
//   chunk (nb, ks, lane), 16 B: W[16ks + 8(lane/32) + 0..7][32nb + lane%32]
// so that the GEMM copies it HBM -> LDS linearly and every wave reads a fragment as one
// conflict-free 16-byte-per-lane access.  A stays row-major; its LDS tile is XOR-swizzled in
// 16-byte chunks so that the fragment reads (32 rows, same k chunk) spread over all banks.
// Tile: 128 x 128 x 64 per 256-thread workgroup, 4 waves as 2 x 2, each 64 x 64 = 2 x 2 MFMA
// blocks, LDS double buffer (64 KiB), one barrier per k-tile.
#include "gemm.h"

namespace climber {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kStageBytes = (BM * BK + BN * BK) * 2;  // 32 KiB

__global__ __launch_bounds__(256) void pack_weight_kernel(const __bf16 *w, __bf16 *out, int K, int N)
{
    // one thread per 16-byte chunk (nb, ks, lane)
    const int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n_chunks = (int64_t)(N / 32) * (K / 16) * 64;
    if (chunk >= n_chunks) return;
    const int lane = (int)(chunk & 63);
    const int64_t t = chunk >> 6;
    const int ks = (int)(t % (K / 16)), nb = (int)(t / (K / 16));
    const int n = 32 * nb + (lane & 31), k0 = 16 * ks + 8 * (lane >> 5);
    __attribute__((aligned(16))) __bf16 v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = w[(int64_t)(k0 + e) * N + n];
    ((uint4 *)out)[chunk] = *(const uint4 *)v;
}

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752f)); }

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(const __bf16 *A, int64_t lda,
                                                           const __bf16 *Wp, int M, int N, int K,
                                                           void *C, int64_t ldc, const float *resid,
                                                           int64_t ldr)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * kStageBytes];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int n_kt = K / BK;
    const int64_t kchunks = (int64_t)(K / 16) * 64;  // 16-byte chunks per 32-column block of Wp

    // per-thread copy plan: 4 A chunks and 4 W chunks per k-tile
    const __bf16 *a_src[4];
    int a_dst[4];
    const uint4 *w_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = tid + 256 * i;
        const int row = q >> 3, c = q & 7;
        a_src[i] = A + (int64_t)min(m0 + row, M - 1) * lda + c * 8;
        a_dst[i] = row * 128 + ((c ^ (row & 7)) * 16);
        const int nbl = q >> 8, rem = q & 255;
        w_src[i] = (const uint4 *)Wp + ((int64_t)(n0 / 32 + nbl) * kchunks + rem);
    }
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 pa[4], pw[4];
    auto fetch = [&](int kt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pa[i] = *(const uint4 *)(a_src[i] + kt * BK);
            pw[i] = w_src[i][(int64_t)kt * 256];
        }
    };
    auto stash = [&](int buf) {
        uint8_t *base = lds + buf * kStageBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *(uint4 *)(base + a_dst[i]) = pa[i];
            ((uint4 *)(base + BM * BK * 2))[tid + 256 * i] = pw[i];
        }
    };
    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < n_kt; ++kt) {
        const uint8_t *sa = lds + (kt & 1) * kStageBytes;
        const uint8_t *sw = sa + BM * BK * 2;
        const bool more = kt + 1 < n_kt;
        if (more) fetch(kt + 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 af[2], bfr[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = 64 * wm + 32 * i + l32;
                af[i] = *(const bf16x8 *)(sa + row * 128 + (((2 * ks + hf) ^ (row & 7)) * 16));
                bfr[i] = *(const bf16x8 *)(sw + (((2 * wn + i) * 256) + ks * 64 + lane) * 16);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (more) stash((kt + 1) & 1);
        __syncthreads();
    }

    // epilogue: lane holds D[8(r/4) + 4hf + r%4][l32] of each 32 x 32 block
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + 64 * wn + 32 * j + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + 64 * wm + 32 * i + 8 * (r >> 2) + 4 * hf + (r & 3);
                if (row < M) {
                    const float v = acc[i][j][r];
                    if (EPI == EPI_STORE_BF16)
                        ((__bf16 *)C)[(int64_t)row * ldc + col] = (__bf16)v;
                    else if (EPI == EPI_GELU_BF16)
                        ((__bf16 *)C)[(int64_t)row * ldc + col] = (__bf16)gelu_erf(v);
                    else
                        ((float *)C)[(int64_t)row * ldc + col] = v + resid[(int64_t)row * ldr + col];
                }
            }
        }
}

}  // namespace

hipError_t pack_weight(const void *w, void *packed, int K, int N, hipStream_t s)
{
    const int64_t n_chunks = (int64_t)(N / 32) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, s,
                       (const __bf16 *)w, (__bf16 *)packed, K, N);
    return hipGetLastError();
}

hipError_t gemm_bf16(int epi, const void *A, int64_t lda, const void *w_packed, int M, int N, int K,
                     void *C, int64_t ldc, const float *resid, int64_t ldr, hipStream_t s)
{
    if (M <= 0) return hipSuccess;
    if (N % BN != 0 || K % BK != 0) return hipErrorInvalidValue;
    const dim3 grid(N / BN, (M + BM - 1) / BM), block(256);
    const __bf16 *a = (const __bf16 *)A, *w = (const __bf16 *)w_packed;
    switch (epi) {
    case EPI_STORE_BF16:
        hipLaunchKernelGGL(gemm_bf16_kernel<EPI_STORE_BF16>, grid, block, 0, s, a, lda, w, M, N, K, C, ldc, resid, ldr);
        break;
    case EPI_GELU_BF16:
        hipLaunchKernelGGL(gemm_bf16_kernel<EPI_GELU_BF16>, grid, block, 0, s, a, lda, w, M, N, K, C, ldc, resid, ldr);
        break;
    case EPI_RESID_F32:
        hipLaunchKernelGGL(gemm_bf16_kernel<EPI_RESID_F32>, grid, block, 0, s, a, lda, w, M, N, K, C, ldc, resid, ldr);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace climber
