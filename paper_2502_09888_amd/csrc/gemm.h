// GEMM and row-wise kernels of the layer stack (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace climber {

enum { EPI_STORE_BF16 = 0, EPI_GELU_BF16 = 1, EPI_RESID_F32 = 2, EPI_RELU_BF16 = 3 };

// RMSNorm folded into the projections around it.  A projection whose input is RMSNorm(x; g) runs on
// the plain bf16 rows of x with the gain folded into the weight rows (pack job with `gain`) and
// multiplies every output row by r = 1/sqrt(mean(x^2) + eps) in its epilogue (`in_norm`).  The
// projection that produces x (EPI_RESID_F32) writes, besides the fp32 rows, their bf16 copy and
// the sums of squares of its 64-column slices (`out_norm`); d/64 partial sums per row.
struct RowNormIn {          // consumer side; ss == nullptr: no scaling
    const float *ss;        // [rows][n_part] partial sums of squares of the input rows
    int n_part;
    float inv_d, eps;
};
struct RowNormOut {         // producer side; ss == nullptr: fp32 rows only
    float *ss;              // [rows][N/64]
    void *xb;               // bf16 copy of the output rows, [rows][ldb]
    int64_t ldb;
};

// W [K][N] bf16 row-major -> MFMA B-operand fragments (same byte size).  K % 16 == 0, N % 32 == 0.
hipError_t pack_weight(const void *w, void *packed, int K, int N, hipStream_t s);

// Several weights in one launch (n <= kMaxPackJobs): job i packs w[i] [K[i]][N[i]] into packed[i].
constexpr int kMaxPackJobs = 16;
struct PackJobs {
    const void *w[kMaxPackJobs];
    const void *gain[kMaxPackJobs];  // bf16 [K] multiplied into the rows of w, or nullptr
    void *packed[kMaxPackJobs];
    int K[kMaxPackJobs], N[kMaxPackJobs];
    int n;
};
hipError_t pack_weights(const PackJobs &jobs, hipStream_t s);

// Tiled activation layout (bf16, X columns): the rows are cut into groups of 16 and the columns into
// k-tiles of 32; piece (g, t) = 1 KiB at ((g * X/32) + t) * 1024, holding for row r of the group and
// 16-byte slot s (at r*64 + s*16) the 8 columns 32t + 8(s ^ (r >> 2)) ..: exactly the bytes one
// global->LDS copy of the consuming projection lands, so that the copy reads 1 KiB contiguous and
// the k-tiles of a row group follow each other in memory.  Buffers hold a multiple of 16 rows.
// Used for the FFN hidden (X = d_ffn: with row-major rows a copy would touch 16 rows 4 KiB apart).
enum { kTiledA = 1, kTiledC = 2 };

// Fused QKV projection of the history rows of a batch (all `rows` padded rows of the cache):
// output columns [0, d) (queries) go to C as rows of d, columns [d, 2d) and [2d, 3d) (keys, values)
// straight into the layer's bf16 KV cache as MFMA operand fragments (the layout of internal.h;
// slots past a user's valid length as zeros), so that no key / value rows are written and read back.
// which0 = 1: the weight and N cover the key and value columns only (last layer: no attention).
// l_pad > 0: every user has this padded and l_valid valid rows; l_pad == 0: ragged batch, a block of
// 32 rows finds its user in seg (one entry per 64 rows) and the user's rows in tok_off / hist_len.
struct QkvToCache {         // layer_base == nullptr: plain store
    uint8_t *layer_base;    // cache payload of the layer
    int H, l_valid, l_pad;  // heads of 64; uniform batches: every user's valid and padded length
    int d, which0;
    const int32_t *seg, *tok_off, *hist_len;  // dev: [rows/64], [B+1], [B]
    int64_t rows;
};

// C = A W (+ epilogue).  A: bf16 [M][lda], or tiled (kTiledA; lda unused); w_packed from pack_weight;
// N % 128 == 0, K % 64 == 0.  EPI_STORE_BF16 / EPI_GELU_BF16 / EPI_RELU_BF16: C is bf16 [M][ldc] (EPI_GELU_BF16 with
// kTiledC: tiled, ldc unused).  EPI_RESID_F32: C is fp32, C = acc + resid.
hipError_t gemm_bf16(int epi, const void *A, int64_t lda, const void *w_packed, int M, int N, int K,
                     void *C, int64_t ldc, const float *resid, int64_t ldr, const RowNormIn &in_norm,
                     const RowNormOut &out_norm, int tiled, hipStream_t s, const QkvToCache *to_cache = nullptr);

// What the first projection of a stack call needs of its input rows: the sum of squares of every
// row into ss[row][0] (ss[row][1 .. n_part-1] = 0) and
//   from bf16 rows x (the embeddings): the fp32 copy x32 (the residual stream);
//   from fp32 rows x: the bf16 copy xb.
hipError_t row_prep_bf16(const void *x, float *x32, float *ss, int n_part, int64_t rows, int d, hipStream_t s);
hipError_t row_prep_f32(const float *x, void *xb, float *ss, int n_part, int64_t rows, int d, hipStream_t s);

}  // namespace climber
