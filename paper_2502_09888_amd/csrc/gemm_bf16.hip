// bf16 MFMA GEMM for the projections of the layer stack (f_QKV and f_FFN of Eq. (3), Climber,
// arXiv 2502.09888): C[M][N] = A[M][K] * W[K][N] with fp32 accumulation and a fused epilogue
// (plain bf16 store, residual add into the fp32 stream, erf-GELU).
//
// W is first repacked (pack_weight) into B-operand fragments of v_mfma_f32_32x32x16_bf16:
//   chunk (nb, ks, lane), 16 B: W[16ks + 8(lane/32) + 0..7][32nb + lane%32]
// so that a k-tile of a 32-column block is contiguous and is copied HBM -> LDS linearly.
// A is row-major (its tile is copied row by row, 64 B per row and k-tile, with the 16-byte chunks
// of a row XOR-swizzled by (row / 4) % 4 through the choice of the global address each lane loads:
// 16 consecutive rows of one k chunk then cover all 64 banks) or in the tiled layout of gemm.h,
// where one copy is 1 KiB contiguous.
// Both copies are direct global_load_lds (no register staging) into a ring of 3 or 4 k-tiles of 32,
// one or two tiles in flight, one bare s_barrier per k-tile; the copies of a k-tile are dealt out
// between the MFMAs of the tile two ahead of it, not queued in front of them.
// Workgroup = 4 waves as 2 x 2; a wave owns WM x WN blocks of 32 x 32:
//   4 x 2 (macro tile 256 x 128): 128 accumulator registers, two workgroups per CU (the projections
//         here have K = 512 or 2048: short k-loops, and they sit near the HBM/MFMA ridge);
//   2 x 2 (macro tile 128 x 128): for problems too small to fill the chip with larger tiles.
// Workgroups that share A rows are launched onto the same XCD (see the kernel).
#include "gemm.h"
#include "lanes.h"

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <type_traits>
#include <utility>

namespace climber {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef const __attribute__((address_space(1))) uint8_t glb_u8;

constexpr int BK = 32;      // k-tile

__device__ __forceinline__ void pack_chunk(const __bf16 *w, const __bf16 *gain, __bf16 *out, int K, int N,
                                           int64_t chunk)
{
    // one thread per 16-byte chunk (nb, ks, lane)
    const int lane = (int)(chunk & 63);
    const int64_t t = chunk >> 6;
    const int ks = (int)(t % (K / 16)), nb = (int)(t / (K / 16));
    const int n = 32 * nb + (lane & 31), k0 = 16 * ks + 8 * (lane >> 5);
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const __bf16 x = w[(int64_t)(k0 + e) * N + n];
        v[e] = gain ? (__bf16)((float)x * (float)gain[k0 + e]) : x;
    }
    ((bf16x8 *)out)[chunk] = v;
}

__global__ __launch_bounds__(256) void pack_weight_kernel(const __bf16 *w, __bf16 *out, int K, int N)
{
    const int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (chunk < (int64_t)(N / 32) * (K / 16) * 64) pack_chunk(w, nullptr, out, K, N, chunk);
}

// blockIdx.y = job
__global__ __launch_bounds__(256) void pack_weights_kernel(const PackJobs jobs)
{
    const int j = blockIdx.y, K = jobs.K[j], N = jobs.N[j];
    const int64_t n_chunks = (int64_t)(N / 32) * (K / 16) * 64;
    for (int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x; chunk < n_chunks;
         chunk += (int64_t)gridDim.x * 256)
        pack_chunk((const __bf16 *)jobs.w[j], (const __bf16 *)jobs.gain[j], (__bf16 *)jobs.packed[j], K, N, chunk);
}

// exact-erf GELU, erf by the rational/exponential formula 7.1.26 of Abramowitz & Stegun
// (|error| <= 1.5e-7, far below the bf16 rounding of the result).  With a = |x|, z = a/sqrt(2),
// t = 1/(1 + p z) and h = (1 - erf z)/2 = (poly(t)/2) t exp(-z^2):
//   GELU(x) = x (1 + erf(x/sqrt 2))/2 = max(x, 0) - a h        (x >= 0: x - x h;  x < 0: x h)
// which needs no sign select; the constants carry the factors 1/2, 1/sqrt(2) and log2(e)/2.
__device__ __forceinline__ float gelu_erf(float x)
{
    const float a = __builtin_fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(a, 0.3275911f * 0.70710678118654752f, 1.f));
    float poly = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
    poly = fmaf(poly, t, 0.5f * 1.421413741f);
    poly = fmaf(poly, t, 0.5f * -0.284496736f);
    poly = fmaf(poly, t, 0.5f * 0.254829592f);
    const float e = __builtin_amdgcn_exp2f((x * x) * -0.72134752044448170f);
    const float h = (poly * t) * e;
    return fmaf(-a, h, fmaxf(x, 0.f));
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), unrolled at compile time
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F &&f)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

template <int N>
__device__ __forceinline__ void wait_vm()
{
    if (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else if (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if (N == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else if (N == 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    else if (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else static_assert(N == 0 || N == 2 || N == 4 || N == 6 || N == 8 || N == 12 || N == 16, "unsupported vmcnt");
}

// WM, WN: 32 x 32 blocks per wave along M and N.  Macro tile (2*WM*32) x (2*WN*32) x 32.
template <int EPI, int WM, int WN, int kStages>
__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(
    const __bf16 *A, int64_t lda, const __bf16 *Wp, int M, int N, int K, void *C, int64_t ldc,
    const float *resid, int64_t ldr, const RowNormIn nin, const RowNormOut nout, const int tiled,
    const QkvToCache qc)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int kABytes = BM * BK * 2, kBBytes = BN * BK * 2, kStageBytes = kABytes + kBBytes;
    constexpr int NA = kABytes / 1024 / 4, NB = kBBytes / 1024 / 4;  // 1 KiB copies per wave and tile
    constexpr int NPRE = NA + NB;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // the wave number as a scalar: LDS destinations of the copies (M0) are then scalar arithmetic
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hf = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    // Tile of this workgroup.  Workgroups are dealt to the 8 XCDs round-robin in launch order and
    // every XCD has an L2 of its own; the n_col workgroups that share a block of A rows are therefore
    // given launch indices that are equal modulo 8 (one XCD, adjacent in time), so that the rows
    // come from HBM once instead of once per XCD.
    const int n_col = N / BN, n_tiles = n_col * ((M + BM - 1) / BM);
    int tile = blockIdx.x;
    if (n_tiles % 8 == 0) tile = (tile & 7) * (n_tiles >> 3) + (tile >> 3);
    const int m0 = (tile / n_col) * BM, n0 = (tile % n_col) * BN;
    const int n_kt = K / BK;

    // copy plan.  A: copy j of this wave covers rows 16*(wave*NA + j) .. +15, lane -> (row, slot),
    // global chunk = slot ^ ((row >> 2) & 3).  W: copy j covers fragment (nbl, ksl) of the tile.
    const __bf16 *a_src[NA];
    const bool a_tiled = tiled & kTiledA;
    const int a_step = a_tiled ? 512 : BK;   // elements from one k-tile of a copy to the next
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int r = 16 * (wave * NA + j) + (lane >> 2), slot = lane & 3;
        if (a_tiled)   // the 1 KiB piece is stored as it lands in LDS, swizzle included
            a_src[j] = A + (int64_t)min((m0 >> 4) + wave * NA + j, (M - 1) >> 4) * (K / BK) * 512 + lane * 8;
        else
            a_src[j] = A + (int64_t)min(m0 + r, M - 1) * lda + ((slot ^ ((r >> 2) & 3)) * 8);
    }
    const uint8_t *w_src[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int f = wave * NB + j, nbl = f >> 1, ksl = f & 1;
        w_src[j] = (const uint8_t *)Wp +
                   (((int64_t)(n0 / 32 + nbl) * (K / 16) + ksl) * 64 + lane) * 16;
    }
    // copy c (0 .. NPRE-1) of k-tile kt into the ring stage at byte offset `stage`: NA pieces of the
    // A tile, then NB pieces of the W tile
    auto issue_one = [&](int kt, int stage, auto c_tag) __attribute__((always_inline)) {
        constexpr int c = decltype(c_tag)::value;
        lds_u8 *base = (lds_u8 *)lds + stage;
        if constexpr (c < NA)
            __builtin_amdgcn_global_load_lds((glb_u8 *)(a_src[c] + kt * a_step), base + (wave * NA + c) * 1024, 16, 0, 0);
        else
            __builtin_amdgcn_global_load_lds((glb_u8 *)(w_src[c - NA] + (int64_t)kt * 2048),
                                             base + kABytes + (wave * NB + (c - NA)) * 1024, 16, 0, 0);
    };
    auto issue = [&](int kt) __attribute__((always_inline)) {
        static_for<NPRE>([&](auto c) __attribute__((always_inline)) { issue_one(kt, (kt % kStages) * kStageBytes, c); });
    };

    // the first tiles start their way in before anything else is set up (accumulators, row
    // statistics, cache geometry: a microsecond or two that the copies' latency covers)
    for (int kt = 0; kt < kStages - 1 && kt < n_kt; ++kt) issue(kt);

    f32x16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Input rows that were not normalised: r = 1/sqrt(mean(x^2) + eps) of row 32i + l32 scales the
    // whole output row (a lane's accumulators of block row i all belong to that one row).  The
    // partial sums of squares are requested here, ahead of the k-loop, and first touched in the
    // epilogue, so nothing waits for them (8 partial sums per row, d_model = 512, is the fast path).
    constexpr bool SCALED = EPI != EPI_RESID_F32;
    float4 raw_ss[SCALED ? WM : 1][2];
    const bool ss8 = SCALED && nin.ss && nin.n_part == 8;
    if (ss8) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int row = min(m0 + 32 * (WM * wm + i) + l32, M - 1);
            raw_ss[i][0] = *(const float4 *)(nin.ss + (int64_t)row * 8);
            raw_ss[i][1] = *(const float4 *)(nin.ss + (int64_t)row * 8 + 4);
        }
    }

    // Direct cache write: the user that block row i of this wave (32 tokens) belongs to -- first
    // row, padded and valid length -- by arithmetic for uniform batches, from the cache's tables for
    // ragged ones (wave-uniform loads, requested here and first used in the epilogue).
    int u_t0[WM], u_lp[WM], u_lv[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        u_t0[i] = 0, u_lp[i] = 64, u_lv[i] = 0;
        if (EPI == EPI_STORE_BF16 && qc.layer_base) {
            const int rb = __builtin_amdgcn_readfirstlane(min(m0 + 32 * (WM * wm + i), M - 32));
            if (qc.l_pad > 0) {
                u_t0[i] = rb / qc.l_pad * qc.l_pad, u_lp[i] = qc.l_pad, u_lv[i] = qc.l_valid;
            } else {
                const int u = qc.seg[rb >> 6];
                u_t0[i] = qc.tok_off[u];
                u_lp[i] = qc.tok_off[u + 1] - u_t0[i];
                u_lv[i] = qc.hist_len[u];
            }
        }
    }

    // One k-tile: wait for it, read both halves' fragments, then the MFMAs with the copies of tile
    // kt + kStages - 1 (if PREFETCH) dealt out between them, one copy after every kStep-th MFMA, so
    // that a wave never queues its copies back to back in front of its own MFMAs.
    constexpr int kMfma = 2 * WM * WN, kStep = kMfma / NPRE >= 1 ? kMfma / NPRE : 1;
    // The ring stages of tile kt and of the tile to prefetch come in as byte offsets carried by the
    // loop (derived from kt % kStages in here, every fragment address cost vector additions on the
    // path from the barrier to the first MFMA instead of being an immediate).
    auto k_tile = [&](int kt, int st_cur, int st_fill, auto prefetch_tag) __attribute__((always_inline)) {
        constexpr bool PREFETCH = decltype(prefetch_tag)::value;
        const int ahead = min(kt + kStages - 1, n_kt) - (kt + 1);  // tiles that may stay in flight
        if (kStages > 3 && ahead >= 2) wait_vm<(kStages > 3 ? 2 : 1) * NPRE>();
        else if (ahead >= 1) wait_vm<NPRE>();
        else wait_vm<0>();
        __builtin_amdgcn_s_barrier();
        const uint8_t *sa = lds + st_cur;
        const uint8_t *sw = sa + kABytes;
        bf16x8 af[2][WM], bfr[2][WN];
        auto read_frags = [&](auto ks_tag) __attribute__((always_inline)) {
            constexpr int ks = decltype(ks_tag)::value;
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                const int row = 32 * (WM * wm + i) + l32;
                af[ks][i] = *(const bf16x8 *)(sa + row * 64 + (((2 * ks + hf) ^ ((row >> 2) & 3)) * 16));
            }
#pragma unroll
            for (int j = 0; j < WN; ++j)
                bfr[ks][j] = *(const bf16x8 *)(sw + (((WN * wn + j) * 2 + ks) * 64 + lane) * 16);
        };
        // the second half's fragments are requested behind the first MFMA, not ahead of it: the four
        // waves leave the barrier together and queue their reads at the one LDS port
        read_frags(std::integral_constant<int, 0>{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<kMfma>([&](auto m_tag) __attribute__((always_inline)) {
            constexpr int Ms = decltype(m_tag)::value;
            constexpr int ks = Ms / (WM * WN), i = (Ms % (WM * WN)) / WN, j = Ms % WN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks][j], af[ks][i], acc[i][j], 0, 0, 0);
            if constexpr (Ms == 0) {
                read_frags(std::integral_constant<int, 1>{});
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (PREFETCH && Ms % kStep == kStep - 1 && Ms / kStep < NPRE) {
                issue_one(kt + kStages - 1, st_fill, std::integral_constant<int, Ms / kStep>{});
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };
    {
        constexpr int kRing = kStages * kStageBytes;
        int kt = 0, st_cur = 0, st_fill = kRing - kStageBytes;   // stage of tile kt, stage of tile kt - 1
        auto advance = [&]() __attribute__((always_inline)) {
            st_fill = st_cur;
            st_cur = st_cur + kStageBytes == kRing ? 0 : st_cur + kStageBytes;
        };
        for (; kt + kStages - 1 < n_kt; ++kt, advance()) k_tile(kt, st_cur, st_fill, std::true_type{});
        for (; kt < n_kt; ++kt, advance()) k_tile(kt, st_cur, st_fill, std::false_type{});
    }

    // Epilogue.  The operands were fed as (W fragment, A fragment), so a block accumulator is the
    // transposed product: lane holds C[32i + l32][32j + 8g + 4hf + 0..3] for g = r/4 -- four
    // consecutive columns of ONE row.  Each wave turns 32 rows x (WN*32) columns around in its own
    // corner of the (now idle) LDS ring and stores whole rows, 16 bytes per lane.
    __syncthreads();  // every wave is done reading the last k-tile
    constexpr bool F32 = EPI == EPI_RESID_F32;
    float rs[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) rs[i] = 1.f;
    if (SCALED && nin.ss) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            float ss = 0.f;
            if (ss8) {
                const float4 u = raw_ss[i][0], v = raw_ss[i][1];
                ss = ((u.x + u.y) + (u.z + u.w)) + ((v.x + v.y) + (v.z + v.w));
            } else {
                const int row = min(m0 + 32 * (WM * wm + i) + l32, M - 1);
                for (int q = 0; q < nin.n_part; ++q) ss += nin.ss[(int64_t)row * nin.n_part + q];
            }
            rs[i] = 1.f / sqrtf(ss * nin.inv_d + nin.eps);
        }
    }

    constexpr int CW = WN * 32;                       // columns of a wave's block
    constexpr int kElem = F32 ? 4 : 2;
    constexpr int kPitch = CW * kElem + 16;           // bytes per staged row
    constexpr int kChunksPerRow = CW * kElem / 16;
    uint8_t *tr = lds + wave * (32 * kPitch);
    constexpr int kIters = 32 * kChunksPerRow / 64;   // 16-byte pieces per lane and block row
    const int col_base = n0 + CW * wn;
    // Residual rows of block row i, all requested before anything waits for them (a load placed
    // after a store would make the wait for it drain the stores as well: one memory round trip per
    // 16 bytes).  Block row i + 1 is requested before block row i is stored.
    float4 rsd[2][F32 ? kIters : 1];
    auto load_resid = [&](int i, float4 *buf) __attribute__((always_inline)) {
        if constexpr (F32) {
#pragma unroll
            for (int it = 0; it < kIters; ++it) {
                const int id = it * 64 + lane, r = id / kChunksPerRow, cc = id % kChunksPerRow;
                const int row = min(m0 + 32 * (WM * wm + i) + r, M - 1);
                buf[it] = *(const float4 *)(resid + (int64_t)row * ldr + col_base + cc * 4);
            }
        }
    };
    load_resid(0, rsd[0]);
    // direct cache write: slots past a user's valid length hold zeros
    bool zero_row[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i)
        zero_row[i] = EPI == EPI_STORE_BF16 && qc.layer_base &&
                      m0 + 32 * (WM * wm + i) - u_t0[i] + l32 >= u_lv[i];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = 32 * j + 8 * g + 4 * hf;
                if (F32) {
                    float4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                    *(float4 *)(tr + l32 * kPitch + col * 4) = v;
                } else {
                    __attribute__((aligned(8))) __bf16 v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float x = acc[i][j][4 * g + e] * rs[i];
                        v[e] = (__bf16)(EPI == EPI_GELU_BF16 ? gelu_erf(x) : EPI == EPI_RELU_BF16 ? fmaxf(x, 0.f) : x);
                    }
                    if (EPI == EPI_STORE_BF16 && zero_row[i]) v[0] = v[1] = v[2] = v[3] = (__bf16)0.f;
                    *(uint2 *)(tr + l32 * kPitch + col * 2) = *(const uint2 *)v;
                }
            }
        if (i + 1 < WM) load_resid(i + 1, rsd[(i + 1) & 1]);
        const int row_base = m0 + 32 * (WM * wm + i);
        if (EPI == EPI_STORE_BF16 && qc.layer_base) {
            // the wave's 32 x 64 block is one head of the queries, keys or values of 32 tokens of one
            // user (padded lengths are multiples of 64)
            static_assert(EPI != EPI_STORE_BF16 || CW == 64, "a wave's block = one head");
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            const int which = qc.which0 + col_base / qc.d, h = (col_base % qc.d) / 64;
            if (row_base < M) {
                const int kb = (row_base - u_t0[i]) / 32;
                uint8_t *blk = qc.layer_base + ((size_t)u_t0[i] * qc.H + (size_t)h * u_lp[i]) * 256 + (size_t)kb * 8192;
                if (which == 0) {        // query rows
#pragma unroll
                    for (int it = 0; it < kIters; ++it) {
                        const int id = it * 64 + lane, r = id / kChunksPerRow, cc = id % kChunksPerRow;
                        if (row_base + r < M)
                            *(uint4 *)((__bf16 *)C + (int64_t)(row_base + r) * ldc + h * 64 + cc * 8) =
                                *(const uint4 *)(tr + r * kPitch + cc * 16);
                    }
                } else if (which == 1) {  // K fragments: chunk (s, lane) = K[lane % 32][16 s + 8 (lane / 32) ..]
#pragma unroll
                    for (int s4 = 0; s4 < 4; ++s4)
                        *(uint4 *)(blk + (s4 * 64 + lane) * 16) = *(const uint4 *)(tr + l32 * kPitch + (2 * s4 + hf) * 16);
                } else {                  // V^T chunks by LDS transpose reads (see hist_fused_bf16.hip)
                    const int G = lane >> 4, i16 = lane & 15;
#pragma unroll
                    for (int gg = 0; gg < 2; ++gg)
#pragma unroll
                        for (int db = 0; db < 2; ++db) {
                            s16x4 hv[2];
#pragma unroll
                            for (int hh = 0; hh < 2; ++hh) {
                                const int r = 16 * gg + 8 * hh + 4 * (G >> 1) + (i16 >> 2);
                                const int cb = 64 * db + 32 * (G & 1) + 8 * (i16 & 3);
                                hv[hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                    (__attribute__((address_space(3))) s16x4 *)(tr + r * kPitch + cb));
                            }
                            const s16x8 both = __builtin_shufflevector(hv[0], hv[1], 0, 1, 2, 3, 4, 5, 6, 7);
                            *(uint4 *)(blk + 4096 + ((gg * 2 + db) * 64 + lane) * 16) = __builtin_bit_cast(uint4, both);
                        }
                }
            }
            continue;
        }
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int id = it * 64 + lane, r = id / kChunksPerRow, cc = id % kChunksPerRow;
            const int row = row_base + r;
            uint4 val = *(const uint4 *)(tr + r * kPitch + cc * 16);
            if (F32) {
                const int col = col_base + cc * 4;
                const float4 rd = rsd[i & 1][it];
                float4 o = *(const float4 *)&val;
                o.x += rd.x; o.y += rd.y; o.z += rd.z; o.w += rd.w;
                if (row < M) {
                    *(float4 *)((float *)C + (int64_t)row * ldc + col) = o;
                    if (nout.ss) {
                        bf16x4 ob;
                        ob[0] = (__bf16)o.x; ob[1] = (__bf16)o.y; ob[2] = (__bf16)o.z; ob[3] = (__bf16)o.w;
                        *(bf16x4 *)((__bf16 *)nout.xb + (int64_t)row * nout.ldb + col) = ob;
                    }
                }
                if (nout.ss) {  // sums of squares of 64-column slices of the row: 16 lanes each
                    static_assert(!F32 || kChunksPerRow % 16 == 0, "a 64-column slice = 16 lanes of one row");
                    const float sq = row_sum16(o.x * o.x + o.y * o.y + o.z * o.z + o.w * o.w);
                    if ((cc & 15) == 0 && row < M)
                        nout.ss[(int64_t)row * (N / 64) + (col_base + cc * 4) / 64] = sq;
                }
            } else if (EPI == EPI_GELU_BF16 && (tiled & kTiledC)) {
                // piece `it` = (16-row group it / 2, k-tile it % 2) of the block; a lane takes the chunk
                // that the consuming projection's copy puts at its place in LDS
                static_assert(EPI != EPI_GELU_BF16 || (CW == 64 && kIters == 4), "block = 2 x 2 pieces");
                const int rr = 16 * (it >> 1) + (lane >> 2), c = (lane & 3) ^ ((lane >> 4) & 3);
                val = *(const uint4 *)(tr + rr * kPitch + ((it & 1) * 4 + c) * 16);
                if (row_base + rr < M)
                    *(uint4 *)((uint8_t *)C + ((int64_t)((row_base >> 4) + (it >> 1)) * (N / 32) +
                                               (col_base >> 5) + (it & 1)) * 1024 + lane * 16) = val;
            } else if (row < M) {
                *(uint4 *)((__bf16 *)C + (int64_t)row * ldc + col_base + cc * 8) = val;
            }
        }
    }
}

template <int EPI, int WM, int WN, int kStages>
hipError_t launch(const __bf16 *a, int64_t lda, const __bf16 *w, int M, int N, int K, void *C,
                  int64_t ldc, const float *resid, int64_t ldr, const RowNormIn &nin, const RowNormOut &nout,
                  int tiled, const QkvToCache &qc, hipStream_t s)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr size_t lds_bytes = (size_t)kStages * (BM + BN) * BK * 2;
    // the kernel's dynamic LDS exceeds the default limit: raised once per device (the attribute belongs
    // to the function as loaded on the current device)
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> raised[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!raised[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute((const void *)gemm_bf16_kernel<EPI, WM, WN, kStages>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised[dev].store(true, std::memory_order_release);
    }
    const dim3 grid((N / BN) * ((M + BM - 1) / BM)), block(256);
    hipLaunchKernelGGL((gemm_bf16_kernel<EPI, WM, WN, kStages>), grid, block, lds_bytes, s, a, lda, w, M, N, K,
                       C, ldc, resid, ldr, nin, nout, tiled, qc);
    return hipGetLastError();
}

template <int EPI>
hipError_t dispatch(const __bf16 *a, int64_t lda, const __bf16 *w, int M, int N, int K, void *C,
                    int64_t ldc, const float *resid, int64_t ldr, const RowNormIn &nin,
                    const RowNormOut &nout, int tiled, const QkvToCache &qc, hipStream_t s)
{
    // macro tile 256 x 128 when that still gives every CU two workgroups, else 128 x 128
    const int64_t big_tiles = (int64_t)(N / 128) * ((M + 255) / 256);
    if (big_tiles >= 512) return launch<EPI, 4, 2, 3>(a, lda, w, M, N, K, C, ldc, resid, ldr, nin, nout, tiled, qc, s);
    return launch<EPI, 2, 2, 4>(a, lda, w, M, N, K, C, ldc, resid, ldr, nin, nout, tiled, qc, s);
}

}  // namespace

hipError_t pack_weight(const void *w, void *packed, int K, int N, hipStream_t s)
{
    const int64_t n_chunks = (int64_t)(N / 32) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, s,
                       (const __bf16 *)w, (__bf16 *)packed, K, N);
    return hipGetLastError();
}

hipError_t pack_weights(const PackJobs &jobs, hipStream_t s)
{
    if (jobs.n <= 0) return hipSuccess;
    if (jobs.n > kMaxPackJobs) return hipErrorInvalidValue;
    int64_t most = 0;
    for (int j = 0; j < jobs.n; ++j)
        most = std::max<int64_t>(most, (int64_t)(jobs.N[j] / 32) * (jobs.K[j] / 16) * 64);
    const unsigned gx = (unsigned)std::min<int64_t>((most + 255) / 256, 1024);
    hipLaunchKernelGGL(pack_weights_kernel, dim3(gx, (unsigned)jobs.n), dim3(256), 0, s, jobs);
    return hipGetLastError();
}

hipError_t gemm_bf16(int epi, const void *A, int64_t lda, const void *w_packed, int M, int N, int K,
                     void *C, int64_t ldc, const float *resid, int64_t ldr, const RowNormIn &nin,
                     const RowNormOut &nout, int tiled, hipStream_t s, const QkvToCache *to_cache)
{
    if (M <= 0) return hipSuccess;
    QkvToCache qc{};
    if (to_cache) {
        qc = *to_cache;
        if (epi != EPI_STORE_BF16 || !qc.layer_base || qc.d % 64 != 0 || qc.H * 64 != qc.d || qc.l_pad % 64 != 0 ||
            qc.l_pad < 0 || qc.l_valid < 0 || qc.l_valid > qc.l_pad || N != (3 - qc.which0) * qc.d ||
            M != qc.rows || M % 64 != 0 || (qc.l_pad > 0 && M % qc.l_pad != 0) ||
            (qc.l_pad == 0 && (!qc.seg || !qc.tok_off || !qc.hist_len)))
            return hipErrorInvalidValue;
    }
    if (N % 128 != 0 || K % 64 != 0) return hipErrorInvalidValue;
    if ((tiled & ~(kTiledA | kTiledC)) || ((tiled & kTiledC) && epi != EPI_GELU_BF16)) return hipErrorInvalidValue;
    const __bf16 *a = (const __bf16 *)A, *w = (const __bf16 *)w_packed;
    switch (epi) {
    case EPI_STORE_BF16: return dispatch<EPI_STORE_BF16>(a, lda, w, M, N, K, C, ldc, resid, ldr, nin, nout, tiled, qc, s);
    case EPI_GELU_BF16: return dispatch<EPI_GELU_BF16>(a, lda, w, M, N, K, C, ldc, resid, ldr, nin, nout, tiled, qc, s);
    case EPI_RESID_F32: return dispatch<EPI_RESID_F32>(a, lda, w, M, N, K, C, ldc, resid, ldr, nin, nout, tiled, qc, s);
    case EPI_RELU_BF16: return dispatch<EPI_RELU_BF16>(a, lda, w, M, N, K, C, ldc, resid, ldr, nin, nout, tiled, qc, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace climber
