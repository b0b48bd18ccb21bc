// Fused history pass for gfx950 (CDNA4), bf16: for subsequences of 128 or 256 behaviours the
// per-layer K/V cache write (Climber, arXiv 2502.09888, Sec. 3.2: history K/V are produced once
// and kept for the candidates) and the attention inside each subsequence (Sec. 3.1.2 + Eq. (3),
// one Transformer block per subsequence, per-row temperature) run in ONE kernel.
//
// One workgroup (4 waves) owns one (user, head, subsequence).  The subsequence's key and value
// rows are read from HBM exactly once:
//   - K rows go HBM -> LDS directly into the MFMA operand fragments the cache stores (the
//     fragment layout is a permutation of 16-byte row pieces, so the copy only needs the right
//     global address per lane),
//   - V rows go HBM -> LDS row-major (XOR-swizzled 16-byte chunks) and are turned into the
//     transposed, key-permuted V^T fragments with 2-byte LDS gathers, half a subsequence at a time
//     so that raw rows and fragments share buffers,
//   - the finished fragments (a contiguous image of the subsequence's cache blocks) are written to
//     the cache AND consumed in place by the attention of the subsequence's own queries: no ring,
//     no barrier inside the attention loop, and the cache is never read back.
// Slots past a user's valid length hold zeros in the cache and are masked in the softmax whatever
// the source rows contain; padded query rows produce zeros.
// The softmax is the FAST / SAFE scheme of attn_bf16.hip (no reference subtraction unless a
// denominator leaves [1e-12, 1e12]); here the SAFE redo is per wave, since waves share only
// read-only data.
#include "attn_common.h"

#include <type_traits>

namespace climber {
namespace {

using namespace attn;

struct HParams {
    uint8_t *layer_base;
    const int32_t *hist_len, *tok_off;
    const __bf16 *q, *k, *v;
    const int32_t *scen, *beh;
    const float *tau;
    __bf16 *o;
    int64_t ld, ld_o;
    int B, H, n_scen, n_beh, n_sub;
    int uni_len, uni_pad;  // >= 0: every user has this valid / padded history length
    float scale_log2e;
};

template <int SUB>
__global__ __launch_bounds__(256, 2) void hist_fused_kernel(const HParams p)
{
    static_assert(SUB == 128 || SUB == 256, "fragments of the whole subsequence stay in LDS");
    constexpr int NB = SUB / 32;    // 32-key blocks per subsequence
    constexpr int QB = SUB / 128;   // 32-query blocks per wave
    constexpr int WQ = 32 * QB;     // query rows per wave
    constexpr int HALF = SUB / 2;   // V rows are transposed in two halves
    constexpr int kKf = 0;                       // K fragments, NB x 4 KiB
    constexpr int kVf = NB * 4096;               // V^T fragments, NB x 4 KiB (halves A, B)
    constexpr int kRawB = kVf + NB * 2048;       // raw V rows of half 0 (later V^T half 1)
    constexpr int kRawC = kVf + NB * 4096;       // raw V rows of half 1 (later output staging)
    constexpr int kOut = SUB == 256 ? kRawC : kRawC + NB * 2048;
    constexpr int kLds = kOut + 16384;
    static_assert(SUB != 256 || kLds == 81920, "two workgroups per CU");
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLds];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const int si = blockIdx.x % p.n_sub, bh = blockIdx.x / p.n_sub;
    const int h = bh % p.H, b = bh / p.H;
    int Lb, t0, Lpad;
    if (p.uni_len >= 0) {
        Lb = p.uni_len;
        Lpad = p.uni_pad;
        t0 = b * Lpad;
    } else {
        Lb = p.hist_len[b];
        t0 = p.tok_off[b];
        Lpad = p.tok_off[b + 1] - t0;
    }
    const int k_lo = si * SUB;
    if (k_lo >= Lpad) return;
    const int n_pad = min(SUB, Lpad - k_lo);           // rows that exist (multiple of 64)
    const int n_valid = max(0, min(n_pad, Lb - k_lo));  // valid keys = valid queries
    const int64_t row0 = (int64_t)t0 + k_lo;

    // ---- 1. everything this workgroup needs from HBM is requested up front -------------------
    QState<QB> st;
    int64_t qrow[QB];
    int sc_id[QB], bh_id[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        qrow[qb] = row0 + min(wave * WQ + qb * 32 + l32, max(n_valid, 1) - 1);
        const __bf16 *qp = p.q + qrow[qb] * p.ld + h * kDHead + 8 * hf;
#pragma unroll
        for (int s = 0; s < 4; ++s) st.qf[qb][s] = *(const bf16x8 *)(qp + 16 * s);
        sc_id[qb] = p.scen[qrow[qb]];
        bh_id[qb] = p.beh[qrow[qb]];
    }
    // K: chunk ck = 4 kb + s of 1 KiB = lanes' pieces K[32kb + lane%32][16s + 8(lane/32) + 0..7]
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int ck = i * 4 + wave, kb = ck >> 2, s = ck & 3;
        const int64_t row = row0 + min(32 * kb + l32, n_pad - 1);
        __builtin_amdgcn_global_load_lds((glb_u8 *)(p.k + row * p.ld + h * kDHead + 16 * s + 8 * hf),
                                         (lds_u8 *)lds + kKf + ck * 1024, 16, 0, 0);
    }
    // V: raw rows, 128 B each, 8 lanes per row, chunk c of row r stored at slot c ^ (r & 7)
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int i = 0; i < SUB / 64; ++i) {
            const int gi = wave * (SUB / 64) + i, pos = gi * 64 + lane, r = pos >> 3;
            const int c = (pos & 7) ^ (r & 7);
            const int64_t row = row0 + min(half * HALF + r, n_pad - 1);
            __builtin_amdgcn_global_load_lds((glb_u8 *)(p.v + row * p.ld + h * kDHead + c * 8),
                                             (lds_u8 *)lds + (half ? kRawC : kRawB) + gi * 1024, 16, 0, 0);
        }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // temperature of the rows (the ids have arrived): the lookups overlap with the transposes
    float c_row[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int sc = min(max(sc_id[qb], 0), p.n_scen - 1);
        const int bhv = min(max(bh_id[qb], 0), p.n_beh - 1);
        c_row[qb] = p.tau[sc * p.n_beh + bhv];
    }
    // keys past the valid length: zeros in the fragments (each lane clears the pieces it copied)
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int ck = i * 4 + wave, kb = ck >> 2;
        if (32 * kb + l32 >= n_valid) *(uint4 *)(lds + kKf + ck * 1024 + lane * 16) = uint4{0, 0, 0, 0};
    }
    __syncthreads();

    // ---- 2. V^T fragments: chunk (g, db, lane), element e =
    //         V[32kb + 16g + 8(e/4) + 4(lane/32) + e%4][32db + lane%32] ------------------------
    auto transpose_half = [&](int half, int raw_off, int frag_off) __attribute__((always_inline)) {
        const int g = tid >> 7, db = (tid >> 6) & 1, d = 32 * db + l32;
#pragma unroll
        for (int kbh = 0; kbh < NB / 2; ++kbh) {
            __attribute__((aligned(16))) __bf16 out[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int r = 32 * kbh + 16 * g + 8 * (e >> 2) + 4 * hf + (e & 3);
                const __bf16 x =
                    *(const __bf16 *)(lds + raw_off + r * 128 + (((d >> 3) ^ (r & 7)) * 16) + (d & 7) * 2);
                out[e] = half * HALF + r < n_valid ? x : (__bf16)0.f;
            }
            *(uint4 *)(lds + frag_off + kbh * 4096 + tid * 16) = *(const uint4 *)out;
        }
    };
    transpose_half(0, kRawB, kVf);
    __syncthreads();  // half 0 is in place; its raw rows are no longer needed
    transpose_half(1, kRawC, kRawB);
    __syncthreads();  // all fragments are in place

    // ---- 3. the cache blocks of this subsequence ---------------------------------------------
    {
        uint8_t *dst = p.layer_base + ((size_t)t0 * p.H + (size_t)h * Lpad) * (kDHead * 4) +
                       (size_t)(k_lo / kBlockKeys) * kBlockBytes;
        const int nb_pad = n_pad / kBlockKeys;
#pragma unroll
        for (int kb = 0; kb < NB; ++kb)
            if (kb < nb_pad) {
                const uint4 kk = *(const uint4 *)(lds + kKf + kb * 4096 + tid * 16);
                const uint4 vv = *(const uint4 *)(lds + kVf + kb * 4096 + tid * 16);
                *(uint4 *)(dst + (size_t)kb * kBlockBytes + tid * 16) = kk;
                *(uint4 *)(dst + (size_t)kb * kBlockBytes + 4096 + tid * 16) = vv;
            }
    }

    // ---- 4. attention of the subsequence's own queries (waves are independent from here) ------
    const int n_blk = (n_valid + kBlockKeys - 1) / kBlockKeys;
    auto run = [&](auto safe_tag) __attribute__((always_inline)) {
        constexpr bool SAFE = decltype(safe_tag)::value;
        f32x16 S0[QB], S1[QB];
        bf16x8 P[QB][2];
        if (n_blk > 0) qk_block(st, load_k(lds + kKf, lane), S0);
        auto block = [&](int blk, f32x16 (&Sc)[QB], f32x16 (&Sn)[QB]) __attribute__((always_inline)) {
            if (blk + 1 < n_blk) qk_block(st, load_k(lds + kKf + (blk + 1) * 4096, lane), Sn);
            if (32 * (blk + 1) > n_valid) mask_block(Sc, hf, 32 * blk, n_valid);
            if (SAFE) softmax_safe(st, Sc, P); else softmax_fast(st, Sc, P);
            pv_block(st, load_v(lds + kKf + blk * 4096 + (kVf - 4096), lane), P);
        };
        for (int blk = 0; blk < n_blk; blk += 2) {
            block(blk, S0, S1);
            if (blk + 1 < n_blk) block(blk + 1, S1, S0);
        }
    };
    auto clear_state = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            st.l[qb] = 0.f;
            st.m_ref[qb] = 0.f;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.O[db][qb][r] = 0.f;
        }
    };
    // FAST: q' = bf16(q * c)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        st.c[qb] = p.scale_log2e / c_row[qb];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const bf16x8 qq = st.qf[qb][s];
#pragma unroll
            for (int e = 0; e < 8; ++e) st.qf[qb][s][e] = (__bf16)((float)qq[e] * st.c[qb]);
        }
    }
    clear_state();
    run(std::false_type{});
    float lt[QB];
    bool bad = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        lt[qb] = st.l[qb] + xhalf(st.l[qb]);
        bad |= n_valid > 0 && !(lt[qb] > kDenomLo && lt[qb] < kDenomHi);
    }
    if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // SAFE (rare): unscaled q, running maximum
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const __bf16 *qp = p.q + qrow[qb] * p.ld + h * kDHead + 8 * hf;
#pragma unroll
            for (int s = 0; s < 4; ++s) st.qf[qb][s] = *(const bf16x8 *)(qp + 16 * s);
        }
        clear_state();
        run(std::true_type{});
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) lt[qb] = st.l[qb] + xhalf(st.l[qb]);
    }

    // ---- 5. normalise, turn each 32 x 64 block around in the wave's own 4 KiB of staging, store
    //         whole 128-byte rows; padded query rows that exist get zeros --------------------
    uint8_t *tr = lds + kOut + wave * 4096;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float inv = 1.f / lt[qb];
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 ov;
#pragma unroll
                for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(st.O[db][qb][4 * g + e] * inv);
                *(bf16x4 *)(tr + l32 * 128 + (((4 * db + g) ^ (l32 & 7)) * 16) + 8 * hf) = ov;
            }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = i * 64 + lane, r = id >> 3, cc = id & 7;
            const int wq = wave * WQ + qb * 32 + r;
            const uint4 val = *(const uint4 *)(tr + r * 128 + ((cc ^ (r & 7)) * 16));
            __bf16 *op = p.o + (row0 + wq) * p.ld_o + h * kDHead + cc * 8;
            if (wq < n_valid) {
                __builtin_nontemporal_store(__builtin_bit_cast(u32x4, val), (u32x4 *)op);
            } else if (wq < n_pad) {
                *(uint4 *)op = uint4{0, 0, 0, 0};
            }
        }
    }
}

}  // namespace

bool hist_fused_supported(int sub_len, int causal) { return !causal && (sub_len == 128 || sub_len == 256); }

hipError_t launch_hist_fused_bf16(const AttnArgs &a, hipStream_t s)
{
    HParams p;
    p.layer_base = a.cache.layer_base;
    p.hist_len = a.cache.hist_len;
    p.tok_off = a.cache.tok_off;
    p.q = (const __bf16 *)a.q;
    p.k = (const __bf16 *)a.k_self;
    p.v = (const __bf16 *)a.v_self;
    p.scen = a.scen;
    p.beh = a.beh;
    p.tau = a.tau;
    p.o = (__bf16 *)a.o;
    p.ld = a.ld_q;
    p.ld_o = a.ld_o;
    p.B = a.cache.B;
    p.H = a.H;
    p.n_scen = a.n_scen;
    p.n_beh = a.n_beh;
    p.n_sub = (a.max_rows_per_user + a.sub_len - 1) / a.sub_len;
    p.uni_len = a.uni_len;
    p.uni_pad = a.uni_pad;
    p.scale_log2e = a.qk_scale * 1.4426950408889634f;
    const int64_t grid = (int64_t)p.n_sub * p.B * p.H;
    if (grid <= 0) return hipSuccess;
    if (grid > 0x7fffffff || a.ld_q != a.ld_kv) return hipErrorInvalidValue;
    if (a.sub_len == 256)
        hipLaunchKernelGGL(hist_fused_kernel<256>, dim3((unsigned)grid), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL(hist_fused_kernel<128>, dim3((unsigned)grid), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace climber
