// Device-side building blocks shared by the bf16 MFMA attention kernels (attn_bf16.hip,
// hist_fused_bf16.hip): operand fragment types, the per-wave softmax state and the block-level
// steps S^T = K Q^T, softmax (FAST: no reference; SAFE: running maximum) and O^T += V^T P^T of
// Eq. (3) of Climber (arXiv 2502.09888) in the transposed formulation described in attn_bf16.hip.
#pragma once
#include "internal.h"

namespace climber {
namespace attn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef const __attribute__((address_space(1))) uint8_t glb_u8;

constexpr float kSafeSlack = 8.0f;           // SAFE: exp2-domain slack before the row maximum moves
// FAST is accepted iff kDenomLo < denominator < kDenomHi for every row.  The window bounds the
// largest logit of a row (in log2 units it is at most log2 of the denominator), and with it the
// error that rounding q * c to bf16 puts on the dominant probabilities; rows beyond it are redone
// by the SAFE pass, which scales in fp32.
constexpr float kDenomHi = 1048576.f;        // 2^20
constexpr float kDenomLo = 1.f / 1048576.f;  // 2^-20
// The exact-scale form of the FAST pass (queries unrounded, p = exp2(s * c) with c in fp32) has no
// error that grows with the logits; its window only keeps the exponentials inside the fp32 / bf16
// exponent range.
constexpr float kDenomHiExact = 1.0e30f;
constexpr float kDenomLoExact = 1.0e-30f;
// largest root mean square of the first block's exponents s * c (log2 units) for which a wave
// folds c into its bf16 queries (the benchmark's logits have 2.9 at the smallest temperature), and
// the fewest keys a row must see for it: the folded form's error per logit averages out over
// many comparable keys, not over a few
constexpr float kPilotSpread = 4.25f;
constexpr int kFoldMinKeys = 256;
constexpr float kSafeNoRef = -1.0e30f;       // SAFE: "no reference yet", below any finite logit
constexpr int kBiasLdsFloats = 4096;         // LDS floats for one head's rows of the bias tables

// Per-wave softmax state for QB blocks of 32 queries.
template <int QB>
struct QState {
    bf16x8 qf[QB][4];  // B operands of S^T: FAST q' = bf16(q*c), SAFE q; [query][16s + 8hf + 0..7]
    float c[QB];      // qk_scale * log2(e) / tau_row                       (SAFE)
    float m_ref[QB];  // running reference maximum, raw logit units         (SAFE)
    float l[QB];      // this half-wave's share of the softmax denominator
    f32x16 O[2][QB];  // O^T[d block][query block]
};

struct KFrags { bf16x8 a[4]; };  // K A-operands of a 32-key block (4 k-steps of 16 dims)
struct VFrags { bf16x8 a[2][2]; };  // V^T A-operands [16-key group][32-dim block]

// A pointer the caller knows to be wave-uniform, as a value in scalar registers.
static __device__ __forceinline__ const uint8_t *uniform_ptr(const uint8_t *p)
{
    const uint64_t a = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return (const uint8_t *)(((uint64_t)hi << 32) | lo);
}

static __device__ __forceinline__ float xhalf(float x) { return __shfl_xor(x, 32, 64); }

// Exchange between the two half-waves: returns max(x, x of the lane 32 away).
static __device__ __forceinline__ float xhalf_max(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

static __device__ __forceinline__ KFrags load_k(const uint8_t *blk, int lane)
{
    KFrags f;
#pragma unroll
    for (int s = 0; s < 4; ++s) f.a[s] = *(const bf16x8 *)(blk + (s * 64 + lane) * 16);
    return f;
}

static __device__ __forceinline__ VFrags load_v(const uint8_t *blk, int lane)
{
    VFrags f;
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int db = 0; db < 2; ++db)
            f.a[g][db] = *(const bf16x8 *)(blk + 4096 + ((g * 2 + db) * 64 + lane) * 16);
    return f;
}

// S^T[qb] = K_blk q_qb^T for both query blocks
template <int QB>
static __device__ __forceinline__ void qk_block(const QState<QB> &st, const KFrags &k, f32x16 (&S)[QB])
{
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) S[qb][r] = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            S[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k.a[s], st.qf[qb][s], S[qb], 0, 0, 0);
}

// S^T[qb] += K_blk q_qb^T onto whatever S holds (the relative attention bias of the block)
template <int QB>
static __device__ __forceinline__ void qk_block_acc(const QState<QB> &st, const KFrags &k, f32x16 (&S)[QB])
{
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            S[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k.a[s], st.qf[qb][s], S[qb], 0, 0, 0);
}

// O^T[db][qb] += V^T_{g,db} P^T
template <int QB>
static __device__ __forceinline__ void pv_block(QState<QB> &st, const VFrags &v, const bf16x8 (&P)[QB][2])
{
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                st.O[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v.a[g][db], P[qb][g], st.O[db][qb], 0, 0, 0);
}

// keys with index >= k_hi are excluded (last blocks of a range only)
template <int QB>
static __device__ __forceinline__ void mask_block(f32x16 (&S)[QB], int hf, int blk_lo, int k_hi)
{
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int kidx = blk_lo + 8 * (r >> 2) + 4 * hf + (r & 3);
        if (kidx >= k_hi) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) S[qb][r] = -INFINITY;
        }
    }
}

// causal history attention: the lane's query of block qb sees keys with index < lim[qb] only
template <int QB>
static __device__ __forceinline__ void mask_causal(f32x16 (&S)[QB], int hf, int blk_lo, const int (&lim)[QB])
{
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int kidx = blk_lo + 8 * (r >> 2) + 4 * hf + (r & 3);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            if (kidx >= lim[qb]) S[qb][r] = -INFINITY;
    }
}

// p = exp2(S*scale - sub) rounded to bf16 in B-operand order (P[g] holds the keys of 16-key
// group g); returns the row's share of the denominator.
//   AFFINE = false (scale folded into the query, logits of ordinary size): the sum of the values
//     before rounding.  Round-to-nearest is unbiased, so with many comparable terms the denominator
//     and the bf16 numerators agree to well below the bf16 rounding of a single term, and the sum
//     costs one addition per value.
//     Plain v_add_f32 on purpose: the v_dot2 family issues into the matrix pipe and would take MFMA
//     slots there, whereas adds overlap with the MFMAs of the other wave on the SIMD.
//   AFFINE = true (fp32 scale: large logits, causal rows, bias, the history pass that is bound by
//     memory, the running-maximum pass): the sum of the ROUNDED values.  These rows can be sharply
//     peaked; a single dominant probability rounded to bf16 in the numerator and not in the
//     denominator would put its rounding, a relative 2^-9, straight into the output.
template <bool AFFINE>
static __device__ __forceinline__ float exp_pack(const f32x16 &S, float scale, float sub, bf16x8 (&P)[2])
{
    float sum = 0.f;
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(AFFINE ? fmaf(S[8 * g + e], scale, -sub) : S[8 * g + e]);
            const float p1 = __builtin_amdgcn_exp2f(AFFINE ? fmaf(S[8 * g + e + 1], scale, -sub) : S[8 * g + e + 1]);
            P[g][e] = (__bf16)p0;
            P[g][e + 1] = (__bf16)p1;
            if constexpr (AFFINE) {
                // sum += P[e] * 1 + P[e + 1] * 1 on the rounded pair, one instruction (it issues into the
                // matrix pipe, which these forms leave room in).  Through the builtin, not inline assembly:
                // the compiler knows the wait states the instruction needs before its result is read.
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                const bf16x2_t pr = {P[g][e], P[g][e + 1]}, ones = {(__bf16)1.f, (__bf16)1.f};
                sum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum, false);
            } else {
                sum += p0 + p1;
            }
        }
    return sum;
}

// FAST softmax of one block: p = exp2(t)
template <int QB>
static __device__ __forceinline__ void softmax_fast(QState<QB> &st, const f32x16 (&S)[QB], bf16x8 (&P)[QB][2])
{
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) st.l[qb] += exp_pack<false>(S[qb], 1.f, 0.f, P[qb]);
}

// SAFE softmax of one block: running maximum in raw logit units, p = exp2((s - m) * c)
template <int QB>
static __device__ __forceinline__ void softmax_safe(QState<QB> &st, const f32x16 (&S)[QB], bf16x8 (&P)[QB][2])
{
    float mx[QB];
    bool need[QB];
    bool any = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float v = fmaxf(S[qb][0], S[qb][1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) v = fmaxf(fmaxf(v, S[qb][r]), S[qb][r + 1]);
        mx[qb] = xhalf_max(v);  // same in both half-waves
        need[qb] = (mx[qb] - st.m_ref[qb]) * st.c[qb] > kSafeSlack;
        any |= need[qb];
    }
    if (__builtin_amdgcn_ballot_w64(any) != 0) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float alpha =
                need[qb] ? __builtin_amdgcn_exp2f((st.m_ref[qb] - mx[qb]) * st.c[qb]) : 1.f;
            st.m_ref[qb] = need[qb] ? mx[qb] : st.m_ref[qb];
            st.l[qb] *= alpha;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.O[db][qb][r] *= alpha;
        }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
        st.l[qb] += exp_pack<true>(S[qb], st.c[qb], st.m_ref[qb] * st.c[qb], P[qb]);
}


}  // namespace attn
}  // namespace climber
