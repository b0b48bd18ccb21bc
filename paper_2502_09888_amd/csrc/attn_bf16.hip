// bf16 MFMA flash attention for gfx950 (CDNA4): the SUMI candidate pass and the block-diagonal
// history pass of Climber (arXiv 2502.09888): Eq. (3) attention with a per-query-row temperature,
// the "single user, multiple items" mask of Sec. 3.2 and the per-subsequence attention of
// Sec. 3.1.2.
//
// Shape of the computation (one workgroup = one (user, head, tile of NW*64 query rows)):
//   - the transposed problem is computed: S^T = K Q^T and O^T = V^T P^T with
//     v_mfma_f32_32x32x16_bf16.  In the accumulator layout of that instruction a lane owns ONE
//     query column (lane % 32), so the softmax statistics of a query are per-lane scalars, the
//     row max / row sum are in-register reductions plus one exchange between the two half-waves,
//     and the probabilities leave the S^T accumulator already in the B-operand layout the P V
//     product needs (the cache stores V with the matching key permutation).
//   - history K/V tiles of 64 keys are copied HBM -> LDS linearly (the cache is stored as MFMA
//     fragments) into a double buffer and are reused by every wave, i.e. by the whole query tile.
//   - online softmax in the exp2 domain: p = exp2(s*c - m*c) with c = qk_scale*log2(e)/tau_row,
//     one FMA + one v_exp_f32 per logit; the reference maximum m is only moved (and O, l
//     rescaled) when a row maximum exceeds it by more than 2^8 in the exp2 domain, so the rescale
//     is rare; results are exact because O and l always share the same reference.
//   - SUMI: the candidate's own key/value initialise the running state (m = own logit, l = 1,
//     O = own value), which is the "+ itself" term of the mask.
#include "internal.h"

namespace climber {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kTileKeys = 64;                  // keys per LDS tile = 2 cache blocks
constexpr int kTileBytes = 2 * kBlockBytes;    // 16 KiB
constexpr float kRescaleThreshold = 8.0f;      // exp2-domain slack before the reference max moves

struct KParams {
    const uint8_t *layer_base;
    const int32_t *hist_len, *tok_off, *order, *cand_off;
    const __bf16 *q, *k_self, *v_self;
    const int32_t *scen, *beh;
    const float *tau;
    __bf16 *o;
    int64_t ld_q, ld_kv, ld_o;
    int B, H, n_scen, n_beh, sub_len, n_qtiles;
    float scale_log2e;
};

__device__ __forceinline__ float xhalf(float x) { return __shfl_xor(x, 32, 64); }

template <int NW, bool SUMI>
__global__ __launch_bounds__(NW * 64) void attn_bf16_kernel(const KParams p)
{
    constexpr int NT = NW * 64;
    constexpr int TQ = NW * 64;            // query rows per workgroup
    constexpr int NPRE = kTileBytes / 16 / NT;
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * kTileBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;

    // workgroup -> (user, head, query tile).  Consecutive workgroup ids are dealt round-robin to
    // the 8 XCDs; tiles of the same (user, head) get ids congruent mod 8 so that they run on one
    // XCD and share its L2 copy of that head's K/V.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, j = wg >> 3;
    const int qt = j % p.n_qtiles;
    const int bh = (j / p.n_qtiles) * 8 + xcd;
    if (bh >= p.B * p.H) return;
    const int b = p.order[bh / p.H], h = bh % p.H;
    const int Lb = p.hist_len[b], t0 = p.tok_off[b], Lpad = p.tok_off[b + 1] - t0;

    const int q0 = qt * TQ;
    int64_t row0;
    int nq, k_lo, k_hi;
    if (SUMI) {
        const int c0 = p.cand_off[b], Mb = p.cand_off[b + 1] - c0;
        if (q0 >= Mb) return;
        row0 = (int64_t)c0 + q0;
        nq = min(TQ, Mb - q0);
        k_lo = 0;
        k_hi = Lb;
    } else {
        if (q0 >= Lpad) return;
        row0 = (int64_t)t0 + q0;
        nq = max(0, min(TQ, Lb - q0));
        if (nq == 0) {  // a tile of padding rows only: defined output, zeros
            for (int idx = tid; idx < TQ * (kDHead / 8); idx += NT) {
                const int r = idx / (kDHead / 8), cc = idx % (kDHead / 8);
                if (q0 + r < Lpad)
                    *(uint4 *)(p.o + (row0 + r) * p.ld_o + h * kDHead + cc * 8) = uint4{0, 0, 0, 0};
            }
            return;
        }
        k_lo = p.sub_len > 0 ? (q0 / p.sub_len) * p.sub_len : 0;
        k_hi = p.sub_len > 0 ? min(k_lo + p.sub_len, Lb) : Lb;
    }
    const int n_tiles = (k_hi - k_lo + kTileKeys - 1) / kTileKeys;
    const uint8_t *kv = p.layer_base + ((size_t)t0 * p.H + (size_t)h * Lpad) * (kDHead * 4) +
                        (size_t)(k_lo / kBlockKeys) * kBlockBytes;

    // ---- per-lane query state: two 32-query blocks per wave ---------------------------------
    bf16x8 qf[2][4];     // B operands of S^T: Q[query][16s + 8hf + 0..7]
    float c[2];          // qk_scale * log2(e) / tau_row
    float m_ref[2];      // reference maximum (raw logit units)
    float l[2];          // this half-wave's share of the softmax denominator
    f32x16 O[2][2];      // O^T[d block][query block]
    int64_t qrow[2];
    bool qvalid[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int wq = wave * 64 + qb * 32 + l32;
        qvalid[qb] = wq < nq;
        qrow[qb] = row0 + min(wq, nq - 1);
        const __bf16 *qp = p.q + qrow[qb] * p.ld_q + h * kDHead + 8 * hf;
#pragma unroll
        for (int s = 0; s < 4; ++s) qf[qb][s] = *(const bf16x8 *)(qp + 16 * s);
        const int sc = min(max(p.scen[qrow[qb]], 0), p.n_scen - 1);
        const int bhv = min(max(p.beh[qrow[qb]], 0), p.n_beh - 1);
        c[qb] = p.scale_log2e / p.tau[sc * p.n_beh + bhv];
        if (SUMI) {
            const __bf16 *kp = p.k_self + qrow[qb] * p.ld_kv + h * kDHead + 8 * hf;
            float dot = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 kk = *(const bf16x8 *)(kp + 16 * s);
#pragma unroll
                for (int e = 0; e < 8; ++e) dot += (float)qf[qb][s][e] * (float)kk[e];
            }
            m_ref[qb] = dot + xhalf(dot);
            l[qb] = hf == 0 ? 1.f : 0.f;
            const __bf16 *vp = p.v_self + qrow[qb] * p.ld_kv + h * kDHead + 4 * hf;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const bf16x4 vv = *(const bf16x4 *)(vp + 32 * db + 8 * g);
#pragma unroll
                    for (int e = 0; e < 4; ++e) O[db][qb][4 * g + e] = (float)vv[e];
                }
        } else {
            m_ref[qb] = -INFINITY;
            l[qb] = 0.f;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[db][qb][r] = 0.f;
        }
    }

    // ---- K/V tile pipeline: HBM -> registers -> LDS double buffer ---------------------------
    uint4 pre[NPRE];
    if (n_tiles > 0) {
#pragma unroll
        for (int i = 0; i < NPRE; ++i) pre[i] = ((const uint4 *)kv)[tid + i * NT];
#pragma unroll
        for (int i = 0; i < NPRE; ++i) ((uint4 *)lds)[tid + i * NT] = pre[i];
    }
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
        const uint8_t *cur = lds + (t & 1) * kTileBytes;
        const bool more = t + 1 < n_tiles;
        if (more) {
            const uint4 *src = (const uint4 *)(kv + (size_t)(t + 1) * kTileBytes);
#pragma unroll
            for (int i = 0; i < NPRE; ++i) pre[i] = src[tid + i * NT];
        }

        // S^T[kb][qb] = K_kb Q_qb^T
        f32x16 S[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[kb][qb][r] = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 a = *(const bf16x8 *)(cur + kb * kBlockBytes + (s * 64 + lane) * 16);
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
                    S[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][s], S[kb][qb], 0, 0, 0);
            }
        }

        // keys past the end of the visible range (only possible in the last tile)
        const int tile_lo = k_lo + t * kTileKeys;
        if (tile_lo + kTileKeys > k_hi) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kidx = tile_lo + kb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (kidx >= k_hi) {
                        S[kb][0][r] = -INFINITY;
                        S[kb][1][r] = -INFINITY;
                    }
                }
        }

        // row maxima and (rarely) a move of the reference maximum
        float mx[2];
        bool need[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float v = S[0][qb][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) v = fmaxf(v, S[kb][qb][r]);
            v = fmaxf(v, xhalf(v));
            mx[qb] = v;
            need[qb] = (v - m_ref[qb]) * c[qb] > kRescaleThreshold;
        }
        if (__builtin_amdgcn_ballot_w64(need[0] || need[1]) != 0) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const float alpha = need[qb] ? __builtin_amdgcn_exp2f((m_ref[qb] - mx[qb]) * c[qb]) : 1.f;
                m_ref[qb] = need[qb] ? mx[qb] : m_ref[qb];
                l[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) O[db][qb][r] *= alpha;
            }
        }

        // probabilities, rounded to bf16, in B-operand order: P[qb][kb][g] holds keys of group g
        bf16x8 P[2][2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float mc = m_ref[qb] * c[qb];
            float sum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float pv = __builtin_amdgcn_exp2f(fmaf(S[kb][qb][8 * g + e], c[qb], -mc));
                        const __bf16 pb = (__bf16)pv;
                        P[qb][kb][g][e] = pb;
                        sum += (float)pb;
                    }
            l[qb] += sum;
        }

        // O^T[db][qb] += V^T_{kb,g,db} P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int db = 0; db < 2; ++db) {
                    const bf16x8 a = *(const bf16x8 *)(cur + kb * kBlockBytes + 4096 +
                                                       ((g * 2 + db) * 64 + lane) * 16);
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
                        O[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, P[qb][kb][g], O[db][qb], 0, 0, 0);
                }

        if (more) {
            uint4 *dst = (uint4 *)(lds + ((t + 1) & 1) * kTileBytes);
#pragma unroll
            for (int i = 0; i < NPRE; ++i) dst[tid + i * NT] = pre[i];
        }
        __syncthreads();
    }

    // ---- normalise and store: lane holds O^T[32db + 8g + 4hf + 0..3][query] -----------------
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float lt = l[qb] + xhalf(l[qb]);
        const float inv = 1.f / lt;
        const int wq = wave * 64 + qb * 32 + l32;
        __bf16 *op = p.o + (row0 + wq) * p.ld_o + h * kDHead + 4 * hf;
        if (qvalid[qb]) {
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 ov;
#pragma unroll
                    for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(O[db][qb][4 * g + e] * inv);
                    *(bf16x4 *)(op + 32 * db + 8 * g) = ov;
                }
        } else if (!SUMI && q0 + wq < Lpad) {
            const bf16x4 z = {(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) *(bf16x4 *)(op + 32 * db + 8 * g) = z;
        }
    }
}

KParams make_params(const AttnArgs &a, int n_qtiles)
{
    KParams p;
    p.layer_base = a.cache.layer_base;
    p.hist_len = a.cache.hist_len;
    p.tok_off = a.cache.tok_off;
    p.order = a.cache.order;
    p.cand_off = a.cand_off;
    p.q = (const __bf16 *)a.q;
    p.k_self = (const __bf16 *)a.k_self;
    p.v_self = (const __bf16 *)a.v_self;
    p.scen = a.scen;
    p.beh = a.beh;
    p.tau = a.tau;
    p.o = (__bf16 *)a.o;
    p.ld_q = a.ld_q;
    p.ld_kv = a.ld_kv;
    p.ld_o = a.ld_o;
    p.B = a.cache.B;
    p.H = a.H;
    p.n_scen = a.n_scen;
    p.n_beh = a.n_beh;
    p.sub_len = a.sub_len;
    p.n_qtiles = n_qtiles;
    p.scale_log2e = a.qk_scale * 1.4426950408889634f;
    return p;
}

template <int NW, bool SUMI>
hipError_t launch(const AttnArgs &a, hipStream_t s)
{
    constexpr int TQ = NW * 64;
    const int n_qtiles = (a.max_rows_per_user + TQ - 1) / TQ;
    const int groups = (a.cache.B * a.H + 7) / 8;
    const int64_t grid = (int64_t)8 * n_qtiles * groups;
    if (grid <= 0 || grid > 0x7fffffff) return hipErrorInvalidValue;
    const KParams p = make_params(a, n_qtiles);
    hipLaunchKernelGGL((attn_bf16_kernel<NW, SUMI>), dim3((unsigned)grid), dim3(NW * 64), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_sumi_bf16(const AttnArgs &a, hipStream_t s)
{
    return launch<2, true>(a, s);
}

hipError_t launch_attn_hist_bf16(const AttnArgs &a, hipStream_t s)
{
    return launch<2, false>(a, s);
}

}  // namespace climber
