// bf16 MFMA flash attention for gfx950 (CDNA4): the SUMI candidate pass and the block-diagonal
// history pass of Climber (arXiv 2502.09888): Eq. (3) attention with a per-query-row temperature,
// the "single user, multiple items" mask of Sec. 3.2 and the per-subsequence attention of
// Sec. 3.1.2.
//
// Shape of the computation (one workgroup = one (user, head, tile of NW*64 query rows)):
//   - the transposed problem is computed: S^T = K Q^T and O^T = V^T P^T with
//     v_mfma_f32_32x32x16_bf16.  In the accumulator layout of that instruction a lane owns ONE
//     query column (lane % 32), so the softmax statistics of a query are per-lane scalars and the
//     probabilities leave the S^T accumulator already in the B-operand layout the P V product
//     needs (the cache stores V with the matching key permutation).
//   - history K/V tiles of 64 keys are copied HBM -> LDS directly (global_load_lds, no register
//     staging; the cache is stored as MFMA fragments so the copy is linear) into a ring of 3
//     buffers (the tile being computed, the next one, and the one being refilled) and are reused
//     by every wave, i.e. by the whole query tile.  Query rows and the candidates' own key / value
//     rows arrive the same way in a landing buffer behind the ring, one slice per wave.
//   - FAST pass.  Softmax does not depend on the reference subtracted from the logits as long as
//     numerator and denominator share it, and fp32 / bf16 carry 8 exponent bits, so for logits of
//     ordinary size NO reference is needed at all: p = exp2(t) with t the logit in log2 units, one
//     v_exp_f32, half a v_cvt_pk_bf16_f32 and one v_add_f32 (denominator) per logit -- no row
//     maximum, no subtraction, no rescale of O.  Two forms, chosen per wave from the first block's
//     logits: "folded", q' = bf16(q * c) with c = qk_scale*log2(e)/tau_row, so that t = <q',k>
//     comes straight out of the MFMA (rounding q*c costs every logit a relative 2^-9: kept only
//     while a row's denominator stays in [kDenomLo, kDenomHi]); and "exact scale", q as given and
//     t = <q,k> * c in fp32 (one more multiplication per logit; the denominator only has to stay
//     inside the exponent range, [kDenomLoExact, kDenomHiExact]; the denominator is summed from the
//     probabilities as rounded to bf16, so that a one-hot row does not carry the rounding of its
//     dominant term into the output).  Only the candidate pass folds; history rows and the bias
//     variants always take the exact form.  The loop is software pipelined
//     over 32-key blocks: the S^T MFMAs of block i+1 are issued before the exponentials of block
//     i, so matrix and vector pipes overlap inside one wave.
//   - SAFE pass.  If any row's denominator leaves its window (or is not finite) the workgroup
//     redoes its work with the classical online softmax: unscaled q, fp32 scale
//     p = exp2(s*c - m*c), running row maximum (moved when exceeded by 2^8, O and l rescaled).
//     This covers logits of any size.  The choice of form is per wave and the redo per workgroup,
//     so a row's rounding depends on whether a neighbour of its tile has large logits: results
//     are bitwise independent of the other rows only within one form.
//   - SUMI: the candidate's own key / value join the softmax as one more member (FAST: between
//     two tiles, from the landing buffer; SAFE: as the initial state): the "+ itself" term of the
//     mask.
#include "attn_common.h"

#include <type_traits>

namespace climber {
namespace {

using namespace attn;

constexpr int kTileKeys = 64;                // keys per LDS tile = 2 cache blocks
constexpr int kTileBytes = 2 * kBlockBytes;  // 16 KiB
constexpr int kStages = 3;                   // LDS ring of K/V tiles

struct KParams {
    const uint8_t *layer_base;
    const int32_t *hist_len, *tok_off, *order, *cand_off;
    const __bf16 *q, *k_self, *v_self;
    const int32_t *scen, *beh;
    const float *tau;
    __bf16 *o;
    int64_t ld_q, ld_kv, ld_o;
    int B, H, n_scen, n_beh, sub_len, n_qtiles;
    int uni_len, uni_pad;  // >= 0: every user has this valid / padded history length
    int uni_cand;          // >= 0: every user has this many candidates (SUMI)
    float scale_log2e, inv_qk_scale;
    BiasArgs bias;  // relative attention bias (the BIAS variants of the kernel)
    int bias_H;
};

// wait until at most `tiles_in_flight` later tiles (NPRE loads each) are still outstanding
template <int NPRE>
__device__ __forceinline__ void wait_tiles(int tiles_in_flight)
{
    static_assert(NPRE == 2 || NPRE == 4 || NPRE == 8, "vmcnt immediates below");
    if (tiles_in_flight >= 2) {
        if (NPRE == 8) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        if (NPRE == 4) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        if (NPRE == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    } else if (tiles_in_flight == 1) {
        if (NPRE == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        if (NPRE == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        if (NPRE == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
}

// BIAS: the relative attention bias of Eq. (3) joins the logits before the temperature divide.  A
// lane works its 16 bias values of a block out of the two bucket tables (clipped relative position,
// log2 bucket of the time distance; one table row per (scenario, behaviour, head) of the query) and
// hands them to the S^T MFMAs as the initial value of the accumulator, scaled like the logits
// (FAST: by log2(e)/tau, SAFE: by 1/qk_scale, the fp32 scale of the pass doing the rest).
template <int NW, int QB, bool SUMI, bool CAUSAL = false, bool BIAS = false>
__global__ __launch_bounds__(NW * 64, 2) void attn_bf16_kernel(const KParams p)
{
    static_assert(!(SUMI && CAUSAL), "the causal flag concerns the history pass");
    static_assert(kStages == 3, "tile t+1 is read while tile t is computed and one more is in flight; "
                                "every wait in the FAST loop drains all copies");
    constexpr int NT = NW * 64;
    constexpr int WQ = 32 * QB;  // query rows per wave
    constexpr int TQ = NW * WQ;  // query rows per workgroup
    constexpr int NPRE = kTileBytes / 16 / NT;
    // BIAS: this head's rows of the two bias tables live behind the landing buffer when they fit
    // (lookups per logit: LDS gathers instead of gathers from global memory)
    constexpr int kBiasLds = BIAS ? kBiasLdsFloats : 0;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kStages * kTileBytes + TQ * 128 + kBiasLds * 4];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar
    int l32 = lane & 31;
    const int hf = lane >> 5;

    // workgroup -> (user, head, query tile).  Consecutive workgroup ids are dealt round-robin to
    // the 8 XCDs; tiles of the same (user, head) get ids congruent mod 8 so that they run on one
    // XCD and share its L2 copy of that head's K/V.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, j = wg >> 3;
    const int qt = j % p.n_qtiles;
    const int bh = (j / p.n_qtiles) * 8 + xcd;
    if (bh >= p.B * p.H) return;
    // Uniform batches (the host knows): user geometry comes from kernel arguments, which saves
    // two dependent trips to memory at the start of every workgroup.
    const int h = bh % p.H;
    int b = bh / p.H, Lb, t0, Lpad;
    if (p.uni_len >= 0) {
        Lb = p.uni_len;
        Lpad = p.uni_pad;
        t0 = b * Lpad;
    } else {
        b = p.order[b];
        Lb = p.hist_len[b];
        t0 = p.tok_off[b];
        Lpad = p.tok_off[b + 1] - t0;
    }

    const int q0 = qt * TQ;
    int64_t row0;
    int nq, k_lo, k_hi;
    if (SUMI) {
        int c0, Mb;
        if (p.uni_cand >= 0) {
            Mb = p.uni_cand;
            c0 = b * Mb;
        } else {
            c0 = p.cand_off[b];
            Mb = p.cand_off[b + 1] - c0;
        }
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
        if (CAUSAL) k_hi = min(k_hi, q0 + TQ);  // no query of this tile sees a later key
    }
    // Causal history pass: token i sees the keys j <= i of its subsequence.  A block of 32 keys is
    // masked per lane (the lane's queries are q0 + wave*WQ + 32 qb + lane%32) when it reaches up to
    // or beyond the wave's first query; blocks wholly beyond a wave's queries contribute zeros.
    int lim[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) lim[qb] = q0 + wave * WQ + qb * 32 + l32 + 1;
    const int q_wave_lo = q0 + wave * WQ;
    auto causal = [&](f32x16 (&S)[QB], int blk_lo) __attribute__((always_inline)) {
        if (CAUSAL && blk_lo + kBlockKeys > q_wave_lo) mask_causal(S, hf, blk_lo, lim);
    };
    const int n_tiles = (k_hi - k_lo + kTileKeys - 1) / kTileKeys;
    const uint8_t *kv = p.layer_base + ((size_t)t0 * p.H + (size_t)h * Lpad) * (kDHead * 4) +
                        (size_t)(k_lo / kBlockKeys) * kBlockBytes;

    // K/V tiles go HBM -> LDS directly (no register staging): every wave copies NPRE slabs of
    // 1 KiB (64 lanes x 16 B) per tile; the LDS image equals the HBM image.
    // tile t into the ring stage at byte offset `stage` (= (t % kStages) * kTileBytes)
    auto issue_tile_at = [&](int t, int stage) __attribute__((always_inline)) {
        glb_u8 *src = (glb_u8 *)(kv + (size_t)t * kTileBytes + (size_t)tid * 16);
        lds_u8 *dst = (lds_u8 *)lds + stage + wave * 1024;
#pragma unroll
        for (int i = 0; i < NPRE; ++i)
            __builtin_amdgcn_global_load_lds(src + i * NT * 16, dst + i * NT * 16, 16, 0, 0);
    };
    auto issue_tile = [&](int t) __attribute__((always_inline)) { issue_tile_at(t, (t % kStages) * kTileBytes); };
    QState<QB> st;
    // per query row of the lane: position, time stamp, rows of the two bias tables, logit scale
    int b_pos[QB];
    uint32_t b_ts[QB];               // time stamp, sign bit flipped (bias_time_key)
    const float *b_prow[QB], *b_trow[QB];  // the row's slices of the two tables (LDS copy or global)
    float fb[QB], bias_self[QB];
    // LDS copy of the head's table rows: [n_tau][n_pos] then [n_tau][n_time]
    const float *bias_lds = (const float *)(lds + kStages * kTileBytes + TQ * 128);
    const int n_groups = p.n_scen * p.n_beh;
    const bool bias_in_lds = BIAS && n_groups * (p.bias.n_pos + p.bias.n_time) <= kBiasLds;
    if constexpr (BIAS) {
        if (bias_in_lds) {  // visible to the workgroup after the barrier that follows the first tile's wait
            float *dst = (float *)(lds + kStages * kTileBytes + TQ * 128);
            const int np_ = p.bias.n_pos, nt_ = p.bias.n_time;
            for (int i = tid; i < n_groups * np_; i += NT)
                dst[i] = p.bias.pos_table[((i / np_) * p.bias_H + h) * np_ + i % np_];
            for (int i = tid; i < n_groups * nt_; i += NT)
                dst[n_groups * np_ + i] = p.bias.time_table[((i / nt_) * p.bias_H + h) * nt_ + i % nt_];
        }
    }
    auto qk = [&](const KFrags &kf, f32x16 (&S)[QB], int blk_lo) __attribute__((always_inline)) {
        if constexpr (BIAS) {
            const int half = (p.bias.n_pos - 1) >> 1;
            const int64_t kr = (int64_t)t0 + blk_lo + 4 * hf;  // packed history row of the lane's first key
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int4 kp = *(const int4 *)(p.bias.key_pos + kr + 8 * g4);
                const int4 kt = *(const int4 *)(p.bias.key_ts + kr + 8 * g4);
                const int kpe[4] = {kp.x, kp.y, kp.z, kp.w};
                const uint32_t kte[4] = {bias_time_key(kt.x), bias_time_key(kt.y), bias_time_key(kt.z), bias_time_key(kt.w)};
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) {
                        const int ip = bias_bucket_pos(b_pos[qb], kpe[e], half);
                        const int it = bias_bucket_time_u(b_ts[qb], kte[e], p.bias.n_time);
                        S[qb][4 * g4 + e] = fb[qb] * (b_prow[qb][ip] + b_trow[qb][it]);
                    }
            }
            qk_block_acc(st, kf, S);
        } else {
            qk_block(st, kf, S);
        }
    };

    // FAST start: the raw query rows stay in st.qf and the row scale in st.c until the first block's
    // logits have shown which form of the pass the wave takes; empty state (the candidate's own
    // key/value joins later, from the landing buffer).
    auto init_fast = [&](const float (&c)[QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            st.c[qb] = c[qb];
            st.l[qb] = 0.f;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.O[db][qb][r] = 0.f;
        }
    };
    // SAFE start (rare): everything is fetched again, straight from global memory, so that nothing
    // of it has to stay in registers across the FAST pass (the empty asm keeps the compiler from
    // reusing the FAST pass's row addresses).  q unscaled; the own key/value is the first member
    // of the softmax and its logit the first reference.
    auto init_safe = [&]() __attribute__((always_inline)) {
        int l32s = l32, hfs = hf;
        asm volatile("" : "+v"(l32s), "+v"(hfs));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int64_t row = row0 + min(wave * WQ + qb * 32 + l32s, nq - 1);
            const int sc = min(max(p.scen[row], 0), p.n_scen - 1);
            const int bhv = min(max(p.beh[row], 0), p.n_beh - 1);
            st.c[qb] = p.scale_log2e / p.tau[sc * p.n_beh + bhv];
            const __bf16 *qp = p.q + row * p.ld_q + h * kDHead + 8 * hfs;
            float dot = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                st.qf[qb][s] = *(const bf16x8 *)(qp + 16 * s);
                if (SUMI) {
                    const bf16x8 kk = *(const bf16x8 *)(p.k_self + row * p.ld_kv + h * kDHead + 8 * hfs + 16 * s);
#pragma unroll
                    for (int e = 0; e < 8; ++e) dot += (float)st.qf[qb][s][e] * (float)kk[e];
                }
            }
            // SUMI: the own logit (both halves add the same two numbers).  History pass: no member
            // of the row is known yet; a reference far below any logit makes the first block's
            // maximum the reference (0 would leave rows whose logits are all very negative with an
            // empty sum).  Every row sees a key of its first block, so the reference is finite
            // before the first exponential.
            if constexpr (BIAS) fb[qb] = p.inv_qk_scale;  // SAFE: logits in raw units, scaled by c in fp32
            st.m_ref[qb] = SUMI ? dot + xhalf(dot) + (BIAS ? fb[qb] * bias_self[qb] : 0.f) : kSafeNoRef;
            st.l[qb] = (SUMI && hfs == 0) ? 1.f : 0.f;
            if (SUMI) {
                const __bf16 *vp = p.v_self + row * p.ld_kv + h * kDHead + 4 * hfs;
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const bf16x4 vv = *(const bf16x4 *)(vp + 32 * db + 8 * g);
#pragma unroll
                        for (int e = 0; e < 4; ++e) st.O[db][qb][4 * g + e] = (float)vv[e];
                    }
            } else {
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) st.O[db][qb][r] = 0.f;
            }
        }
    };
    auto prologue = [&]() __attribute__((always_inline)) {
        // tiles 0 .. kStages-2 in flight (SAFE pass)
        for (int t = 0; t < kStages - 1 && t < n_tiles; ++t) issue_tile(t);
    };

    // ---- FAST pass, software pipelined over 32-key blocks -----------------------------------
    // Start-up order = what the first MFMA needs first: tile 0, the query rows, then the tiles
    // that are only needed a little later (loads return in order).
    // ... and the row ids and the temperature table, whose values are needed together with the
    // query rows.  The table is staged in the last ring buffer (first refilled during tile 0, i.e.
    // after the lookups), so the per-row lookup is not a second dependent trip to memory.
    constexpr int kTauLds = kTileBytes / 4;
    float *tau_lds = (float *)(lds + (kStages - 1) * kTileBytes);
    const int n_tau = p.n_scen * p.n_beh;
    const bool tau_in_lds = n_tau <= kTauLds;
    // Query rows land in the landing buffer behind the ring: whole 128-byte rows, copied
    // HBM -> LDS by the wave that owns them (8 lanes per row, so every request is a full line),
    // 16-byte chunks XOR-swizzled by the row number so that the fragment reads below are
    // conflict-free.  A wave only ever touches its own slice of that buffer.
    uint8_t *rows_lds = lds + kStages * kTileBytes + wave * (WQ * 128);
    auto issue_rows = [&](const __bf16 *base, int64_t ld) __attribute__((always_inline)) {
        // wave-uniform base (the tile's first row) in scalar registers + a 32-bit offset per lane (at most
        // TQ - 1 rows): half the address registers of 64-bit lane addresses
        const uint8_t *sb = uniform_ptr((const uint8_t *)(base + row0 * ld + h * kDHead));
#pragma unroll
        for (int i = 0; i < WQ / 8; ++i) {
            const int pos = i * 64 + lane, r = pos >> 3, c = (pos & 7) ^ (r & 7);
            const uint32_t off = ((uint32_t)min(wave * WQ + r, nq - 1) * (uint32_t)ld + (uint32_t)c * 8u) * 2u;
            __builtin_amdgcn_global_load_lds((glb_u8 *)sb + off, (lds_u8 *)rows_lds + i * 1024, 16, 0, 0);
        }
    };
    auto load_q_lds = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int r = qb * 32 + l32, c = (2 * s + hf) ^ (r & 7);
                st.qf[qb][s] = *(const bf16x8 *)(rows_lds + r * 128 + c * 16);
            }
    };
    // FAST, SUMI: the candidate's own key/value.  Their rows travel through the same landing
    // buffer while the history loop runs (keys first, values once the keys are consumed), so no
    // wave ever waits for them: weight w = exp2(<q', k_own>), then O += w * v_own.
    float w_own[QB];
    bool fold = false;  // the wave runs the pass with the scale folded into a bf16 query (decided below)
    auto own_k = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int r = qb * 32 + l32;
            float dot = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 kk = *(const bf16x8 *)(rows_lds + r * 128 + (((2 * s + hf) ^ (r & 7)) * 16));
                // read q' back out of the packed operand registers (the empty asm hides where
                // they came from: otherwise the unpacked halves stay live across the whole loop)
                u32x4 qv = __builtin_bit_cast(u32x4, st.qf[qb][s]);
                asm volatile("" : "+v"(qv));
                const bf16x8 qq = __builtin_bit_cast(bf16x8, qv);
#pragma unroll
                for (int e = 0; e < 8; ++e) dot += (float)qq[e] * (float)kk[e];
            }
            w_own[qb] = __builtin_amdgcn_exp2f((dot + xhalf(dot) + (BIAS ? fb[qb] * bias_self[qb] : 0.f)) * (fold ? 1.f : st.c[qb]));
            st.l[qb] += hf == 0 ? w_own[qb] : 0.f;
        }
    };
    auto own_v = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int r = qb * 32 + l32;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const bf16x4 vv =
                        *(const bf16x4 *)(rows_lds + r * 128 + (((4 * db + g) ^ (r & 7)) * 16) + 8 * hf);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        st.O[db][qb][4 * g + e] = fmaf(w_own[qb], (float)vv[e], st.O[db][qb][4 * g + e]);
                }
        }
    };
    if (n_tiles > 0) issue_tile(0);
    int tau_idx[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) tau_idx[qb] = p.scen[row0 + min(wave * WQ + qb * 32 + l32, nq - 1)];
    int beh_id[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) beh_id[qb] = p.beh[row0 + min(wave * WQ + qb * 32 + l32, nq - 1)];
    float tau_first = 0.f;
    if (tau_in_lds && tid < n_tau) tau_first = p.tau[tid];
    __builtin_amdgcn_sched_barrier(0);
    issue_rows(p.q, p.ld_q);
    if (n_tiles > 1) issue_tile(1);
    __builtin_amdgcn_sched_barrier(0);
    if (tau_in_lds) {
        if (tid < n_tau) tau_lds[tid] = tau_first;
        for (int i = tid + NT; i < n_tau; i += NT) tau_lds[i] = p.tau[i];
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int sc = min(max(tau_idx[qb], 0), p.n_scen - 1);
        const int bhv = min(max(beh_id[qb], 0), p.n_beh - 1);
        tau_idx[qb] = sc * p.n_beh + bhv;
        if constexpr (BIAS) {
            const int64_t row = row0 + min(wave * WQ + qb * 32 + l32, nq - 1);
            b_pos[qb] = p.bias.q_pos[row];
            b_ts[qb] = bias_time_key(p.bias.q_ts[row]);
            const int grow = (tau_idx[qb] * p.bias_H + h);
            // a candidate's own key: zero distance in position and time
            bias_self[qb] = p.bias.pos_table[grow * p.bias.n_pos + ((p.bias.n_pos - 1) >> 1)] +
                            p.bias.time_table[grow * p.bias.n_time];
            // rows of the lane's (scenario, behaviour) pair: in the LDS copy, or in the tables themselves
            b_prow[qb] = bias_in_lds ? bias_lds + tau_idx[qb] * p.bias.n_pos : p.bias.pos_table + grow * p.bias.n_pos;
            b_trow[qb] = bias_in_lds ? bias_lds + n_groups * p.bias.n_pos + tau_idx[qb] * p.bias.n_time
                                     : p.bias.time_table + grow * p.bias.n_time;
        }
    }
    // tile 0 and the query rows of this wave have landed (only tile 1 may still be in flight);
    // tau_lds is visible to the workgroup after the bare barrier (a fence would also wait for
    // tile 1)
    if (n_tiles > 1)
        wait_tiles<NPRE>(1);
    else
        wait_tiles<NPRE>(0);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    {
        float c[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            c[qb] = p.scale_log2e / (tau_in_lds ? tau_lds[tau_idx[qb]] : p.tau[tau_idx[qb]]);
        if constexpr (BIAS) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) fb[qb] = p.inv_qk_scale;  // bias in the units of the raw <q, k>
        }
        load_q_lds();
        init_fast(c);
    }
    if (n_tiles > 0) {
        f32x16 S0[QB], S1[QB];
        bf16x8 P[QB][2];
        // every wave has looked up its temperatures in the table staged in the last ring stage,
        // which the first refill (tile 2) overwrites
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        {
            const KFrags k0 = load_k(lds, lane);
            qk(k0, S0, k_lo);
            // Which form of the FAST pass?  Folding the row scale c = qk_scale*log2(e)/tau into the bf16
            // query saves a multiplication per logit but rounds q*c to 8 bits, an error of 2^-9 of every
            // logit: harmless while the exponents stay small.  The first block's exponents s*c tell:
            // their root mean square estimates the spread of the row's exponents, and with it the size of
            // the denominator (log2 of it ~ log2(keys) + 0.35 spread^2 for bell-shaped logits).  Below
            // kPilotSpread for every row of the wave -> fold; otherwise the queries stay exact and every
            // logit is multiplied by c in fp32.  A wrong guess is caught by the window on the denominators.
            // (Waves decide on their own: both forms read the same tiles and pass the same barriers.)
            bool big = k_hi - k_lo < kFoldMinKeys;  // (a short history: too few keys to average the folded form's error over)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float ss = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) ss = fmaf(S0[qb][r], S0[qb][r], ss);
                ss += xhalf(ss);  // the 32 keys of the block
                big |= !(ss * st.c[qb] * st.c[qb] < kBlockKeys * kPilotSpread * kPilotSpread);
            }
            // Only the candidate pass folds, and only against a history of some length: its rows then have
            // many comparable keys to average the per-logit error over.  History rows
            // see one subsequence (a few keys only under the causal flag) and can be sharply peaked, where
            // the folded form's error shows in the output; the bias variants have larger logits and their
            // cost lies elsewhere.  Those always take the exact form.
            fold = SUMI && !BIAS && __builtin_amdgcn_ballot_w64(big) == 0;
            if (fold) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
                    for (int sx = 0; sx < 4; ++sx) {
                        const bf16x8 qq = st.qf[qb][sx];
#pragma unroll
                        for (int e = 0; e < 8; ++e) st.qf[qb][sx][e] = (__bf16)((float)qq[e] * st.c[qb]);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) S0[qb][r] *= st.c[qb];  // the first block's logits, formed already
                    if constexpr (BIAS) fb[qb] = st.c[qb] * p.inv_qk_scale;  // log2(e) / tau
                }
            }
            causal(S0, k_lo);
        }
        auto run = [&](auto fold_tag) __attribute__((always_inline)) {
        constexpr bool FOLD = decltype(fold_tag)::value;
        // p = exp2(t): t straight from the MFMA (FOLD), or s * c in fp32
        auto soft = [&](const f32x16 (&S)[QB]) __attribute__((always_inline)) {
            if constexpr (FOLD) {
                softmax_fast(st, S, P);
            } else {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) st.l[qb] += exp_pack<true>(S[qb], st.c[qb], 0.f, P[qb]);
            }
        };
        // One step = every tile but the last: 64 unmasked keys.  EV numbers the tile that becomes
        // readable in the middle of the step when something rides along with its refill or is
        // due afterwards (the own rows of a candidate tile); 0 = plain step.  The steps with
        // events are peeled off the loop: inside it they would make the compiler shuffle the
        // accumulators around the branches.
        // The ring stages of tiles t, t + 1 and t + 2 come in as byte offsets that the loop carries
        // along: derived from t % kStages inside the loop, every fragment address took two vector
        // additions and its own address register instead of an immediate.
        auto tile_step = [&](int t, int so_cur, int so_nxt, int so_fill, auto ev_tag) __attribute__((always_inline)) {
            constexpr int EV = decltype(ev_tag)::value;
            const uint8_t *cur = lds + so_cur;
            const uint8_t *nxt = lds + so_nxt;
            {   // block 0 of tile t: its logits are in S0; start block 1's logits
                const KFrags k1 = load_k(cur + kBlockBytes, lane);
                const VFrags v0 = load_v(cur, lane);
                __builtin_amdgcn_sched_barrier(0);
                qk(k1, S1, k_lo + t * kTileKeys + kBlockKeys);
                causal(S1, k_lo + t * kTileKeys + kBlockKeys);
                soft(S0);
                pv_block(st, v0, P);
            }
            // tile t+1 becomes readable (kStages == 3: no later tile is in flight, the wait
            // drains every copy, own rows included); the own rows ride along with the refill
            wait_tiles<NPRE>(0);
            __builtin_amdgcn_s_barrier();
            // the landing slice is overwritten: this wave's earlier reads of it must have returned
            if (SUMI && (EV == 1 || EV == 3)) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (SUMI && EV == 1) issue_rows(p.k_self, p.ld_kv);
            if (SUMI && EV == 3) issue_rows(p.v_self, p.ld_kv);
            if (t + 2 < n_tiles) issue_tile_at(t + 2, so_fill);
            if (SUMI && EV == 2) own_k();
            if (SUMI && EV == 4) own_v();
            {   // block 1 of tile t; start block 0 of tile t+1
                const KFrags k0 = load_k(nxt, lane);
                const VFrags v1 = load_v(cur + kBlockBytes, lane);
                __builtin_amdgcn_sched_barrier(0);
                qk(k0, S0, k_lo + (t + 1) * kTileKeys);
                causal(S0, k_lo + (t + 1) * kTileKeys);
                soft(S1);
                pv_block(st, v1, P);
            }
        };
        static_assert(kStages == 3, "stage offsets below are written out for a ring of three");
        constexpr int T1 = kTileBytes, T2 = 2 * kTileBytes;
        if (n_tiles > 1) {
            tile_step(0, 0, T1, T2, std::integral_constant<int, 1>{});
            if (n_tiles > 2) {
                tile_step(1, T1, T2, 0, std::integral_constant<int, 2>{});
                if (n_tiles > 3) {
                    tile_step(2, T2, 0, T1, std::integral_constant<int, 3>{});
                    if (n_tiles > 4) {
                        tile_step(3, 0, T1, T2, std::integral_constant<int, 4>{});
                        int so_cur = T1, so_nxt = T2, so_fill = 0;
                        for (int t = 4; t + 1 < n_tiles; ++t) {
                            tile_step(t, so_cur, so_nxt, so_fill, std::integral_constant<int, 0>{});
                            const int so = so_cur;
                            so_cur = so_nxt, so_nxt = so_fill, so_fill = so;
                        }
                    }
                }
            }
        }
        {   // last tile: 1..64 keys, S0 holds its first block
            const int t = n_tiles - 1;
            const uint8_t *cur = lds + (t % kStages) * kTileBytes;
            const int tile_lo = k_lo + t * kTileKeys;
            const bool two = tile_lo + kBlockKeys < k_hi;
            if (two) {
                const KFrags k1 = load_k(cur + kBlockBytes, lane);
                qk(k1, S1, tile_lo + kBlockKeys);
                causal(S1, tile_lo + kBlockKeys);
            }
            if (tile_lo + kBlockKeys > k_hi) mask_block(S0, hf, tile_lo, k_hi);
            {
                const VFrags v0 = load_v(cur, lane);
                soft(S0);
                pv_block(st, v0, P);
            }
            if (two) {
                if (tile_lo + kTileKeys > k_hi) mask_block(S1, hf, tile_lo + kBlockKeys, k_hi);
                const VFrags v1 = load_v(cur + kBlockBytes, lane);
                soft(S1);
                pv_block(st, v1, P);
            }
        }
        };
        if (__builtin_expect(fold, 1))
            run(std::true_type{});
        else
            run(std::false_type{});
    }

    // lane % 32 again, opaquely: otherwise the compiler carries the old copy across the loop (in
    // scratch memory, which would be this kernel's only use of it)
    asm volatile("v_and_b32 %0, 31, %1" : "=v"(l32) : "v"(tid));
    if (SUMI) {  // whatever part of the own-row schedule a short history left undone
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (n_tiles < 2) issue_rows(p.k_self, p.ld_kv);
        if (n_tiles < 3) {
            wait_tiles<NPRE>(0);
            own_k();
        }
        if (n_tiles < 4) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            issue_rows(p.v_self, p.ld_kv);
        }
        if (n_tiles < 5) {
            wait_tiles<NPRE>(0);
            own_v();
        }
    }

    // ---- SAFE pass (rare): whole workgroup redoes its rows with a running maximum -----------
    float lt[QB];
    bool bad = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        lt[qb] = st.l[qb] + xhalf(st.l[qb]);
        bad |= fold ? !(lt[qb] > kDenomLo && lt[qb] < kDenomHi) : !(lt[qb] > kDenomLoExact && lt[qb] < kDenomHiExact);
    }
    // Workgroup-wide OR of `bad` through the (idle) landing buffer: one flag per wave in its own
    // slice, one barrier; the barrier also orders the reuse of the LDS ring below.
    int *flag_lds = (int *)(lds + kStages * kTileBytes);
    // (the ballot is taken by the whole wave: inside the branch it would see lane 0 only)
    const int wave_bad = __builtin_amdgcn_ballot_w64(bad) != 0;
    if (lane == 0) flag_lds[wave * (WQ * 32)] = wave_bad;
    __syncthreads();
    int any_bad = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) any_bad |= flag_lds[w * (WQ * 32)];
    if (any_bad) {
        prologue();
        init_safe();
        for (int t = 0; t < n_tiles; ++t) {
            wait_tiles<NPRE>(min(t + kStages - 1, n_tiles) - (t + 1));
            __builtin_amdgcn_s_barrier();
            if (t + kStages - 1 < n_tiles) issue_tile(t + kStages - 1);
            const uint8_t *cur = lds + (t % kStages) * kTileBytes;
            const int tile_lo = k_lo + t * kTileKeys;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const int blk_lo = tile_lo + blk * kBlockKeys;
                if (blk_lo < k_hi) {
                    f32x16 S[QB];
                    bf16x8 P[QB][2];
                    const KFrags kf = load_k(cur + blk * kBlockBytes, lane);
                    qk(kf, S, blk_lo);
                    if (blk_lo + kBlockKeys > k_hi) mask_block(S, hf, blk_lo, k_hi);
                    causal(S, blk_lo);
                    softmax_safe(st, S, P);
                    const VFrags vf = load_v(cur + blk * kBlockBytes, lane);
                    pv_block(st, vf, P);
                }
            }
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) lt[qb] = st.l[qb] + xhalf(st.l[qb]);
    }

    // ---- normalise and store ----------------------------------------------------------------
    // A lane holds O^T[32db + 8g + 4hf + 0..3][query]: 8-byte pieces of 32 different rows.  Each
    // wave turns its 32 x 64 block around in its own corner of the (now idle) LDS ring so that
    // the global stores are whole 128-byte rows, 16 bytes per lane.
    if (any_bad) __syncthreads();  // SAFE pass: every wave is done reading K/V tiles
    constexpr int kRowPitch = 144;  // 128 B of a row + 16 B pad, keeps 16-byte alignment
    uint8_t *tr = lds + wave * (32 * kRowPitch);
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
                *(bf16x4 *)(tr + l32 * kRowPitch + (32 * db + 8 * g + 4 * hf) * 2) = ov;
            }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = i * 64 + lane, r = id >> 3, cc = id & 7;
            const int wq = wave * WQ + qb * 32 + r;
            uint4 val = *(const uint4 *)(tr + r * kRowPitch + cc * 16);
            __bf16 *op = p.o + (row0 + wq) * p.ld_o + h * kDHead + cc * 8;
            if (wq < nq) {
                __builtin_nontemporal_store(__builtin_bit_cast(u32x4, val), (u32x4 *)op);
            } else if (!SUMI && q0 + wq < Lpad) {
                *(uint4 *)op = uint4{0, 0, 0, 0};
            }
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
    p.inv_qk_scale = 1.f / a.qk_scale;
    p.bias = a.bias;
    p.bias_H = a.H;
    p.uni_len = a.uni_len;
    p.uni_pad = a.uni_pad;
    p.uni_cand = a.uni_cand;
    return p;
}

template <int NW, int QB, bool SUMI, bool CAUSAL = false, bool BIAS = false>
hipError_t launch(const AttnArgs &a, hipStream_t s)
{
    constexpr int TQ = NW * 32 * QB;
    const int n_qtiles = (a.max_rows_per_user + TQ - 1) / TQ;
    const int groups = (a.cache.B * a.H + 7) / 8;
    const int64_t grid = (int64_t)8 * n_qtiles * groups;
    if (grid <= 0 || grid > 0x7fffffff) return hipErrorInvalidValue;
    const KParams p = make_params(a, n_qtiles);
    hipLaunchKernelGGL((attn_bf16_kernel<NW, QB, SUMI, CAUSAL, BIAS>), dim3((unsigned)grid), dim3(NW * 64), 0, s, p);
    return hipGetLastError();
}

// Query-tile shape: 4 waves x QB blocks of 32 queries per workgroup.  QB = 2 (256 queries) re-reads
// a head's K/V from L2 half as often and reuses every LDS fragment for two MFMAs; QB = 1 (128
// queries) keeps two waves per SIMD busy when a head has few queries.
}  // namespace

hipError_t launch_attn_sumi_bf16(const AttnArgs &a, hipStream_t s)
{
    if (a.bias.pos_table) return launch<4, 1, true, false, true>(a, s);
    return a.max_rows_per_user > 128 ? launch<4, 2, true>(a, s) : launch<4, 1, true>(a, s);
}

hipError_t launch_attn_hist_bf16(const AttnArgs &a, hipStream_t s)
{
    // a query tile must lie inside one subsequence (sub_len is 0 or a multiple of 128)
    if (a.bias.pos_table) return a.causal ? launch<4, 1, false, true, true>(a, s) : launch<4, 1, false, false, true>(a, s);
    const bool wide = a.sub_len % 256 == 0;
    if (a.causal) return wide ? launch<4, 2, false, true>(a, s) : launch<4, 1, false, true>(a, s);
    return wide ? launch<4, 2, false>(a, s) : launch<4, 1, false>(a, s);
}

}  // namespace climber
