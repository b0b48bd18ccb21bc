// Fused history pass for gfx950 (CDNA4), bf16: for subsequences of 128 or 256 behaviours the
// per-layer K/V cache write (Climber, arXiv 2502.09888, Sec. 3.2: history K/V are produced once
// and kept for the candidates) and the attention inside each subsequence (Sec. 3.1.2 + Eq. (3),
// one Transformer block per subsequence, per-row temperature) run in ONE kernel.
//
// A workgroup (one wave per 32 queries) handles one (user, head, subsequence) at a time.  The
// subsequence's key and value rows are read from HBM exactly once, HBM -> LDS directly, as whole
// 128-byte rows (16-byte chunks XOR-swizzled by the row number), and are never rearranged:
//   - a K operand fragment is a set of 16-byte row pieces: the attention reads it out of the raw
//     rows with the right address per lane;
//   - a V^T operand fragment (d along the lanes, keys along the registers) is read out of the raw
//     rows by the LDS transpose read (ds_read_b64_tr_b16): every lane names 8 bytes of a row, and
//     within each group of 16 lanes the 4 x 4 blocks of 2-byte elements are exchanged so that a
//     lane receives 4 consecutive keys of one d;
//   - every wave reads every block's fragments for its own queries anyway; wave w also writes
//     block w of the subsequence (4 K fragments, 4 V^T chunks) to the cache from those registers,
//     so the cache image costs no LDS traffic of its own and is never read back.
// Rows of the next subsequence travel into the other half of the buffers while this one is
// attended to: no rearrangement phase, one barrier per subsequence.
// Slots past a user's valid length hold zeros in the cache and are masked in the softmax whatever
// the source rows contain (the raw rows are zeroed in LDS after landing); padded query rows
// produce zeros.
// The softmax is the exact-scale FAST form of attn_bf16.hip (query as given, logits multiplied by the
// row scale in fp32, no reference subtraction: this pass is bound by memory, so the multiplication is
// free and the 2^-9 per logit of the folded form is saved) with the window [kDenomLoExact,
// kDenomHiExact] on the denominators; a wave whose rows leave the window redoes its subsequence
// with the SAFE online softmax -- per wave, since waves share only read-only data.
#include "attn_common.h"

#include <algorithm>
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
    int B, H, n_scen, n_beh, n_sub, n_items;
    int uni_len, uni_pad;  // >= 0: every user has this valid / padded history length
    float scale_log2e;
};

// One (user, head, subsequence): where its rows are and how many of them count.
struct Item {
    int h, t0, Lpad, k_lo;
    int n_pad;    // rows of the subsequence that exist in the padded buffers (multiple of 64)
    int n_valid;  // valid keys = valid queries
    int64_t row0;
};

// Persistent workgroups (SUB/32 waves, one wave per 32 queries) walk over the subsequences
// blockIdx.x, blockIdx.x + gridDim.x, ...  While a subsequence is attended to, the rows of the
// next one are already on their way into the second set of buffers, so HBM stays busy through
// the compute phases and no wave ever waits for rows.
// CAUSAL (token i sees the keys j <= i of its subsequence): wave w's 32 queries stop after key block w,
// whose logits are masked per lane; the wave still reads and stores what it is responsible for (block w
// of the cache image), which its own blocks 0 .. w cover.
template <int SUB, bool CAUSAL = false>
__global__ __launch_bounds__(SUB * 2, 256 / SUB) void hist_fused_kernel(const HParams p)
{
    static_assert(SUB == 128 || SUB == 256, "fragments of the whole subsequence stay in LDS");
    constexpr int NB = SUB / 32;   // 32-key blocks per subsequence = waves per workgroup
    constexpr int kBuf = NB * 4096;     // K (or V) rows of one subsequence, 128 B each
    constexpr int kKraw = 0;            // two buffers of K rows: one attended to, one being fetched
    constexpr int kVraw = 2 * kBuf;     // two buffers of V rows
    constexpr int kOut = 4 * kBuf;      // per wave 4 KiB: query rows in, output rows out
    constexpr int kLds = 5 * NB * 4096; // SUB = 256: 160 KiB, one workgroup per CU; 128: 80 KiB, two
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLds];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar
    const int l32 = lane & 31, hf = lane >> 5;

    auto geometry = [&](int item, Item &g) __attribute__((always_inline)) -> bool {
        const int si = item % p.n_sub, bh = item / p.n_sub;
        const int b = bh / p.H;
        int Lb;
        g.h = bh % p.H;
        if (p.uni_len >= 0) {
            Lb = p.uni_len;
            g.Lpad = p.uni_pad;
            g.t0 = b * g.Lpad;
        } else {
            Lb = p.hist_len[b];
            g.t0 = p.tok_off[b];
            g.Lpad = p.tok_off[b + 1] - g.t0;
        }
        g.k_lo = si * SUB;
        g.n_pad = min(SUB, g.Lpad - g.k_lo);
        g.n_valid = max(0, min(g.n_pad, Lb - g.k_lo));
        g.row0 = (int64_t)g.t0 + g.k_lo;
        return g.k_lo < g.Lpad;
    };
    // first subsequence at or after `item` (stride gridDim.x) that exists
    auto next_item = [&](int item, Item &g) __attribute__((always_inline)) -> int {
        while (item < p.n_items && !geometry(item, g)) item += gridDim.x;
        return item;
    };
    // K and V rows travel HBM -> LDS as whole 128-byte rows (8 lanes per row, so every request is
    // a full line), chunk c of row r stored at slot c ^ swz(r).  With swz(r) = (r / 2) % 8 both the K
    // fragment reads (16 consecutive rows, one chunk) and the transpose reads of V (8 rows, 64 bytes
    // each) spread over all banks.  Wave w fetches rows 32w .. 32w + 31.
    auto swz = [](int r) __attribute__((always_inline)) { return (r >> 1) & 7; };
    auto issue_kv_piece = [&](const Item &g, int buf, int i) __attribute__((always_inline)) {
        const int gi = wave * 4 + i, pos = gi * 64 + lane, r = pos >> 3;
        const int c = (pos & 7) ^ swz(r);
        const int64_t off = (g.row0 + min(r, g.n_pad - 1)) * p.ld + g.h * kDHead + c * 8;
        // read once: non-temporal (aux bit 1), so that the rows do not displace the cache blocks being
        // written, which the candidate pass reads next, from L2
        __builtin_amdgcn_global_load_lds((glb_u8 *)(p.k + off), (lds_u8 *)lds + kKraw + buf * kBuf + gi * 1024, 16, 0, 2);
        __builtin_amdgcn_global_load_lds((glb_u8 *)(p.v + off), (lds_u8 *)lds + kVraw + buf * kBuf + gi * 1024, 16, 0, 2);
    };
    auto issue_kv = [&](const Item &g, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) issue_kv_piece(g, buf, i);
    };
    // fragments of 32-key block blk out of the raw rows
    // (Both kinds of fragment reads are written as inline assembly: the compiler cannot tell the rows
    // being read from the rows a copy in flight is writing -- the other buffer half -- and would wait
    // for all copies (vmcnt(0)) before every read, i.e. undo the prefetch.  Its own count of LDS
    // operations in flight does not include these reads, which only makes its waits stricter (LDS
    // operations return in order); the results are valid after the explicit wait.)
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    struct KRaw { u32x4 x[4]; };
    struct VRaw { s16x4 h[2][2][2]; };
    auto read_k = [&](const uint8_t *kraw, int blk, KRaw &k) __attribute__((always_inline)) {
        const int r = 32 * blk + l32;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            const uint32_t src = (uint32_t)(uintptr_t)(lds_u8 *)(kraw + r * 128 + (((2 * s4 + hf) ^ swz(r)) * 16));
            asm volatile("ds_read_b128 %0, %1" : "=v"(k.x[s4]) : "v"(src));
        }
    };
    // the K reads have returned although up to BEHIND later LDS reads are still in flight
    auto done_k = [&](KRaw &k, auto behind_tag) __attribute__((always_inline)) {
        constexpr int BEHIND = decltype(behind_tag)::value;
        static_assert(BEHIND == 0 || BEHIND == 8, "");
        if (BEHIND == 8)
            asm volatile("s_waitcnt lgkmcnt(8)" : "+v"(k.x[0]), "+v"(k.x[1]), "+v"(k.x[2]), "+v"(k.x[3]));
        else
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(k.x[0]), "+v"(k.x[1]), "+v"(k.x[2]), "+v"(k.x[3]));
        KFrags f;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) f.a[s4] = __builtin_bit_cast(bf16x8, k.x[s4]);
        return f;
    };
    // V^T chunk (gg, db), element e = V[32 blk + 16 gg + 8 (e / 4) + 4 (lane / 32) + e % 4][32 db + lane % 32]:
    // two transpose reads (e / 4 = 0, 1).  In a group of 16 lanes, lane i receives as element j the
    // element i % 4 of the 8 bytes named by lane i / 4 + 4 j of the group; so lane 4 j + a of group G
    // names row .. + j, columns 32 db + 16 (G % 2) + 4 a .. + 3, and lane i ends up with column
    // 32 db + 16 (G % 2) + i = 32 db + lane % 32 of the rows .. + 0 .. 3.
    // With swz(r) = (r / 2) % 8 the address of read (gg, db, hh) of block blk is
    //   32 blk * 128 + gg * 2048 + hh * 1024 + (db ^ hh) * 64 + (a term of the lane alone):
    // the swizzle of row .. + 8 hh + 4 (G / 2) + i16 / 4 is 4 hh + 2 (G / 2) + i16 / 8, the chunk is
    // 4 db + 2 (G % 2) + (i16 / 2) % 2, and the exclusive or of the two splits into 4 (db ^ hh) and a
    // lane term.  So the eight reads of a block are one address register and eight immediates (the
    // compiler, given the expression, recomputes every address with ~20 vector instructions per block).
    const uint32_t v_lane = [&] {
        const int G = lane >> 4, i16 = lane & 15;
        const int x = 2 * (G & 1) + ((i16 >> 1) & 1), y = 2 * (G >> 1) + (i16 >> 3);
        return (uint32_t)((4 * (G >> 1) + (i16 >> 2)) * 128 + (x ^ y) * 16 + 8 * (i16 & 1));
    }();
    auto read_v = [&](const uint8_t *vraw, int blk, VRaw &v) __attribute__((always_inline)) {
        const uint32_t src = (uint32_t)(uintptr_t)(lds_u8 *)vraw + v_lane + blk * 4096;
        auto one = [](s16x4 &dst, uint32_t a, auto imm_tag) __attribute__((always_inline)) {
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(a), "n"(decltype(imm_tag)::value));
        };
#define CLIMBER_V_READ(gg, db, hh) \
        one(v.h[gg][db][hh], src, std::integral_constant<int, (gg) * 2048 + (hh) * 1024 + ((db) ^ (hh)) * 64>{})
        CLIMBER_V_READ(0, 0, 0); CLIMBER_V_READ(0, 0, 1); CLIMBER_V_READ(0, 1, 0); CLIMBER_V_READ(0, 1, 1);
        CLIMBER_V_READ(1, 0, 0); CLIMBER_V_READ(1, 0, 1); CLIMBER_V_READ(1, 1, 0); CLIMBER_V_READ(1, 1, 1);
#undef CLIMBER_V_READ
    };
    // the V reads have returned, although the four K reads requested after them (if k_behind) may
    // still be in flight.  (One statement carries the registers whatever the case: a result that
    // came out of two alternative statements would be copied at their join.)
    auto done_v = [&](VRaw &v, bool k_behind) __attribute__((always_inline)) {
        if (!k_behind) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        asm volatile("s_waitcnt lgkmcnt(4)"
                     : "+v"(v.h[0][0][0]), "+v"(v.h[0][0][1]), "+v"(v.h[0][1][0]), "+v"(v.h[0][1][1]),
                       "+v"(v.h[1][0][0]), "+v"(v.h[1][0][1]), "+v"(v.h[1][1][0]), "+v"(v.h[1][1][1]));
        VFrags f;
#pragma unroll
        for (int gg = 0; gg < 2; ++gg)
#pragma unroll
            for (int db = 0; db < 2; ++db) {
                const s16x8 both = __builtin_shufflevector(v.h[gg][db][0], v.h[gg][db][1], 0, 1, 2, 3, 4, 5, 6, 7);
                f.a[gg][db] = __builtin_bit_cast(bf16x8, both);
            }
        return f;
    };
    struct Rows {  // what a lane fetches ahead for the wave's 32 query rows
        u32x4 q[4];   // piece i: row (i * 64 + lane) / 8 of the wave, 16-byte chunk lane % 8
        int sc, bh;   // ids of row lane % 32
    };
    auto load_q_piece = [&](const Item &g, Rows &r, auto i_tag) __attribute__((always_inline)) {
        constexpr int i = decltype(i_tag)::value;
        const int id = i * 64 + lane;
        const int64_t row = g.row0 + min(wave * 32 + (id >> 3), max(g.n_valid, 1) - 1);
        r.q[i] = *(const u32x4 *)(p.q + row * p.ld + g.h * kDHead + (id & 7) * 8);
    };
    auto load_ids = [&](const Item &g, Rows &r) __attribute__((always_inline)) {
        const int64_t row = g.row0 + min(wave * 32 + l32, max(g.n_valid, 1) - 1);
        r.sc = p.scen[row];
        r.bh = p.beh[row];
    };
    auto load_rows = [&](const Item &g, Rows &r) __attribute__((always_inline)) {
        load_q_piece(g, r, std::integral_constant<int, 0>{});
        load_q_piece(g, r, std::integral_constant<int, 1>{});
        load_q_piece(g, r, std::integral_constant<int, 2>{});
        load_q_piece(g, r, std::integral_constant<int, 3>{});
        load_ids(g, r);
    };
    // the temperature table in a register (entry lane % 64), if it has no more than 64 entries: the
    // per-row lookup is then a cross-lane read instead of a trip to memory at the top of every
    // subsequence
    const int n_tau = p.n_scen * p.n_beh;
    const float tau_reg = n_tau <= 64 ? p.tau[min(lane, n_tau - 1)] : 0.f;
    Item g, gn;
    Rows rows, rows_n;
    int item = next_item(blockIdx.x, g);
    if (item >= p.n_items) return;
    load_rows(g, rows);
    issue_kv(g, 0);
    // The body exists twice, once per buffer half, so that every LDS offset is a compile-time
    // constant: the compiler can then see that the rows being read and the rows a copy in flight is
    // writing are different memory, and does not wait for the copies before each LDS read.
    auto subsequence = [&](auto buf_tag) __attribute__((always_inline)) -> bool {
        constexpr int buf = decltype(buf_tag)::value;
        const uint8_t *kraw = lds + kKraw + buf * kBuf, *vraw = lds + kVraw + buf * kBuf;
        // ---- 1. this subsequence's rows have landed ------------------------------------------
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const int sc = min(max(rows.sc, 0), p.n_scen - 1);
        const int bhv = min(max(rows.bh, 0), p.n_beh - 1);
        const float tau_row = n_tau <= 64 ? __shfl(tau_reg, sc * p.n_beh + bhv, 64) : p.tau[sc * p.n_beh + bhv];
        // rows past the valid length become zeros (each wave in the rows it fetched itself)
        if (g.n_valid < SUB) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int gi = wave * 4 + i, pos = gi * 64 + lane, r = pos >> 3;
                if (r >= g.n_valid) {
                    *(u32x4 *)(lds + kKraw + buf * kBuf + pos * 16) = u32x4{0, 0, 0, 0};
                    *(u32x4 *)(lds + kVraw + buf * kBuf + pos * 16) = u32x4{0, 0, 0, 0};
                }
            }
        }
        // the wave's query rows: through its own staging slice into B-operand order
        uint8_t *tr = lds + kOut + wave * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = i * 64 + lane, r = id >> 3, c = id & 7;
            *(u32x4 *)(tr + r * 128 + ((c ^ (r & 7)) * 16)) = rows.q[i];
        }
        auto read_q = [&](bf16x8 (&q_raw)[4]) __attribute__((always_inline)) {
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4)
                q_raw[s4] = *(const bf16x8 *)(tr + l32 * 128 + (((2 * s4 + hf) ^ (l32 & 7)) * 16));
        };
        // the temperature has to be in a register before the next rows are requested: a wait for
        // it placed after those requests would wait for them as well (loads return in order)
        const float c_scale = p.scale_log2e / tau_row;
        asm volatile("" ::"v"(c_scale));
        __syncthreads();  // every wave's rows are in LDS, and every wave is done with the previous
                          // subsequence: the other buffers may be refilled
        // ---- 2. the next subsequence's rows start their way in ------------------------------
        //         piece by piece from inside the attention loop below (a wave that queues all its
        //         requests at once waits in front of its own MFMAs while the memory pipe takes them)
        //         The loads into registers (query rows, ids) are not made conditional on there being a
        //         next subsequence: a conditional load ends in a copy of its result at the join, and
        //         that copy would wait for the load -- and, completion being in order, for every copy
        //         issued before it.  After the last subsequence they fetch its own rows once more.
        const int item_n = next_item(item + gridDim.x, gn);
        const bool more = item_n < p.n_items;
        if (!more) gn = g;
        load_ids(gn, rows_n);
        auto prefetch_piece = [&](auto i_tag) __attribute__((always_inline)) {
            if (more) issue_kv_piece(gn, buf ^ 1, decltype(i_tag)::value);
            load_q_piece(gn, rows_n, i_tag);
        };
        // ---- 3. the cache blocks of this subsequence: 8 pieces of 1 KiB per block (K fragments
        //         s = 0 .. 3, then V^T chunks (gg, db)); every wave holds every block's fragments in
        //         registers at some point, and wave w writes block w from them (a choice by the
        //         block, not by the piece: no register has to be selected by the wave number) ----
        uint8_t *cache_dst = p.layer_base + ((size_t)g.t0 * p.H + (size_t)g.h * g.Lpad) * (kDHead * 4) +
                             (size_t)(g.k_lo / kBlockKeys) * kBlockBytes;
        const int nb_pad = g.n_pad / kBlockKeys;
        const int wv = __builtin_amdgcn_readfirstlane(wave);
        auto put = [&](int kb, int piece, const bf16x8 &x) __attribute__((always_inline)) {
            *(u32x4 *)(cache_dst + (size_t)kb * kBlockBytes + (piece * 64 + lane) * 16) = __builtin_bit_cast(u32x4, x);
        };
        auto store_k = [&](int kb, const KFrags &f) __attribute__((always_inline)) {
            if (kb == wv) {
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) put(kb, s4, f.a[s4]);
            }
        };
        auto store_v = [&](int kb, const VFrags &f) __attribute__((always_inline)) {
            if (kb == wv) {
#pragma unroll
                for (int gg = 0; gg < 2; ++gg)
#pragma unroll
                    for (int db = 0; db < 2; ++db) put(kb, 4 + gg * 2 + db, f.a[gg][db]);
            }
        };
        // ---- 5. attention of the subsequence's own queries, 32 per wave ----------------------
        QState<1> st;
        const int n_blk = (g.n_valid + kBlockKeys - 1) / kBlockKeys;
        const int n_att = CAUSAL ? min(n_blk, wv + 1) : n_blk;  // key blocks this wave's queries attend to
        auto run = [&](auto safe_tag) __attribute__((always_inline)) {
            constexpr bool SAFE = decltype(safe_tag)::value;
            f32x16 S0[1], S1[1];
            bf16x8 P[1][2];
            st.l[0] = 0.f;
            st.m_ref[0] = kSafeNoRef;  // SAFE: the first block's maximum becomes the reference
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.O[db][0][r] = 0.f;
            // K fragments are requested two blocks ahead, V^T fragments at the top of their block: when
            // a block starts, the next block's K has had a whole block's time to arrive, its logits (MFMA)
            // and this block's exponentials (vector unit) then run while the V^T reads are on their way.
            // The K registers are requested again as soon as the MFMAs that read them have been issued.
            KRaw kr;
            if (n_att > 0) {
                read_k(kraw, 0, kr);
                const KFrags k0 = done_k(kr, std::integral_constant<int, 0>{});
                qk_block(st, k0, S0);
                if (!SAFE) store_k(0, k0);
                if (n_att > 1) read_k(kraw, 1, kr);
            }
            auto block = [&](int blk, f32x16 (&Sc)[1], f32x16 (&Sn)[1]) __attribute__((always_inline)) {
                VRaw vr;
                const bool next = blk + 1 < n_att, next2 = blk + 2 < n_att;
                read_v(vraw, blk, vr);
                if (next) {
                    const KFrags kn = done_k(kr, std::integral_constant<int, 8>{});
                    qk_block(st, kn, Sn);
                    if (!SAFE) store_k(blk + 1, kn);
                    if (next2) read_k(kraw, blk + 2, kr);
                }
                if (32 * (blk + 1) > g.n_valid) mask_block(Sc, hf, 32 * blk, g.n_valid);
                if (CAUSAL && blk == wv) {  // the diagonal block: the lane's query is row 32 wv + l32
                    const int lim[1] = {32 * wv + l32 + 1};
                    mask_causal(Sc, hf, 32 * blk, lim);
                }
                if (SAFE) softmax_safe(st, Sc, P);
                else st.l[0] += exp_pack<true>(Sc[0], st.c[0], 0.f, P[0]);  // exact scale: p = exp2(s * c)
                const VFrags vf = done_v(vr, next2);
                pv_block(st, vf, P);
                if (!SAFE) store_v(blk, vf);
            };
            // two halves with half of the next subsequence's requests ahead of each (a wave that queues
            // all its requests at once waits in front of its own MFMAs while the memory pipe takes them)
            if (!SAFE) {
                prefetch_piece(std::integral_constant<int, 0>{});
                prefetch_piece(std::integral_constant<int, 1>{});
                if (NB == 4) {
                    prefetch_piece(std::integral_constant<int, 2>{});
                    prefetch_piece(std::integral_constant<int, 3>{});
                }
            }
            constexpr int kHalf = NB == 8 ? NB / 4 : NB / 2;
#pragma unroll 1
            for (int b2 = 0; b2 < kHalf; ++b2) {
                if (2 * b2 < n_att) block(2 * b2, S0, S1);
                if (2 * b2 + 1 < n_att) block(2 * b2 + 1, S1, S0);
            }
            if (NB == 8) {
                if (!SAFE) {
                    prefetch_piece(std::integral_constant<int, 2>{});
                    prefetch_piece(std::integral_constant<int, 3>{});
                }
#pragma unroll 1
                for (int b2 = kHalf; b2 < NB / 2; ++b2) {
                    if (2 * b2 < n_att) block(2 * b2, S0, S1);
                    if (2 * b2 + 1 < n_att) block(2 * b2 + 1, S1, S0);
                }
            }
        };
        st.c[0] = c_scale;
        {
            bf16x8 q_raw[4];
            read_q(q_raw);
#pragma unroll
            for (int s = 0; s < 4; ++s)  // q as given: the row scale multiplies the logits in fp32
#pragma unroll
                for (int e = 0; e < 8; ++e) st.qf[0][s][e] = q_raw[s][e];
        }
        run(std::false_type{});
        for (int kb = n_blk; kb < nb_pad; ++kb) {  // blocks of padding only: zeros
            const bf16x8 zero = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
            if (NB == 8) put(kb, wv, zero);
            else { put(kb, wv, zero); put(kb, wv + 4, zero); }
        }
        float lt = st.l[0] + xhalf(st.l[0]);
        const bool bad = g.n_valid > 0 && !(lt > kDenomLoExact && lt < kDenomHiExact);
        if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // SAFE (rare): unscaled q, running maximum
            read_q(st.qf[0]);  // the staging slice still holds the wave's query rows
            run(std::true_type{});
            lt = st.l[0] + xhalf(st.l[0]);
        }
        // ---- 6. normalise, turn the 32 x 64 block around in the wave's own 4 KiB of staging,
        //         store whole 128-byte rows; padded query rows that exist get zeros ------------
        {
            const float inv = 1.f / lt;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    bf16x4 ov;
#pragma unroll
                    for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(st.O[db][0][4 * gg + e] * inv);
                    *(bf16x4 *)(tr + l32 * 128 + (((4 * db + gg) ^ (l32 & 7)) * 16) + 8 * hf) = ov;
                }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int id = i * 64 + lane, r = id >> 3, cc = id & 7;
                const int wq = wave * 32 + r;
                const u32x4 val = *(const u32x4 *)(tr + r * 128 + ((cc ^ (r & 7)) * 16));
                __bf16 *op = p.o + (g.row0 + wq) * p.ld_o + g.h * kDHead + cc * 8;
                if (wq < g.n_valid) {
                    __builtin_nontemporal_store(val, (u32x4 *)op);
                } else if (wq < g.n_pad) {
                    *(u32x4 *)op = u32x4{0, 0, 0, 0};
                }
            }
        }
        if (item_n >= p.n_items) return false;
        item = item_n;
        g = gn;
        rows = rows_n;
        return true;
    };
    while (subsequence(std::integral_constant<int, 0>{}) && subsequence(std::integral_constant<int, 1>{})) {
    }
}

}  // namespace

bool hist_fused_supported(int sub_len, int causal) { (void)causal; return sub_len == 128 || sub_len == 256; }

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
    const int64_t items = (int64_t)p.n_sub * p.B * p.H;
    if (items <= 0) return hipSuccess;
    if (items > 0x7fffffff || a.ld_q != a.ld_kv) return hipErrorInvalidValue;
    p.n_items = (int)items;
    static const int n_cu = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        return n;
    }();
    if (a.sub_len == 256) {  // 160 KiB of LDS: one 8-wave workgroup per CU
        const unsigned grid = (unsigned)std::min<int64_t>(items, n_cu);
        if (a.causal) hipLaunchKernelGGL((hist_fused_kernel<256, true>), dim3(grid), dim3(512), 0, s, p);
        else hipLaunchKernelGGL((hist_fused_kernel<256, false>), dim3(grid), dim3(512), 0, s, p);
    } else {                 // 80 KiB: two 4-wave workgroups per CU
        const unsigned grid = (unsigned)std::min<int64_t>(items, 2 * n_cu);
        if (a.causal) hipLaunchKernelGGL((hist_fused_kernel<128, true>), dim3(grid), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((hist_fused_kernel<128, false>), dim3(grid), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}

}  // namespace climber
