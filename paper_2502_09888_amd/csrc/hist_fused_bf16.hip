// Fused history pass for gfx950 (CDNA4), bf16: for subsequences of 128 or 256 behaviours the
// per-layer K/V cache write (Climber, arXiv 2502.09888, Sec. 3.2: history K/V are produced once
// and kept for the candidates) and the attention inside each subsequence (Sec. 3.1.2 + Eq. (3),
// one Transformer block per subsequence, per-row temperature) run in ONE kernel.
//
// A workgroup (one wave per 32 queries) handles one (user, head, subsequence) at a time.  The subsequence's key and value
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
// the compute phases: the kernel as a whole is bound by HBM traffic (K, V, Q rows in; cache
// blocks and outputs out), not by the latency of any one phase.
template <int SUB>
__global__ __launch_bounds__(SUB * 2, 256 / SUB) void hist_fused_kernel(const HParams p)
{
    static_assert(SUB == 128 || SUB == 256, "fragments of the whole subsequence stay in LDS");
    constexpr int NB = SUB / 32;   // 32-key blocks per subsequence = waves per workgroup
    constexpr int NT = NB * 64;
    constexpr int kKraw = 0;            // raw K rows of the subsequence being fetched, NB x 4 KiB
    constexpr int kVraw = NB * 4096;    // raw V rows, NB x 4 KiB
    constexpr int kKf = 2 * NB * 4096;  // K fragments of the subsequence being attended to
    constexpr int kVf = 3 * NB * 4096;  // V^T fragments
    constexpr int kOut = 4 * NB * 4096; // per wave 4 KiB: query rows in, output rows out
    constexpr int kLds = 5 * NB * 4096; // SUB = 256: 160 KiB, one workgroup per CU; 128: 80 KiB, two
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLds];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    // a full line), chunk c of row r stored at slot c ^ (r & 7).
    auto issue_kv = [&](const Item &g) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int gi = wave * 4 + i, pos = gi * 64 + lane, r = pos >> 3;
            const int c = (pos & 7) ^ (r & 7);
            const int64_t off = (g.row0 + min(r, g.n_pad - 1)) * p.ld + g.h * kDHead + c * 8;
            __builtin_amdgcn_global_load_lds((glb_u8 *)(p.k + off), (lds_u8 *)lds + kKraw + gi * 1024, 16, 0, 0);
            __builtin_amdgcn_global_load_lds((glb_u8 *)(p.v + off), (lds_u8 *)lds + kVraw + gi * 1024, 16, 0, 0);
        }
    };
    struct Rows {  // what a lane fetches ahead for the wave's 32 query rows
        u32x4 q[4];   // piece i: row (i * 64 + lane) / 8 of the wave, 16-byte chunk lane % 8
        int sc, bh;   // ids of row lane % 32
    };
    auto load_rows = [&](const Item &g, Rows &r) __attribute__((always_inline)) {
        const int last = max(g.n_valid, 1) - 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = i * 64 + lane;
            const int64_t row = g.row0 + min(wave * 32 + (id >> 3), last);
            r.q[i] = *(const u32x4 *)(p.q + row * p.ld + g.h * kDHead + (id & 7) * 8);
        }
        const int64_t row = g.row0 + min(wave * 32 + l32, last);
        r.sc = p.scen[row];
        r.bh = p.beh[row];
    };
    Item g, gn;
    Rows rows, rows_n;
    int item = next_item(blockIdx.x, g);
    if (item >= p.n_items) return;
    load_rows(g, rows);
    issue_kv(g);
    while (true) {
        uint8_t *kf = lds + kKf;
        // ---- 1. this subsequence's rows have landed ------------------------------------------
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const int sc = min(max(rows.sc, 0), p.n_scen - 1);
        const int bhv = min(max(rows.bh, 0), p.n_beh - 1);
        const float tau_row = p.tau[sc * p.n_beh + bhv];
        // the wave's query rows: through its own staging slice into B-operand order
        uint8_t *tr = lds + kOut + wave * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = i * 64 + lane, r = id >> 3, c = id & 7;
            *(u32x4 *)(tr + r * 128 + ((c ^ (r & 7)) * 16)) = rows.q[i];
        }
        __syncthreads();  // every wave's copies are in LDS and every wave is done with the
                          // previous subsequence (its fragments may be overwritten)
        // ---- 2. operand fragments; slots past the valid length become zeros.
        //   K chunk (s, lane)      = K[32kb + lane%32][16s + 8(lane/32) + 0..7]   (16-byte moves)
        //   V^T chunk (g, db, lane), element e =
        //                            V[32kb + 16g + 8(e/4) + 4(lane/32) + e%4][32db + lane%32]
#pragma unroll 1
        for (int j = 0; j < 4; ++j) {
            const int pi = j * NT + tid, kb = pi >> 8;
            {
                const int s4 = (pi >> 6) & 3, r = 32 * kb + l32, c = 2 * s4 + hf;
                uint4 kk = *(const uint4 *)(lds + kKraw + r * 128 + ((c ^ (r & 7)) * 16));
                if (r >= g.n_valid) kk = uint4{0, 0, 0, 0};
                *(uint4 *)(lds + kKf + pi * 16) = kk;
            }
            const int gg = (pi >> 7) & 1, db = (pi >> 6) & 1, d = 32 * db + l32;
            bf16x8 out;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int r = 32 * kb + 16 * gg + 8 * (e >> 2) + 4 * hf + (e & 3);
                const __bf16 x =
                    *(const __bf16 *)(lds + kVraw + r * 128 + (((d >> 3) ^ (r & 7)) * 16) + (d & 7) * 2);
                out[e] = r < g.n_valid ? x : (__bf16)0.f;
            }
            *(bf16x8 *)(lds + kVf + pi * 16) = out;
        }
        bf16x8 q_raw[4];
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4)
            q_raw[s4] = *(const bf16x8 *)(tr + l32 * 128 + (((2 * s4 + hf) ^ (l32 & 7)) * 16));
        __syncthreads();  // fragments complete; the raw rows are no longer needed
        // the temperature has to be in a register before the next rows are requested: a wait for
        // it placed after those requests would wait for them as well (loads return in order)
        const float c_scale = p.scale_log2e / tau_row;
        asm volatile("" ::"v"(c_scale));
        // ---- 3. the next subsequence's rows start their way in ------------------------------
        const int item_n = next_item(item + gridDim.x, gn);
        if (item_n < p.n_items) {
            load_rows(gn, rows_n);
            issue_kv(gn);
        }
        // ---- 4. the cache blocks of this subsequence: block kb is written out by all waves, each
        //         its share, when they reach block kb of the attention loop below, so the stores
        //         trickle out during the computation instead of arriving as one burst (all
        //         workgroups of the chip run these phases at about the same time) -------------
        uint8_t *cache_dst = p.layer_base + ((size_t)g.t0 * p.H + (size_t)g.h * g.Lpad) * (kDHead * 4) +
                             (size_t)(g.k_lo / kBlockKeys) * kBlockBytes;
        const int nb_pad = g.n_pad / kBlockKeys;
        auto store_block = [&](int kb) __attribute__((always_inline)) {
            // 8 KiB = 512 pieces of 16 B: K fragments then V^T fragments
#pragma unroll
            for (int j = 0; j < 512 / NT; ++j) {
                const int pc = j * NT + tid;
                const int off = (pc < 256 ? kKf : kVf - 4096) + kb * 4096 + pc * 16;
                *(u32x4 *)(cache_dst + (size_t)kb * kBlockBytes + pc * 16) = *(const u32x4 *)(lds + off);
            }
        };
        // ---- 5. attention of the subsequence's own queries, 32 per wave ----------------------
        QState<1> st;
        const int n_blk = (g.n_valid + kBlockKeys - 1) / kBlockKeys;
        auto run = [&](auto safe_tag) __attribute__((always_inline)) {
            constexpr bool SAFE = decltype(safe_tag)::value;
            f32x16 S0[1], S1[1];
            bf16x8 P[1][2];
            st.l[0] = 0.f;
            st.m_ref[0] = 0.f;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.O[db][0][r] = 0.f;
            if (n_blk > 0) qk_block(st, load_k(kf, lane), S0);
            auto block = [&](int blk, f32x16 (&Sc)[1], f32x16 (&Sn)[1]) __attribute__((always_inline)) {
                if (blk + 1 < n_blk) qk_block(st, load_k(kf + (blk + 1) * 4096, lane), Sn);
                if (32 * (blk + 1) > g.n_valid) mask_block(Sc, hf, 32 * blk, g.n_valid);
                if (SAFE) softmax_safe(st, Sc, P); else softmax_fast(st, Sc, P);
                VFrags vf;
#pragma unroll
                for (int gg = 0; gg < 2; ++gg)
#pragma unroll
                    for (int db = 0; db < 2; ++db)
                        vf.a[gg][db] = *(const bf16x8 *)(lds + kVf + blk * 4096 + ((gg * 2 + db) * 64 + lane) * 16);
                pv_block(st, vf, P);
                if (!SAFE) store_block(blk);
            };
            for (int blk = 0; blk < n_blk; blk += 2) {
                block(blk, S0, S1);
                if (blk + 1 < n_blk) block(blk + 1, S1, S0);
            }
        };
        st.c[0] = c_scale;
#pragma unroll
        for (int s = 0; s < 4; ++s)  // FAST: q' = bf16(q * c)
#pragma unroll
            for (int e = 0; e < 8; ++e) st.qf[0][s][e] = (__bf16)((float)q_raw[s][e] * st.c[0]);
        run(std::false_type{});
        for (int kb = n_blk; kb < nb_pad; ++kb) store_block(kb);  // blocks of padding only: zeros
        float lt = st.l[0] + xhalf(st.l[0]);
        const bool bad = g.n_valid > 0 && !(lt > kDenomLo && lt < kDenomHi);
        if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // SAFE (rare): unscaled q, running maximum
#pragma unroll
            for (int s = 0; s < 4; ++s) st.qf[0][s] = q_raw[s];
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
        if (item_n >= p.n_items) break;
        item = item_n;
        g = gn;
        rows = rows_n;
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
        hipLaunchKernelGGL(hist_fused_kernel<256>, dim3(grid), dim3(512), 0, s, p);
    } else {                 // 80 KiB: two 4-wave workgroups per CU
        const unsigned grid = (unsigned)std::min<int64_t>(items, 2 * n_cu);
        hipLaunchKernelGGL(hist_fused_kernel<128>, dim3(grid), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}

}  // namespace climber
