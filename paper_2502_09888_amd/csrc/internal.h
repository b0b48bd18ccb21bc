// Internal declarations shared by the translation units of libclimber.so.
// Host-side launch wrappers; every kernel lives in exactly one .hip file.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bias.h"

namespace climber {

// ---- bf16 KV-cache geometry (d_head = 64) ---------------------------------------------------
// A (user, head) owns L_pad/32 consecutive 8 KiB blocks.  Block kb holds keys 32kb .. 32kb+31:
//   bytes [0, 4096)    K as A-operand fragments of v_mfma_f32_32x32x16_bf16 for S^T = K Q^T:
//                      chunk (s, lane), 16 B: K[32kb + lane%32][16s + 8(lane/32) + 0..7]
//   bytes [4096, 8192) V^T as A-operand fragments for O^T = V^T P^T, with the key order inside a
//                      16-key group permuted to the order the S^T accumulator delivers P:
//                      chunk (g, db, lane), element e:
//                      V[32kb + 16g + 8(e/4) + 4(lane/32) + e%4][32db + lane%32]
// so that a wave reads every fragment as one conflict-free 16-byte-per-lane LDS access and the
// HBM -> LDS copy of a tile is linear.
constexpr int kDHead = 64;
constexpr int kBlockKeys = 32;
constexpr int kBlockBytes = 8192;

struct CacheView {          // device-side view of one cache
    const int32_t *hist_len; // [B]
    const int32_t *tok_off;  // [B+1] padded row offsets
    const int32_t *order;    // [B] users by decreasing history length
    const int32_t *seg;      // bf16: [rows/64] user of every group of 64 padded rows
    uint8_t *layer_base;     // payload of the selected layer
    int B;
};

struct AttnArgs {
    CacheView cache;
    const void *q, *k_self, *v_self; // query rows; candidates' own k/v (SUMI) -- element type of path
    int64_t ld_q, ld_kv;             // row strides in elements
    const int32_t *scen, *beh;       // per query row
    const float *tau;                // [n_scen][n_beh]
    const int32_t *cand_off;         // SUMI: [B+1]
    void *o;
    int64_t ld_o;
    int H, d_head, n_scen, n_beh, sub_len, causal;
    int max_rows_per_user;           // SUMI: m_max; history: longest padded history
    int64_t total_q_rows;            // SUMI: m_total; history: padded rows of the batch
    int max_hist_len;                // longest valid history of the batch
    int uni_len, uni_pad;            // >= 0: all users share this valid / padded history length
    int uni_cand;                    // >= 0: all users have this many candidates (SUMI)
    float qk_scale;
    BiasArgs bias;                   // relative attention bias; bias.pos_table == nullptr: none
};

// bf16 MFMA flash attention (attn_bf16.hip)
hipError_t launch_attn_sumi_bf16(const AttnArgs &a, hipStream_t s);
hipError_t launch_attn_hist_bf16(const AttnArgs &a, hipStream_t s);
// fused cache write + attention inside short subsequences (hist_fused_bf16.hip): a.k_self / a.v_self
// are the history key / value rows (same row stride as the queries)
bool hist_fused_supported(int sub_len, int causal);
hipError_t launch_hist_fused_bf16(const AttnArgs &a, hipStream_t s);
// fp32 reference-path attention (attn_f32.hip); the cache layer holds plain [rows][H][dh] K then V
hipError_t launch_attn_f32(const AttnArgs &a, bool sumi, int64_t cache_rows, hipStream_t s);
size_t attn_f32_max_keys();

// cache writers (kv_cache.hip): k, v are [rows][ld] with head h at column h*d_head
hipError_t launch_kv_write_bf16(const CacheView &c, const void *k, const void *v, int64_t ld, int H,
                                int max_padded_len, hipStream_t s);
hipError_t launch_kv_write_f32(const CacheView &c, const void *k, const void *v, int64_t ld, int H,
                               int d_head, int64_t total_rows, hipStream_t s);

// device-side id / offset / temperature check (check.hip); hist_len / tok_off non-null: history rows
hipError_t launch_check_inputs(const float *tau, const int32_t *scen, const int32_t *beh, int64_t n_rows,
                               const int32_t *hist_len, const int32_t *tok_off, const int32_t *cand_off,
                               int B, int n_scen, int n_beh, int m_max, int32_t *status, hipStream_t s);

}  // namespace climber
