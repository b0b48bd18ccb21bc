// Relative attention bias of Climber's attention layer (arXiv 2502.09888, Eq. (3): R = Q K^T + f_b,
// divided by the temperature afterwards).  The paper names the ingredients (relative position and
// relative time, per extraction strategy and scenario) and leaves the form open; the form of this
// library:
//   bias(i, j; h) = P[g_i][h][bp(pos_i - pos_j)] + T[g_i][h][bt(ts_i - ts_j)]
//   g_i   = (scenario, behaviour) of the query row (the pair that selects its temperature)
//   bp(d) = clip(d, -half, half) + half, half = (n_pos - 1) / 2
//   bt(d) = min(floor(log2(max(|d|, 1))), n_time - 1)
// Integer arithmetic only, exact for any pair of int32 values.
#pragma once
#include <stdint.h>

namespace climber {

struct BiasArgs {
    const float *pos_table;   // [n_scen][n_beh][H][n_pos]; nullptr = no bias
    const float *time_table;  // [n_scen][n_beh][H][n_time]
    const int32_t *key_pos, *key_ts;  // per (padded) history row
    const int32_t *q_pos, *q_ts;      // per query row (history rows or candidates)
    int n_pos, n_time;
};

static __device__ __forceinline__ int bias_bucket_pos(int pos_q, int pos_k, int half)
{
    // |difference| as an unsigned value: exact for any two int32
    const uint32_t a = pos_q >= pos_k ? (uint32_t)pos_q - (uint32_t)pos_k : (uint32_t)pos_k - (uint32_t)pos_q;
    const int m = (int)(a < (uint32_t)half ? a : (uint32_t)half);
    return pos_q >= pos_k ? half + m : half - m;
}

static __device__ __forceinline__ int bias_bucket_time(int ts_q, int ts_k, int n_time)
{
    uint32_t a = ts_q >= ts_k ? (uint32_t)ts_q - (uint32_t)ts_k : (uint32_t)ts_k - (uint32_t)ts_q;
    a = a < 1u ? 1u : a;
    const int b = 31 - __builtin_clz(a);
    return b < n_time - 1 ? b : n_time - 1;
}

}  // namespace climber
