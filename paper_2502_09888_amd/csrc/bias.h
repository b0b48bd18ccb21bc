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
    // the saturating difference clips exactly like the true one (half < 2^30): exact for any two int32
    const int d = __builtin_elementwise_sub_sat(pos_q, pos_k);
    return min(max(d, -half), half) + half;
}

// Flipping the sign bit maps int32 onto uint32 in order, so |ts_q - ts_k| = |u(ts_q) - u(ts_k)| as an
// unsigned value, exact for any two int32.  Callers with many keys per query flip each side once.
static __device__ __forceinline__ uint32_t bias_time_key(int ts) { return (uint32_t)ts ^ 0x80000000u; }

static __device__ __forceinline__ int bias_bucket_time_u(uint32_t uq, uint32_t uk, int n_time)
{
    uint32_t a;
    asm("v_sad_u32 %0, %1, %2, 0" : "=v"(a) : "v"(uq), "v"(uk));  // |uq - uk|
    // floor(log2(max(a, 1))) = floor(log2(a | 1)): position of the highest set bit
    const int b = 31 - __builtin_clz(a | 1u);
    return min(b, n_time - 1);
}

static __device__ __forceinline__ int bias_bucket_time(int ts_q, int ts_k, int n_time)
{
    return bias_bucket_time_u(bias_time_key(ts_q), bias_time_key(ts_k), n_time);
}

}  // namespace climber
