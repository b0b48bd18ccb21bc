// fp32 reference-path attention: one wavefront per (query row, head), every softmax row held in
// LDS.  Covers both masks of Climber (arXiv 2502.09888): the "single user, multiple items" mask of
// Sec. 3.2 (a candidate sees the cached history and itself) and the per-subsequence history
// attention of Sec. 3.1.2, with the per-row temperature of Eq. (3).  Any d_head <= 256; meant for
// the small fp32 configuration and as a second opinion, not for throughput.
#include "internal.h"

namespace climber {
namespace {

constexpr int kMaxKeysF32 = 15 * 1024;  // logits of one row live in LDS (60 KiB)

__device__ __forceinline__ float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <bool SUMI>
__global__ __launch_bounds__(64) void attn_f32_kernel(AttnArgs a, int64_t total_rows)
{
    extern __shared__ float logit[];
    const int lane = threadIdx.x;
    const int64_t row = blockIdx.x / a.H;
    const int h = blockIdx.x % a.H, dh = a.d_head;
    const int32_t *off = SUMI ? a.cand_off : a.cache.tok_off;
    int lo_b = 0, hi_b = a.cache.B;  // largest b with off[b] <= row
    while (hi_b - lo_b > 1) {
        const int mid = (lo_b + hi_b) >> 1;
        if (off[mid] <= row) lo_b = mid; else hi_b = mid;
    }
    const int b = lo_b;
    const int t0 = a.cache.tok_off[b], Lb = a.cache.hist_len[b];
    float *o = (float *)a.o + row * a.ld_o + h * dh;
    int lo = 0, hi = Lb;
    if (SUMI) {
        if (row >= off[a.cache.B]) return;
    } else {
        const int i = (int)(row - t0);
        if (i >= Lb) {
            for (int e = lane; e < dh; e += 64) o[e] = 0.f;
            return;
        }
        if (a.sub_len > 0) {
            lo = (i / a.sub_len) * a.sub_len;
            hi = min(lo + a.sub_len, Lb);
        }
        if (a.causal) hi = i + 1;
    }
    const int nh = hi - lo, nk = nh + (SUMI ? 1 : 0);
    const float *kc = (const float *)a.cache.layer_base;
    const float *vc = kc + total_rows * a.H * dh;
    const float *q = (const float *)a.q + row * a.ld_q + h * dh;
    const float *ks = SUMI ? (const float *)a.k_self + row * a.ld_kv + h * dh : nullptr;
    const float *vs = SUMI ? (const float *)a.v_self + row * a.ld_kv + h * dh : nullptr;
    const int sc = min(max(a.scen[row], 0), a.n_scen - 1);
    const int bv = min(max(a.beh[row], 0), a.n_beh - 1);
    const float tau = a.tau[sc * a.n_beh + bv];

    const bool bias_on = a.bias.pos_table != nullptr;
    const int q_pos = bias_on ? a.bias.q_pos[row] : 0, q_ts = bias_on ? a.bias.q_ts[row] : 0;
    const int64_t grp = ((int64_t)sc * a.n_beh + bv) * a.H + h;
    const int64_t prow = grp * a.bias.n_pos, trow = grp * a.bias.n_time;

    float mx = -INFINITY;
    for (int j = lane; j < nk; j += 64) {
        const float *kp = j < nh ? kc + ((int64_t)(t0 + lo + j) * a.H + h) * dh : ks;
        float dot = 0.f;
        for (int e = 0; e < dh; ++e) dot = fmaf(q[e], kp[e], dot);
        float s = a.qk_scale * dot;
        if (bias_on) {  // Eq. (3): the bias joins the logit before the temperature divide
            const int kp_ = j < nh ? a.bias.key_pos[t0 + lo + j] : q_pos;
            const int kt_ = j < nh ? a.bias.key_ts[t0 + lo + j] : q_ts;
            s += a.bias.pos_table[prow + bias_bucket_pos(q_pos, kp_, (a.bias.n_pos - 1) >> 1)] +
                 a.bias.time_table[trow + bias_bucket_time(q_ts, kt_, a.bias.n_time)];
        }
        s /= tau;
        logit[j] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = lane; j < nk; j += 64) {
        const float pv = expf(logit[j] - mx);
        logit[j] = pv;
        sum += pv;
    }
    sum = wave_sum(sum);
    __syncthreads();
    for (int e = lane; e < dh; e += 64) {
        float acc = 0.f;
        for (int j = 0; j < nh; ++j)
            acc = fmaf(logit[j], vc[((int64_t)(t0 + lo + j) * a.H + h) * dh + e], acc);
        if (SUMI) acc = fmaf(logit[nh], vs[e], acc);
        o[e] = acc / sum;
    }
}

}  // namespace

size_t attn_f32_max_keys() { return kMaxKeysF32; }

hipError_t launch_attn_f32(const AttnArgs &a, bool sumi, int64_t cache_rows, hipStream_t s)
{
    // cache_rows: padded history rows of the cache (V follows K after cache_rows*H*dh floats)
    const int64_t grid = a.total_q_rows * a.H;
    if (grid == 0) return hipSuccess;
    if (grid > 0x7fffffff || a.max_hist_len > kMaxKeysF32) return hipErrorInvalidValue;
    const size_t shmem = (size_t)(a.max_hist_len + 1) * sizeof(float);
    if (sumi)
        hipLaunchKernelGGL(attn_f32_kernel<true>, dim3((unsigned)grid), dim3(64), shmem, s, a, cache_rows);
    else
        hipLaunchKernelGGL(attn_f32_kernel<false>, dim3((unsigned)grid), dim3(64), shmem, s, a, cache_rows);
    return hipGetLastError();
}

}  // namespace climber
