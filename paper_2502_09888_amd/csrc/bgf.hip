// Bit-wise gating fusion of Climber (arXiv 2502.09888, Sec. 3.1.4, Eq. (4)): the two small kernels
// around the projections of the fusion layer.
//   fusion attention: G = ATL(E): every one of a candidate's N_b block outputs attends to all N_b of
//     them, no relative attention bias, temperature from the candidate's scenario only;
//   gate + head: Y = G (.) sigmoid(f_gate(G)), score = <w_head, vec(Y)> + b.
// N_b is a handful (the number of extraction strategies), so the attention is N_b x N_b logits per
// (candidate, head): one wavefront per (candidate, head), a lane per feature of the head (d_head = 64).
#include "bgf.h"

namespace climber {
namespace {

__device__ __forceinline__ float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

constexpr int kMaxBlocks = 16;

// qkv: bf16 [m * nb][3 * d] (queries | keys | values, head h at column h * 64); o: bf16 [m * nb][d]
__global__ __launch_bounds__(256) void bgf_attention_kernel(const __bf16 *qkv, __bf16 *o, const int32_t *scen,
                                                            const float *tau_scen, int n_scen, int64_t m, int nb,
                                                            int H, float scale_log2e)
{
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (candidate, head)
    if (item >= m * H) return;
    const int64_t c = item / H;
    const int h = (int)(item % H), d = H * 64;
    const int sc = min(max(scen[c], 0), n_scen - 1);
    const float cs = scale_log2e / tau_scen[sc];
    const __bf16 *base = qkv + c * nb * 3 * (int64_t)d + h * 64 + lane;
    float kj[kMaxBlocks], vj[kMaxBlocks];
    for (int j = 0; j < nb; ++j) {
        kj[j] = (float)base[(int64_t)j * 3 * d + d];
        vj[j] = (float)base[(int64_t)j * 3 * d + 2 * d];
    }
    for (int i = 0; i < nb; ++i) {
        const float qi = (float)base[(int64_t)i * 3 * d];
        float t[kMaxBlocks], mx = -INFINITY;
        for (int j = 0; j < nb; ++j) {
            t[j] = wave_sum(qi * kj[j]) * cs;  // log2 units
            mx = fmaxf(mx, t[j]);
        }
        float sum = 0.f, acc = 0.f;
        for (int j = 0; j < nb; ++j) {
            const float pj = exp2f(t[j] - mx);
            sum += pj;
            acc = fmaf(pj, vj[j], acc);
        }
        o[(c * nb + i) * (int64_t)d + h * 64 + lane] = (__bf16)(acc / sum);
    }
}

// g: fp32 [m][nd] (the fusion layer's output), pre: bf16 [m][nd] (f_gate(G) before the sigmoid);
// y (nullable): fp32 [m][nd]; score: [m].  One wavefront per candidate.
__global__ __launch_bounds__(256) void bgf_gate_head_kernel(const float *g, const __bf16 *pre, const float *w_head,
                                                            float b_head, float *y, float *score, int64_t m, int nd)
{
    const int lane = threadIdx.x & 63;
    const int64_t c = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= m) return;
    float acc = 0.f;
    for (int e = lane; e < nd; e += 64) {
        const float gate = 1.f / (1.f + __expf(-(float)pre[c * nd + e]));
        const float yv = g[c * nd + e] * gate;
        if (y) y[c * nd + e] = yv;
        acc = fmaf(yv, w_head[e], acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) score[c] = acc + b_head;
}

}  // namespace

hipError_t launch_bgf_attention(const void *qkv, void *o, const int32_t *scen, const float *tau_scen, int n_scen,
                                int64_t m, int nb, int H, float qk_scale, hipStream_t s)
{
    if (m <= 0) return hipSuccess;
    if (nb < 1 || nb > kMaxBlocks) return hipErrorInvalidValue;
    const int64_t items = m * H;
    hipLaunchKernelGGL(bgf_attention_kernel, dim3((unsigned)((items + 3) / 4)), dim3(256), 0, s, (const __bf16 *)qkv,
                       (__bf16 *)o, scen, tau_scen, n_scen, m, nb, H, qk_scale * 1.4426950408889634f);
    return hipGetLastError();
}

hipError_t launch_bgf_gate_head(const float *g, const void *pre, const float *w_head, float b_head, float *y,
                                float *score, int64_t m, int nd, hipStream_t s)
{
    if (m <= 0) return hipSuccess;
    hipLaunchKernelGGL(bgf_gate_head_kernel, dim3((unsigned)((m + 3) / 4)), dim3(256), 0, s, g, (const __bf16 *)pre,
                       w_head, b_head, y, score, m, nd);
    return hipGetLastError();
}

int bgf_max_blocks() { return kMaxBlocks; }

}  // namespace climber
