// Bit-wise gating fusion of Climber (arXiv 2502.09888, Sec. 3.1.4, Eq. (4)): the two small kernels
// around the projections of the fusion layer.
//   fusion attention: G = ATL(E): every one of a candidate's N_b block outputs attends to all N_b of
//     them, no relative attention bias, temperature from the candidate's scenario only;
//   gate + head: Y = G (.) sigmoid(f_gate(G)), score = <w_head, vec(Y)> + b.
// N_b is a handful (the number of extraction strategies), so the attention is N_b x N_b logits per
// (candidate, head), held in registers; d_head = 64.
#include "bgf.h"
#include "lanes.h"

namespace climber {
namespace {

constexpr int kMaxBlocks = 16;

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;

// sum over the 8 lanes 8s .. 8s+7, in each of them
__device__ __forceinline__ float sum8(float x)
{
    auto dpp = [](float v, auto ctrl) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, false));
    };
    x += dpp(x, std::integral_constant<int, 0xB1>{});   // quad_perm [1,0,3,2]
    x += dpp(x, std::integral_constant<int, 0x4E>{});   // quad_perm [2,3,0,1]
    x += dpp(x, std::integral_constant<int, 0x141>{});  // row_half_mirror: the other quad of the eight
    return x;
}

// qkv: bf16 [m * NB][3 * d] (queries | keys | values, head h at column h * 64); o: bf16 [m * NB][d].
// One wavefront per (candidate, group of 8 heads): lane = (head 8g + lane / 8, features 8 (lane % 8) ..
// + 7), so that every row of a head is loaded and stored as whole 128-byte lines, 16 bytes per lane;
// a logit is 8 products per lane and a sum over the 8 lanes of the head.
template <int NB>
__global__ __launch_bounds__(256) void bgf_attention_kernel(const __bf16 *qkv, __bf16 *o, const int32_t *scen,
                                                            const float *tau_scen, int n_scen, int64_t m, int H,
                                                            float scale_log2e)
{
    const int lane = threadIdx.x & 63, c8 = lane & 7;
    const int groups = (H + 7) >> 3;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (candidate, group of heads)
    if (item >= m * groups) return;
    const int64_t c = item / groups;
    const int h = (int)(item % groups) * 8 + (lane >> 3), d = H * 64;
    if (h >= H) return;  // whole groups of 8 lanes leave; the sums below stay inside such a group
    const int sc = min(max(scen[c], 0), n_scen - 1);
    const float cs = scale_log2e / tau_scen[sc];
    const __bf16 *base = qkv + c * NB * 3 * (int64_t)d + h * 64 + c8 * 8;
    bf16x8 kj[NB], vj[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        kj[j] = *(const bf16x8 *)(base + (int64_t)j * 3 * d + d);
        vj[j] = *(const bf16x8 *)(base + (int64_t)j * 3 * d + 2 * d);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const bf16x8 qi = *(const bf16x8 *)(base + (int64_t)i * 3 * d);
        float t[NB], mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = fmaf((float)qi[e], (float)kj[j][e], dot);
            t[j] = sum8(dot) * cs;  // log2 units
            mx = fmaxf(mx, t[j]);
        }
        float sum = 0.f, acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const float pj = exp2f(t[j] - mx);
            sum += pj;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(pj, (float)vj[j][e], acc[e]);
        }
        const float inv = 1.f / sum;
        bf16x8 ov;
#pragma unroll
        for (int e = 0; e < 8; ++e) ov[e] = (__bf16)(acc[e] * inv);
        *(bf16x8 *)(o + (c * NB + i) * (int64_t)d + h * 64 + c8 * 8) = ov;
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
    // four consecutive values per lane and step (nd is a multiple of 64): 16-byte loads and stores
    for (int e = lane * 4; e < nd; e += 256) {
        const float4 gv = *(const float4 *)(g + c * nd + e);
        const float4 wv = *(const float4 *)(w_head + e);
        const bf16x4 pv = *(const bf16x4 *)(pre + c * nd + e);
        float4 yv;
        yv.x = gv.x * __builtin_amdgcn_rcpf(1.f + __expf(-(float)pv[0]));
        yv.y = gv.y * __builtin_amdgcn_rcpf(1.f + __expf(-(float)pv[1]));
        yv.z = gv.z * __builtin_amdgcn_rcpf(1.f + __expf(-(float)pv[2]));
        yv.w = gv.w * __builtin_amdgcn_rcpf(1.f + __expf(-(float)pv[3]));
        if (y) *(float4 *)(y + c * nd + e) = yv;
        acc = fmaf(yv.x, wv.x, fmaf(yv.y, wv.y, fmaf(yv.z, wv.z, fmaf(yv.w, wv.w, acc))));
    }
    acc = wave_sum64(acc);
    if (lane == 0) score[c] = acc + b_head;
}

}  // namespace

hipError_t launch_bgf_attention(const void *qkv, void *o, const int32_t *scen, const float *tau_scen, int n_scen,
                                int64_t m, int nb, int H, float qk_scale, hipStream_t s)
{
    if (m <= 0) return hipSuccess;
    if (nb < 1 || nb > kMaxBlocks) return hipErrorInvalidValue;
    const int64_t items = m * ((H + 7) / 8);
    const dim3 grid((unsigned)((items + 3) / 4)), block(256);
    const float sl = qk_scale * 1.4426950408889634f;
    auto go = [&](auto nb_tag) {
        constexpr int NB = decltype(nb_tag)::value;
        hipLaunchKernelGGL(bgf_attention_kernel<NB>, grid, block, 0, s, (const __bf16 *)qkv, (__bf16 *)o, scen, tau_scen,
                           n_scen, m, H, sl);
    };
    switch (nb) {
#define CLIMBER_BGF_CASE(N) case N: go(std::integral_constant<int, N>{}); break;
        CLIMBER_BGF_CASE(1) CLIMBER_BGF_CASE(2) CLIMBER_BGF_CASE(3) CLIMBER_BGF_CASE(4) CLIMBER_BGF_CASE(5)
        CLIMBER_BGF_CASE(6) CLIMBER_BGF_CASE(7) CLIMBER_BGF_CASE(8) CLIMBER_BGF_CASE(9) CLIMBER_BGF_CASE(10)
        CLIMBER_BGF_CASE(11) CLIMBER_BGF_CASE(12) CLIMBER_BGF_CASE(13) CLIMBER_BGF_CASE(14) CLIMBER_BGF_CASE(15)
        CLIMBER_BGF_CASE(16)
#undef CLIMBER_BGF_CASE
    default: return hipErrorInvalidValue;
    }
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
