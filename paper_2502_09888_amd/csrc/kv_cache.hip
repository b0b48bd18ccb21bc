// KV-cache writers: store one layer's history keys and values (Climber, arXiv 2502.09888,
// Sec. 3.2: per-layer K/V of the user history are produced once and reused by every candidate).
//
// bf16: the cache is written as MFMA operand fragments per 32-key block (layout in internal.h) so
// that the candidate pass reads it with linear 16-byte accesses; slots past a user's valid length
// are written as zeros whatever the source rows hold there.
// fp32: plain [rows][H][d_head] K followed by V, padded rows zeroed.
#include "internal.h"

namespace climber {
namespace {

__global__ __launch_bounds__(256) void kv_write_bf16_kernel(CacheView c, const __bf16 *k,
                                                            const __bf16 *v, int64_t ld, int H)
{
    __shared__ __attribute__((aligned(16))) __bf16 vt[kBlockKeys][kDHead + 8];
    const int kb = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int t0 = c.tok_off[b], Lpad = c.tok_off[b + 1] - t0, Lb = c.hist_len[b];
    if (kb * kBlockKeys >= Lpad) return;
    uint8_t *dst = c.layer_base + ((size_t)t0 * H + (size_t)h * Lpad) * (kDHead * 4) +
                   (size_t)kb * kBlockBytes;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint4 zero = {0, 0, 0, 0};
    {   // K fragments: chunk (s, lane) = K[32kb + lane%32][16s + 8(lane/32) + 0..7]
        const int s = tid >> 6, key = kb * kBlockKeys + (lane & 31);
        uint4 val = zero;
        if (key < Lb)
            val = *(const uint4 *)(k + (int64_t)(t0 + key) * ld + h * kDHead + 16 * s + 8 * (lane >> 5));
        ((uint4 *)dst)[tid] = val;
    }
    {   // stage the 32 x 64 V block, then gather the transposed, key-permuted fragments
        const int key_l = tid >> 3, ch = tid & 7, key = kb * kBlockKeys + key_l;
        uint4 val = zero;
        if (key < Lb) val = *(const uint4 *)(v + (int64_t)(t0 + key) * ld + h * kDHead + ch * 8);
        *(uint4 *)&vt[key_l][ch * 8] = val;
    }
    __syncthreads();
    {
        const int g = tid >> 7, db = (tid >> 6) & 1, hf = lane >> 5, d = 32 * db + (lane & 31);
        __attribute__((aligned(16))) __bf16 out[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = vt[16 * g + 8 * (e >> 2) + 4 * hf + (e & 3)][d];
        ((uint4 *)(dst + 4096))[tid] = *(const uint4 *)out;
    }
}

__global__ void kv_write_f32_kernel(CacheView c, const float *k, const float *v, int64_t ld, int H,
                                    int d_head, int64_t total_rows)
{
    const int64_t n = total_rows * H * d_head;
    float *kd = (float *)c.layer_base, *vd = kd + n;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = i / (H * d_head);
        const int col = (int)(i % (H * d_head));
        int lo = 0, hi = c.B;  // user of the row: largest b with tok_off[b] <= row
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (c.tok_off[mid] <= row) lo = mid; else hi = mid;
        }
        const bool valid = row - c.tok_off[lo] < c.hist_len[lo];
        kd[i] = valid ? k[row * ld + col] : 0.f;
        vd[i] = valid ? v[row * ld + col] : 0.f;
    }
}

}  // namespace

hipError_t launch_kv_write_bf16(const CacheView &c, const void *k, const void *v, int64_t ld, int H,
                                int max_padded_len, hipStream_t s)
{
    const dim3 grid((max_padded_len + kBlockKeys - 1) / kBlockKeys, H, c.B);
    if (grid.x == 0) return hipSuccess;
    hipLaunchKernelGGL(kv_write_bf16_kernel, grid, dim3(256), 0, s, c, (const __bf16 *)k,
                       (const __bf16 *)v, ld, H);
    return hipGetLastError();
}

hipError_t launch_kv_write_f32(const CacheView &c, const void *k, const void *v, int64_t ld, int H,
                               int d_head, int64_t total_rows, hipStream_t s)
{
    const int64_t n = total_rows * H * d_head;
    if (n == 0) return hipSuccess;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(kv_write_f32_kernel, dim3((unsigned)(blocks < 65535 ? blocks : 65535)),
                       dim3(256), 0, s, c, (const float *)k, (const float *)v, ld, H, d_head,
                       total_rows);
    return hipGetLastError();
}

}  // namespace climber
