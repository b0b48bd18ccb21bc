// Measurement aid, not a step of the method: what HBM gives a kernel by direction -- read-only,
// write-only, and copies (mixed read/write streams) in a few launch shapes, on 1 GiB buffers with
// 16 bytes per lane.  The history pass and the residual projections are quoted against these rates.
//
//   hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o hbm_copy paper_2502_09888_amd/probes/hbm_copy.hip && ./hbm_copy
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

__global__ __launch_bounds__(256) void read_kernel(const u32x4 *a, u32x4 *sink, size_t n)
{
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        acc ^= __builtin_nontemporal_load(a + i);
    if (acc[0] == 0x12345678u) sink[threadIdx.x] = acc;   // keeps the loads alive
}

__global__ __launch_bounds__(256) void write_kernel(u32x4 *a, size_t n, uint32_t v)
{
    const u32x4 x = {v, v + 1, v + 2, v + 3};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) a[i] = x;
}

// grid-stride copy, U loads in flight per lane before the stores
template <int U>
__global__ __launch_bounds__(256) void copy_kernel(const u32x4 *a, u32x4 *b, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i + (U - 1) * stride < n; i += U * stride) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = a[i + u * stride];
#pragma unroll
        for (int u = 0; u < U; ++u) b[i + u * stride] = v[u];
    }
}

// every workgroup owns contiguous chunks of 64 KiB (the shape of the history pass: one subsequence's
// rows in, its cache blocks out)
__global__ __launch_bounds__(256) void copy_chunks_kernel(const u32x4 *a, u32x4 *b, size_t n)
{
    constexpr size_t per = 65536 / 16;
    for (size_t c = blockIdx.x; c * per < n; c += gridDim.x) {
        const u32x4 *s = a + c * per;
        u32x4 *d = b + c * per;
        for (size_t i = threadIdx.x; i < per; i += 1024) {
            const u32x4 v0 = s[i], v1 = s[i + 256], v2 = s[i + 512], v3 = s[i + 768];
            d[i] = v0, d[i + 256] = v1, d[i + 512] = v2, d[i + 768] = v3;
        }
    }
}

#define CK(x)                                                                     \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("HIP error %s, line %d\n", hipGetErrorString(e_), __LINE__);   \
            return 1;                                                             \
        }                                                                         \
    } while (0)

template <class F>
int timed(const char *name, double bytes_per_launch, F launch)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch(0);
    launch(1);
    CK(hipEventRecord(e0));
    for (int i = 0; i < 10; ++i) launch(i);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    printf("%-44s %.2f TB/s\n", name, 10.0 * bytes_per_launch / ms / 1e9);
    return 0;
}

int main()
{
    const size_t bytes = (size_t)1 << 30, n = bytes / 16;
    u32x4 *a, *b, *sink;
    CK(hipMalloc(&a, bytes));
    CK(hipMalloc(&b, bytes));
    CK(hipMalloc(&sink, 4096));
    CK(hipMemset(a, 1, bytes));
    CK(hipMemset(b, 2, bytes));
    auto src = [&](int i) { return i & 1 ? a : b; };
    auto dst = [&](int i) { return i & 1 ? b : a; };
    timed("read only", bytes, [&](int i) { read_kernel<<<2048, 256>>>(src(i), sink, n); });
    timed("write only", bytes, [&](int i) { write_kernel<<<2048, 256>>>(src(i), n, i); });
    for (int g : {1024, 2048, 16384}) {
        char nm[64];
        snprintf(nm, sizeof nm, "copy (read + write bytes), grid %d", g);
        timed(nm, 2.0 * bytes, [&](int i) { copy_kernel<1><<<g, 256>>>(src(i), dst(i), n); });
        snprintf(nm, sizeof nm, "copy, 4 loads in flight per lane, grid %d", g);
        timed(nm, 2.0 * bytes, [&](int i) { copy_kernel<4><<<g, 256>>>(src(i), dst(i), n); });
    }
    timed("copy, 64 KiB chunk per workgroup, grid 512", 2.0 * bytes,
          [&](int i) { copy_chunks_kernel<<<512, 256>>>(src(i), dst(i), n); });
    timed("hipMemcpyAsync device to device", 2.0 * bytes,
          [&](int i) { (void)hipMemcpyAsync(dst(i), src(i), bytes, hipMemcpyDeviceToDevice, 0); });
    return 0;
}
