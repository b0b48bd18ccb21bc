// Measurement aid, not a step of the method: what the instructions of the attention inner loop cost
// at the vector issue port of a SIMD, in shader clocks, with one and two waves per SIMD and no
// memory traffic.  The time is that of the whole launch (HIP events: every wave counts, whatever the
// arbitration between the waves of a SIMD); the clock is read inside the kernel as the ratio of the
// cycle counter (clock64) to the 100 MHz wall clock (wall_clock64) over the same loop:
//   - v_exp_f32, v_add_f32, v_cvt_pk_bf16_f32 alone and mixed (do transcendental and plain
//     instructions overlap?);
//   - how long an MFMA keeps the SIMD from issuing vector instructions: slots of one MFMA followed
//     by KV independent v_fma_f32; the time per slot beyond KV times the plain instruction cost is
//     what the MFMA took from the port (variants: accumulator in VGPRs / AGPRs, rotating / chained,
//     operands A and B in AGPRs, 32x32x16 / 16x16x32).
//
//   hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o issue_port paper_2502_09888_amd/probes/issue_port.hip && ./issue_port
#include <hip/hip_runtime.h>

#include <cstdio>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

enum { EXP, ADD, CVT, EXP_THEN_ADD, EXP_ADD_MIXED, EXP_CVT_MIXED, ADD_CVT_MIXED };

template <int MODE>
__global__ __launch_bounds__(256) void valu_kernel(float *out, unsigned long long *ticks, int iters)
{
    float x[16], y[16];
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * (threadIdx.x + i), y[i] = 0.002f * (threadIdx.x + i);
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (MODE == EXP || MODE == EXP_THEN_ADD) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
            if (MODE == ADD) asm volatile("v_add_f32 %0, %0, %0" : "+v"(y[i]));
            if (MODE == CVT) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %0" : "+v"(y[i]));
            if (MODE == EXP_ADD_MIXED) {
                asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
                asm volatile("v_add_f32 %0, %0, %0" : "+v"(y[i]));
            }
            if (MODE == EXP_CVT_MIXED) {
                asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
                asm volatile("v_cvt_pk_bf16_f32 %0, %0, %0" : "+v"(y[i]));
            }
            if (MODE == ADD_CVT_MIXED) {
                asm volatile("v_add_f32 %0, %0, %0" : "+v"(x[i]));
                asm volatile("v_cvt_pk_bf16_f32 %0, %0, %0" : "+v"(y[i]));
            }
        }
        if (MODE == EXP_THEN_ADD) {
#pragma unroll
            for (int i = 0; i < 16; ++i) asm volatile("v_add_f32 %0, %0, %0" : "+v"(y[i]));
        }
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    float s = 0;
    for (int i = 0; i < 16; ++i) s += x[i] + y[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) ticks[0] = c1 - c0, ticks[1] = w1 - w0;
}

enum { M32_VGPR, M32_AGPR, M32_VGPR_CHAINED, M16_VGPR, M32_AB_AGPR, M32_A_AGPR };

template <int MODE, int KV>
__global__ __launch_bounds__(256) void mfma_kernel(float *out, unsigned long long *ticks, int iters)
{
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) a[e] = (__bf16)(float)(threadIdx.x % 7), b[e] = (__bf16)(float)(threadIdx.x % 5);
    f32x16 acc[4];
    f32x4 acs[4];
    for (int i = 0; i < 4; ++i) {
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
        for (int r = 0; r < 4; ++r) acs[i][r] = 0.f;
    }
    float x[16];
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * (threadIdx.x + i);
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = MODE == M32_VGPR_CHAINED ? 0 : i;
            if (MODE == M32_VGPR || MODE == M32_VGPR_CHAINED)
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(a), "v"(b));
            if (MODE == M32_AGPR) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[j]) : "v"(a), "v"(b));
            if (MODE == M16_VGPR) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acs[j]) : "v"(a), "v"(b));
            if (MODE == M32_AB_AGPR) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[j]) : "a"(a), "a"(b));
            if (MODE == M32_A_AGPR) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[j]) : "a"(a), "v"(b));
#pragma unroll
            for (int k = 0; k < KV; ++k) asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[(i * KV + k) % 16]));
        }
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    float s = 0;
    for (int i = 0; i < 4; ++i) {
        for (int r = 0; r < 16; ++r) s += acc[i][r];
        for (int r = 0; r < 4; ++r) s += acs[i][r];
    }
    for (int i = 0; i < 16; ++i) s += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) ticks[0] = c1 - c0, ticks[1] = w1 - w0;
}

#define CK(x)                                                                     \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("HIP error %s, line %d\n", hipGetErrorString(e_), __LINE__);   \
            return 1;                                                             \
        }                                                                         \
    } while (0)

// shader clocks that one iteration of one wave costs at its SIMD: launch time x clock / (waves per
// SIMD x iterations)
template <class F>
int clocks_per_iteration(F launch, int waves_per_simd, int iters, double *out, double *ghz)
{
    unsigned long long *ticks;
    hipEvent_t e0, e1;
    CK(hipMalloc(&ticks, 16));
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch(256 * waves_per_simd, iters / 10, ticks);
    CK(hipEventRecord(e0));
    launch(256 * waves_per_simd, iters, ticks);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    unsigned long long h[2];
    CK(hipMemcpy(h, ticks, 16, hipMemcpyDeviceToHost));
    CK(hipFree(ticks));
    *ghz = (double)h[0] / ((double)h[1] * 10.0);
    *out = ms * 1e6 * *ghz / ((double)waves_per_simd * iters);
    return 0;
}

template <int MODE>
int run_valu(float *buf, const char *name, int n_instr)
{
    for (int w = 1; w <= 2; ++w) {
        double c, ghz;
        if (clocks_per_iteration([&](int g, int it, unsigned long long *t) { valu_kernel<MODE><<<g, 256>>>(buf, t, it); }, w, 20000, &c, &ghz))
            return 1;
        printf("%-26s %d wave(s)/SIMD at %.2f GHz: %.2f clocks per instruction at the SIMD\n", name, w, ghz, c / n_instr);
    }
    return 0;
}

template <int MODE, int KV>
int run_mfma(float *buf, const char *name)
{
    double c, ghz;
    if (clocks_per_iteration([&](int g, int it, unsigned long long *t) { mfma_kernel<MODE, KV><<<g, 256>>>(buf, t, it); }, 2, 20000, &c, &ghz))
        return 1;
    printf("%-26s 2 waves/SIMD at %.2f GHz, 1 MFMA + %2d v_fma_f32 per slot: %5.1f clocks per slot at the SIMD\n", name, ghz, KV, c / 4);
    return 0;
}

int main()
{
    float *buf;
    CK(hipMalloc(&buf, 256 * 2 * 256 * sizeof(float)));
    run_valu<EXP>(buf, "v_exp_f32", 16);
    run_valu<ADD>(buf, "v_add_f32", 16);
    run_valu<CVT>(buf, "v_cvt_pk_bf16_f32", 16);
    run_valu<EXP_THEN_ADD>(buf, "16 exp, then 16 add", 32);
    run_valu<EXP_ADD_MIXED>(buf, "exp / add alternating", 32);
    run_valu<EXP_CVT_MIXED>(buf, "exp / cvt alternating", 32);
    run_valu<ADD_CVT_MIXED>(buf, "add / cvt alternating", 32);
    run_mfma<M32_VGPR, 0>(buf, "32x32x16, VGPR acc");
    run_mfma<M32_VGPR, 8>(buf, "32x32x16, VGPR acc");
    run_mfma<M32_VGPR, 12>(buf, "32x32x16, VGPR acc");
    run_mfma<M32_VGPR, 16>(buf, "32x32x16, VGPR acc");
    run_mfma<M32_AGPR, 12>(buf, "32x32x16, AGPR acc");
    run_mfma<M32_AGPR, 16>(buf, "32x32x16, AGPR acc");
    run_mfma<M32_VGPR_CHAINED, 12>(buf, "32x32x16, one acc chained");
    run_mfma<M32_VGPR_CHAINED, 16>(buf, "32x32x16, one acc chained");
    run_mfma<M32_AB_AGPR, 12>(buf, "32x32x16, A and B in AGPRs");
    run_mfma<M32_AB_AGPR, 16>(buf, "32x32x16, A and B in AGPRs");
    run_mfma<M32_A_AGPR, 12>(buf, "32x32x16, A in AGPRs");
    run_mfma<M32_A_AGPR, 16>(buf, "32x32x16, A in AGPRs");
    run_mfma<M16_VGPR, 0>(buf, "16x16x32, VGPR acc");
    run_mfma<M16_VGPR, 8>(buf, "16x16x32, VGPR acc");
    run_mfma<M16_VGPR, 12>(buf, "16x16x32, VGPR acc");
    return 0;
}
