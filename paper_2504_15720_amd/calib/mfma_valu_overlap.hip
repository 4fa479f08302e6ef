// How far do matrix instructions (v_mfma_f32_16x16x32_bf16) and ordinary vector instructions overlap on one
// SIMD of gfx950?  Times loops of 16 matrix instructions, of 48 multiply-adds, and of both (interleaved in one
// wave, one after the other, or in two waves of the same SIMD), with one and with two waves per SIMD.  The
// prefill kernel's bound on the shared issue port is derived from these figures.
// Build: hipcc --offload-arch=gfx950 -O3 [-DVGPR_SOURCES] mfma_valu_overlap.hip -o mfma_valu_overlap ; run without arguments.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

template <int MODE>
__global__ void __launch_bounds__(512) k(float *out, long long *cyc, int iters) {
    const int lane = threadIdx.x;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(lane % 3); b[i] = (__bf16)(float)(lane % 5); }
    f32x4 c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
    f32x16 w0 = {0}, w1 = w0;
    float x0 = lane, x1 = lane + 1, x2 = lane + 2, x3 = lane + 3, x4 = lane * 0.5f, x5 = lane * 0.25f;
#ifdef VGPR_SOURCES // every fma reads three vector registers (else one register and two constants)
    float m = 1.0001f + 1e-9f * lane, d = 0.5f + 1e-9f * lane;
    asm volatile("" : "+v"(m), "+v"(d));
#else
    const float m = 1.0001f, d = 0.5f;
#endif
    const int wave = threadIdx.x / 64;
    // waves are placed round-robin on the 4 SIMDs: waves w and w+4 share a SIMD
    const bool second = wave >= 4;
    long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#define M4 c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c0, 0, 0, 0); c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c1, 0, 0, 0); \
           c2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c2, 0, 0, 0); c3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c3, 0, 0, 0);
#define V6 x0 = __builtin_fmaf(x0, m, d); x1 = __builtin_fmaf(x1, m, d); x2 = __builtin_fmaf(x2, m, d); x3 = __builtin_fmaf(x3, m, d); \
           x4 = __builtin_fmaf(x4, m, d); x5 = __builtin_fmaf(x5, m, d);
#define E2 x0 = __builtin_amdgcn_exp2f(x0); x1 = __builtin_amdgcn_exp2f(x1);
        if (MODE == 0) { M4 M4 M4 M4 }                       // 16 MFMA
        if (MODE == 1) { V6 V6 V6 V6 V6 V6 V6 V6 }           // 48 VALU
        if (MODE == 2) {                                      // interleaved in one wave: M v v v
#define MV(cc) cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, cc, 0, 0, 0); __builtin_amdgcn_sched_barrier(0); \
               x0 = __builtin_fmaf(x0, m, d); x1 = __builtin_fmaf(x1, m, d); x2 = __builtin_fmaf(x2, m, d); __builtin_amdgcn_sched_barrier(0);
#define MW(cc) cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, cc, 0, 0, 0); __builtin_amdgcn_sched_barrier(0); \
               x3 = __builtin_fmaf(x3, m, d); x4 = __builtin_fmaf(x4, m, d); x5 = __builtin_fmaf(x5, m, d); __builtin_amdgcn_sched_barrier(0);
            MV(c0) MW(c1) MV(c2) MW(c3) MV(c0) MW(c1) MV(c2) MW(c3) MV(c0) MW(c1) MV(c2) MW(c3) MV(c0) MW(c1) MV(c2) MW(c3)
        }
        if (MODE == 3) {                                      // two waves per SIMD: one does MFMA, the other VALU
            if (second) { V6 V6 V6 V6 V6 V6 V6 V6 } else { M4 M4 M4 M4 }
        }
        if (MODE == 4) { E2 E2 E2 E2 E2 E2 E2 E2 }           // 16 v_exp
        if (MODE == 5) {                                      // MFMA block then VALU block in one wave (no interleave)
            M4 M4 M4 M4 __builtin_amdgcn_sched_barrier(0); V6 V6 V6 V6 V6 V6 V6 V6 __builtin_amdgcn_sched_barrier(0);
        }
        if (MODE == 6) {                                      // interleaved M e (exp under MFMA)
#define ME(cc, xx) cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, cc, 0, 0, 0); __builtin_amdgcn_sched_barrier(0); \
               xx = __builtin_amdgcn_exp2f(xx); __builtin_amdgcn_sched_barrier(0);
            ME(c0, x0) ME(c1, x1) ME(c2, x2) ME(c3, x3) ME(c0, x4) ME(c1, x5) ME(c2, x0) ME(c3, x1)
            ME(c0, x2) ME(c1, x3) ME(c2, x4) ME(c3, x5) ME(c0, x0) ME(c1, x1) ME(c2, x2) ME(c3, x3)
        }
        if (MODE == 7) {                                      // 8 matrix instructions of twice the size (32x32x16)
#define B2 w0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, w0, 0, 0, 0); w1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, w1, 0, 0, 0);
            B2 B2 B2 B2
        }
        if (MODE == 8) {                                      // 8 x (32x32x16 + 6 fma) interleaved
#define BV(ww) ww = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, ww, 0, 0, 0); __builtin_amdgcn_sched_barrier(0); V6 __builtin_amdgcn_sched_barrier(0);
            BV(w0) BV(w1) BV(w0) BV(w1) BV(w0) BV(w1) BV(w0) BV(w1)
        }
    }
    long long t1 = __builtin_readcyclecounter();
    out[blockIdx.x * blockDim.x + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3] + w0[5] + w1[7] + x0 + x1 + x2 + x3 + x4 + x5;
    if (threadIdx.x % 64 == 0) cyc[blockIdx.x * (blockDim.x / 64) + wave] = t1 - t0;
}

template <int MODE>
int run(const char *name, int threads, int iters) {
    const int blocks = 256;
    float *out; long long *cyc;
    CHECK(hipMalloc(&out, sizeof(float) * blocks * threads));
    CHECK(hipMalloc(&cyc, sizeof(long long) * blocks * (threads / 64)));
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    hipLaunchKernelGGL(k<MODE>, dim3(blocks), dim3(threads), 0, 0, out, cyc, 10);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL(k<MODE>, dim3(blocks), dim3(threads), 0, 0, out, cyc, iters);
    CHECK(hipEventRecord(e1));
    CHECK(hipDeviceSynchronize());
    float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
    std::vector<long long> h(blocks * (threads / 64));
    CHECK(hipMemcpy(h.data(), cyc, h.size() * sizeof(long long), hipMemcpyDeviceToHost));
    double s = 0; for (auto v : h) s += v;
    printf("%-44s waves/SIMD %d: %.3f ms, %.1f ns per iteration, counter ticks per iteration %.1f\n", name, threads / 256, ms,
           ms * 1e6 / iters, s / h.size() / iters);
    fflush(stdout);
    CHECK(hipFree(out)); CHECK(hipFree(cyc));
    return 0;
}

int main() {
    const int it = 20000;
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    printf("%s, %d CUs, clock %.0f MHz; one workgroup per CU, a wave per SIMD (256 lanes) or two (512)\n", prop.name,
           prop.multiProcessorCount, prop.clockRate / 1000.0);
#ifdef VGPR_SOURCES
    printf("fma with three vector-register sources\n");
#else
    printf("fma with one vector-register source and two constants\n");
#endif
    if (run<0>("16 MFMA", 256, it)) return 1;
    if (run<1>("48 VALU fma", 256, it)) return 1;
    if (run<2>("16 x (MFMA + 3 fma) interleaved", 256, it)) return 1;
    if (run<5>("16 MFMA then 48 fma", 256, it)) return 1;
    if (run<4>("16 v_exp", 256, it)) return 1;
    if (run<6>("16 x (MFMA + v_exp) interleaved", 256, it)) return 1;
    if (run<7>("8 MFMA 32x32x16", 256, it)) return 1;
    if (run<8>("8 x (MFMA 32x32x16 + 6 fma) interleaved", 256, it)) return 1;
    if (run<0>("16 MFMA", 512, it)) return 1;
    if (run<1>("48 VALU fma", 512, it)) return 1;
    if (run<3>("wave A 16 MFMA, wave B 48 fma", 512, it)) return 1;
    if (run<2>("16 x (MFMA + 3 fma) interleaved", 512, it)) return 1;
    if (run<5>("16 MFMA then 48 fma", 512, it)) return 1;
    if (run<7>("8 MFMA 32x32x16", 512, it)) return 1;
    if (run<8>("8 x (MFMA 32x32x16 + 6 fma) interleaved", 512, it)) return 1;
    return 0;
}
