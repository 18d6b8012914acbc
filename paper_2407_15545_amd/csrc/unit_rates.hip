// Issue rate of the VALU instructions the kernels are made of (8 independent chains per lane,
// 8 waves per SIMD, no memory traffic), in lanes per clock and compute unit at 2.4 GHz.  The
// instruction budget per byte quoted for the kernels comes from these figures.
// (v_cndmask_b32 with an implicit VCC that no VALU instruction has written recently measures a
// hazard, not the instruction: the "cmp+cndmask pair" and the e64 form show its real rate.)
//
//   hipcc --offload-arch=gfx950 -O3 -o unit_rates unit_rates.hip && ./unit_rates
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
constexpr int ITER = 4096, CH = 8;
template <int OP> __global__ __launch_bounds__(256) void k(float* out, float seed) {
    float f[CH]; double d[CH];
    for (int i = 0; i < CH; ++i) { f[i] = seed + i + threadIdx.x * 1e-3f; d[i] = f[i]; }
    for (int it = 0; it < ITER; ++it) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            if (OP == 0) asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(f[i]));
            if (OP == 1) asm volatile("v_fma_f64 %0, %0, %0, %0" : "+v"(d[i]));
            if (OP == 2) asm volatile("v_mul_f64 %0, %0, %0" : "+v"(d[i]));
            if (OP == 3) asm volatile("v_add_f64 %0, %0, %0" : "+v"(d[i]));
            if (OP == 4) asm volatile("v_cvt_f64_f32 %0, %1" : "=v"(d[i]) : "v"(f[i]));
            if (OP == 5) asm volatile("v_cvt_f32_f64 %0, %1" : "=v"(f[i]) : "v"(d[i]));
            if (OP == 6) asm volatile("v_exp_f32 %0, %0" : "+v"(f[i]));
            if (OP == 7) asm volatile("v_rcp_f64 %0, %0" : "+v"(d[i]));
            if (OP == 8) asm volatile("v_sqrt_f32 %0, %0" : "+v"(f[i]));
            if (OP == 9) asm volatile("v_cndmask_b32 %0, %0, %0, vcc" : "+v"(f[i]));
            if (OP == 10) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %0" : "+v"(f[i]));
            if (OP == 11) asm volatile("v_mul_f32 %0, %0, %0" : "+v"(f[i]));
            if (OP == 12) asm volatile("v_cmp_lt_f32 vcc, %0, %0" :: "v"(f[i]) : "vcc");
            if (OP == 13) asm volatile("v_rcp_f32 %0, %0" : "+v"(f[i]));
            if (OP == 14) asm volatile("v_ldexp_f32 %0, %0, 1" : "+v"(f[i]));
            if (OP == 15) asm volatile("v_med3_f32 %0, %0, %0, %0" : "+v"(f[i]));
            if (OP == 17) asm volatile("v_fmac_f32 %0, %1, %1" : "+v"(f[i]) : "v"(f[(i+1)%CH]));
            if (OP == 18) asm volatile("v_bfe_u32 %0, %0, 3, 1" : "+v"(f[i]));
            if (OP == 19) asm volatile("v_lshlrev_b32 %0, 16, %0" : "+v"(f[i]));
            if (OP == 20) asm volatile("v_cndmask_b32 %0, %1, %2, vcc" : "=v"(f[i]) : "v"(f[(i+1)%CH]), "v"(f[(i+2)%CH]));
            if (OP == 21) asm volatile("v_cndmask_b32_e64 %0, %1, %2, s[10:11]" : "=v"(f[i]) : "v"(f[(i+1)%CH]), "v"(f[(i+2)%CH]));
            if (OP == 22) asm volatile("v_cmp_lt_f32 vcc, %1, %2\n v_cndmask_b32 %0, %1, %2, vcc" : "=v"(f[i]) : "v"(f[(i+1)%CH]), "v"(f[(i+2)%CH]) : "vcc");
            if (OP == 23) asm volatile("v_add_f32 %0, %0, %0" : "+v"(f[i]));
            if (OP == 24) asm volatile("v_max_f32 %0, %0, %0" : "+v"(f[i]));
            if (OP == 25) asm volatile("v_and_b32 %0, 0xffff0000, %0" : "+v"(f[i]));
            if (OP == 26) asm volatile("v_bfi_b32 %0, %0, %1, %2" : "+v"(f[i]) : "v"(f[(i+1)%CH]), "v"(f[(i+2)%CH]));
            if (OP == 27) asm volatile("v_or3_b32 %0, %0, %1, %2" : "+v"(f[i]) : "v"(f[(i+1)%CH]), "v"(f[(i+2)%CH]));
            if (OP == 28) asm volatile("v_cmp_lt_f32 s[10:11], %0, %1" :: "v"(f[i]), "v"(f[(i+1)%CH]) : "s10", "s11");
            if (OP == 29) asm volatile("v_sub_f32 %0, %0, %1" : "+v"(f[i]) : "v"(f[(i+1)%CH]));
        }
    }
    float s = 0; for (int i = 0; i < CH; ++i) s += f[i] + (float)d[i];
    if (s == 12345.678f) out[threadIdx.x] = s;
}
template <int OP> void run(const char* name, float* out) {
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int blocks = 256 * 8;      // 8 blocks of 4 waves per CU = 8 waves per SIMD
    hipLaunchKernelGGL(k<OP>, dim3(blocks), dim3(256), 0, 0, out, 1.0f); CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0)); hipLaunchKernelGGL(k<OP>, dim3(blocks), dim3(256), 0, 0, out, 1.0f); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    double lane_ops = (double)blocks * 256 * ITER * CH;
    printf("%-18s %8.3f ms  %7.2f T lane-ops/s  (%.2f lanes/clk/CU at 2.4 GHz)\n", name, ms, lane_ops / ms / 1e9, lane_ops / (ms * 1e-3) / 256 / 2.4e9); fflush(stdout);
}
int main() {
    float* out; CK(hipMalloc(&out, 4096));
    run<0>("v_fma_f32", out); run<11>("v_mul_f32", out); run<17>("v_fmac_f32", out);
    run<1>("v_fma_f64", out); run<2>("v_mul_f64", out); run<3>("v_add_f64", out);
    run<4>("v_cvt_f64_f32", out); run<5>("v_cvt_f32_f64", out); run<7>("v_rcp_f64", out);
    run<6>("v_exp_f32", out); run<8>("v_sqrt_f32", out); run<13>("v_rcp_f32", out);
    run<9>("v_cndmask_b32", out); run<12>("v_cmp_lt_f32", out); run<10>("v_cvt_pk_bf16_f32", out);
    run<20>("cndmask vcc 3reg", out); run<21>("cndmask e64 sgpr", out); run<22>("cmp+cndmask pair", out); run<23>("v_add_f32", out); run<24>("v_max_f32", out);
    run<25>("v_and_b32 lit", out); run<26>("v_bfi_b32", out); run<27>("v_or3_b32", out); run<28>("v_cmp -> sgpr", out); run<29>("v_sub_f32", out);
    run<14>("v_ldexp_f32", out); run<15>("v_med3_f32", out); run<18>("v_bfe_u32", out); run<19>("v_lshlrev_b32", out);
    return 0;
}
