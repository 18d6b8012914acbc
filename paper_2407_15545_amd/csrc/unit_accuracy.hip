// Accuracy of the hardware transcendental units the kernels rely on: the error of v_exp_f32,
// v_rcp_f32 and v_sqrt_f32 in ulps of binary32, exhaustively over the stated argument ranges,
// against binary64 references computed on the GPU.  The tolerance derivation of the backward
// kernels uses these figures.  v_rcp_f64 is probed too (on a grid of 2^28 arguments in [1, 2), in
// units of 2^-53 relative): the binary32-storage forward needs a reciprocal good to about 2^-30,
// and the question is whether the instruction alone delivers that.
//
//   hipcc --offload-arch=gfx950 -O2 -o unit_accuracy unit_accuracy.hip && ./unit_accuracy
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <cmath>
#include <cstring>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

__device__ double ulp_err(float got, double ref) {
    int e; frexp(ref, &e);               // ref = m 2^e, m in [0.5,1)
    double u = ldexp(1.0, e - 24);
    return fabs((double)got - ref) / u;
}
// op: 0 exp2 on [lo,hi) patterns, 1 rcp, 2 sqrt, 3 rcp in binary64 (argument 1 + (i + hash) 2^-28)
__global__ void probe(int op, uint32_t first, uint32_t count, double* maxerr, uint32_t* argmax) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t stride = gridDim.x * blockDim.x;
    double best = 0; uint32_t arg = 0;
    for (; i < count; i += stride) {
        uint32_t bits = first + i;
        float x = __uint_as_float(bits);
        if (op == 3) {
            double d = 1.0 + ldexp((double)i, -28) + ldexp((double)(i * 2654435761u), -60);
            double e = fabs(__builtin_amdgcn_rcp(d) - 1.0 / d) * d * 9007199254740992.0;   // relative, in 2^-53
            if (e > best) { best = e; arg = i; }
            continue;
        }
        float got; double ref;
        if (op == 0) { got = __builtin_amdgcn_exp2f(x); ref = exp2((double)x); }
        else if (op == 1) { got = __builtin_amdgcn_rcpf(x); ref = 1.0 / (double)x; }
        else { got = __builtin_amdgcn_sqrtf(x); ref = sqrt((double)x); }
        double e = ulp_err(got, ref);
        if (e > best) { best = e; arg = bits; }
    }
    // block reduce (simple: atomics on a per-block slot)
    __shared__ double sb[256]; __shared__ uint32_t sa[256];
    sb[threadIdx.x] = best; sa[threadIdx.x] = arg; __syncthreads();
    for (int s = 128; s > 0; s >>= 1) { if (threadIdx.x < s && sb[threadIdx.x + s] > sb[threadIdx.x]) { sb[threadIdx.x] = sb[threadIdx.x + s]; sa[threadIdx.x] = sa[threadIdx.x + s]; } __syncthreads(); }
    if (threadIdx.x == 0) { maxerr[blockIdx.x] = sb[0]; argmax[blockIdx.x] = sa[0]; }
}
int run(const char* name, int op, float lo, float hi) {
    uint32_t a, b; memcpy(&a, &lo, 4); memcpy(&b, &hi, 4);
    if (a > b) { uint32_t t = a; a = b; b = t; }
    const int blocks = 2048;
    double* d; uint32_t* g; CK(hipMalloc(&d, blocks * 8)); CK(hipMalloc(&g, blocks * 4));
    hipLaunchKernelGGL(probe, dim3(blocks), dim3(256), 0, 0, op, a, b - a + 1, d, g);
    CK(hipDeviceSynchronize());
    static double h[blocks]; static uint32_t ha[blocks];
    CK(hipMemcpy(h, d, blocks * 8, hipMemcpyDeviceToHost)); CK(hipMemcpy(ha, g, blocks * 4, hipMemcpyDeviceToHost));
    double best = 0; uint32_t arg = 0; for (int i = 0; i < blocks; ++i) if (h[i] > best) { best = h[i]; arg = ha[i]; }
    if (op == 3) {
        printf("%-28s [1, 2) %u values: max relative err %.1f x 2^-53 = 2^%.1f at 1 + %u 2^-28\n", name, b - a + 1, best,
               log2(best) - 53.0, arg);
        fflush(stdout);
        CK(hipFree(d)); CK(hipFree(g));
        return 0;
    }
    float ax; memcpy(&ax, &arg, 4);
    printf("%-28s [%g, %g] %u values: max err %.4f ulp at x = %.9g (0x%08x)\n", name, lo, hi, b - a + 1, best, ax, arg);
    fflush(stdout);
    CK(hipFree(d)); CK(hipFree(g));
    return 0;
}
int main() {
    if (run("v_exp_f32", 0, -1e-6f, -125.9f)) return 1;     // negative arguments: patterns ascend with |x|
    if (run("v_exp_f32 (0,1)", 0, 1e-6f, 1.0f)) return 1;
    if (run("v_rcp_f32 [1,2]", 1, 1.0f, 2.0f)) return 1;
    if (run("v_rcp_f32 [1,1e30]", 1, 1.0f, 1e30f)) return 1;
    if (run("v_sqrt_f32 [1e-30,1e30]", 2, 1e-30f, 1e30f)) return 1;
    if (run("v_sqrt_f32 [2^-20,4]", 2, 9.5367431640625e-07f, 4.0f)) return 1;
    { float lo, hi; uint32_t a = 0, b = (1u << 28) - 1; memcpy(&lo, &a, 4); memcpy(&hi, &b, 4);
      if (run("v_rcp_f64", 3, lo, hi)) return 1; }
    return 0;
}
