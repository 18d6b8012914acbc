// Streaming ceiling of the machine: R read streams and W write streams of 128-bit
// accesses with no arithmetic, over the launch shapes a streaming kernel can
// take.  The figures bound what any kernel with the same stream mix can reach;
// the library's kernels are compared against them, not only against the
// 8 TB/s data-sheet peak, and the library's launch shape (single-wavefront
// workgroups, a cap on resident wavefronts per compute unit) comes from here.
//
//   hipcc --offload-arch=gfx950 -O3 -o membench membench.hip && ./membench
//
// Every tensor has the size of one bf16 tensor of the SwiGLU workload
// (4 x 4096 x 14336 x 2 bytes = 469.8 MB), far beyond the 256 MB Infinity Cache.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); std::exit(1); } } while (0)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
struct Ptrs { const u32x4* r[4]; u32x4* w[4]; };
constexpr unsigned kLdsPerCu = 160 * 1024;

template <bool NT> __device__ __forceinline__ u32x4 ld(const u32x4* p) { return NT ? __builtin_nontemporal_load(p) : *p; }
template <bool NT> __device__ __forceinline__ void st(u32x4* p, u32x4 v) { if (NT) __builtin_nontemporal_store(v, p); else *p = v; }

// One tile of U * blockDim vectors per workgroup (PERSISTENT = false) or a grid-stride loop.
// The workgroup size and the dynamic LDS (never touched: it only limits how many workgroups
// a compute unit holds at a time) are launch parameters.
template <int R, int W, int U, bool NT, bool PERSISTENT>
__global__ __launch_bounds__(1024) void stream(Ptrs p, size_t vecs)
{
    const unsigned bd = blockDim.x;
    auto body = [&](size_t c, size_t step) {
        u32x4 v[U][R > 0 ? R : 1];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r) v[u][r] = ld<NT>(p.r[r] + c + u * step);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            u32x4 acc = {1u, 2u, 3u, (uint32_t)c};
#pragma unroll
            for (int r = 0; r < R; ++r) acc ^= v[u][r];
            if (W == 0) { if (acc[0] == 0x12345678u && acc[1] == 0x9abcdef0u) p.w[0][threadIdx.x] = acc; }
#pragma unroll
            for (int w = 0; w < W; ++w) st<NT>(p.w[w] + c + u * step, acc + (uint32_t)w);
        }
    };
    if (PERSISTENT) {
        const size_t stride = (size_t)gridDim.x * bd;
        for (size_t c = (size_t)blockIdx.x * bd + threadIdx.x; c + (U - 1) * stride < vecs; c += U * stride) body(c, stride);
    } else {
        const size_t c = (size_t)blockIdx.x * bd * U + threadIdx.x;
        if (c + (U - 1) * (size_t)bd < vecs) body(c, bd);
    }
}

// binary32-style access: two vectors per lane and step, adjacent (32 B per lane) or split (1 KiB apart)
template <int R, int W, bool SPLIT>
__global__ __launch_bounds__(64) void stream_pair(Ptrs p, size_t pairs)
{
    const size_t c = (size_t)blockIdx.x * 64 + threadIdx.x;
    if (c >= pairs) return;
    const size_t i0 = SPLIT ? (c / 64) * 128 + c % 64 : 2 * c, i1 = SPLIT ? i0 + 64 : i0 + 1;
    u32x4 a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < R; ++r) { a ^= ld<true>(p.r[r] + i0); b ^= ld<true>(p.r[r] + i1); }
#pragma unroll
    for (int w = 0; w < W; ++w) { st<true>(p.w[w] + i0, a + (uint32_t)w); st<true>(p.w[w] + i1, b + (uint32_t)w); }
}

template <class F> float median_ms(F launch, int iters)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    launch(); launch(); CK(hipDeviceSynchronize());
    std::vector<float> ts;
    for (int t = 0; t < 5; ++t) {
        CK(hipEventRecord(e0));
        for (int i = 0; i < iters; ++i) launch();
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ts.push_back(ms / iters);
    }
    CK(hipGetLastError());
    CK(hipEventDestroy(e0)); CK(hipEventDestroy(e1));
    std::sort(ts.begin(), ts.end());
    return ts[2];
}

// dynamic LDS that lets `waves` wavefronts (in workgroups of `threads`) stay on a compute unit; 0 = no cap
unsigned cap_lds(int waves, int threads)
{
    const int groups = waves / (threads / 64);
    return (waves >= 32 || groups < 1) ? 0u : kLdsPerCu / (unsigned)groups;
}

Ptrs g_p;
size_t g_bytes, g_vecs;

template <int R, int W, int U, bool NT>
double tiled(int threads, int waves)
{
    CK(hipFuncSetAttribute((const void*)stream<R, W, U, NT, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCu));
    const unsigned nb = (unsigned)(g_vecs / ((size_t)threads * U));
    const unsigned lds = cap_lds(waves, threads);
    const float ms = median_ms([&] { hipLaunchKernelGGL((stream<R, W, U, NT, false>), dim3(nb), dim3(threads), lds, 0, g_p, g_vecs); }, 20);
    return (double)g_bytes * (R + W) / ms / 1e6;
}

template <int R, int W>
void grid(const char* what)
{
    static const int kWaves[] = {8, 12, 16, 20, 24, 32};
    std::printf("\n%s: %d read + %d write streams, GB/s by workgroup size, tiles per wavefront (U) and cap on resident\n"
                "wavefronts per compute unit (32 = none)\n  threads U |", what, R, W);
    for (int w : kWaves) std::printf(" %6d", w);
    std::printf("\n");
    for (int threads : {64, 256}) {
        for (int u : {1, 2}) {
            std::printf("  %7d %d |", threads, u);
            for (int w : kWaves) {
                const double gbs = u == 1 ? tiled<R, W, 1, true>(threads, w) : tiled<R, W, 2, true>(threads, w);
                std::printf(" %6.0f", gbs);
                std::fflush(stdout);
            }
            std::printf("\n");
        }
    }
}

int main()
{
    g_bytes = (size_t)4 * 4096 * 14336 * 2;
    g_vecs = g_bytes / 16;
    for (int i = 0; i < 4; ++i) { void* a; CK(hipMalloc(&a, g_bytes)); CK(hipMemset(a, 1, g_bytes)); g_p.r[i] = (const u32x4*)a; }
    for (int i = 0; i < 4; ++i) { void* a; CK(hipMalloc(&a, g_bytes)); g_p.w[i] = (u32x4*)a; }
    int cus = 0; CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
    std::printf("%d compute units; %.1f MB per stream; non-temporal accesses unless stated\n", cus, g_bytes / 1e6);

    grid<1, 0>("read only");
    grid<0, 1>("write only");
    grid<1, 1>("copy / invact_fwd mix (mask aside)");
    grid<2, 1>("invact_bwd mix");
    grid<2, 2>("swiglu_invact_fwd mix");
    grid<3, 2>("swiglu_invact_bwd mix");

    std::printf("\nwithout the non-temporal hint (64 threads, U=1, cap 16 / none)\n");
    std::printf("  2r 2w  %6.0f %6.0f GB/s\n", tiled<2, 2, 1, false>(64, 16), tiled<2, 2, 1, false>(64, 32));
    std::printf("  3r 2w  %6.0f %6.0f GB/s\n", tiled<3, 2, 1, false>(64, 16), tiled<3, 2, 1, false>(64, 32));

    std::printf("\npersistent grid-stride loop instead of one tile per workgroup (64 threads, U=1)\n");
    for (int bpc : {8, 16, 32}) {
        const float a = median_ms([&] { hipLaunchKernelGGL((stream<2, 2, 1, true, true>), dim3(cus * bpc), dim3(64), 0, 0, g_p, g_vecs); }, 20);
        const float b = median_ms([&] { hipLaunchKernelGGL((stream<3, 2, 1, true, true>), dim3(cus * bpc), dim3(64), 0, 0, g_p, g_vecs); }, 20);
        std::printf("  %2d wavefronts per compute unit: 2r 2w %6.0f GB/s, 3r 2w %6.0f GB/s\n", bpc,
                    (double)g_bytes * 4 / a / 1e6, (double)g_bytes * 5 / b / 1e6);
    }

    std::printf("\nbinary32 layout: two vectors per lane and step (64 threads, no cap)\n");
#define PAIR(R, W, SPLIT) do { const unsigned nb = (unsigned)((g_vecs / 2 + 63) / 64); \
        const float ms = median_ms([&] { hipLaunchKernelGGL((stream_pair<R, W, SPLIT>), dim3(nb), dim3(64), 0, 0, g_p, g_vecs / 2); }, 20); \
        std::printf("  %dr %dw  %-32s %6.0f GB/s\n", R, W, SPLIT ? "2 x 16 B per lane, 1 KiB apart" : "32 B contiguous per lane", \
                    (double)g_bytes * (R + W) / ms / 1e6); std::fflush(stdout); } while (0)
    PAIR(1, 1, false); PAIR(1, 1, true); PAIR(3, 2, false); PAIR(3, 2, true);
    return 0;
}
