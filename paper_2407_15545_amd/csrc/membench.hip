// Streaming ceiling of the machine: R read streams and W write streams of 128-bit
// accesses with no arithmetic, in the launch shapes the library's kernels use.
// The figures bound what any kernel with the same stream mix can reach; the
// library's kernels are compared against them, not only against the 8 TB/s
// data-sheet peak.
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

template <bool NT> __device__ __forceinline__ u32x4 ld(const u32x4* p) { return NT ? __builtin_nontemporal_load(p) : *p; }
template <bool NT> __device__ __forceinline__ void st(u32x4* p, u32x4 v) { if (NT) __builtin_nontemporal_store(v, p); else *p = v; }

// One tile of U * 256 vectors per workgroup (PERSISTENT = false) or a grid-stride loop.
// SPLIT: a lane's two accesses of a step are 1 KiB apart (each coalesced) instead of adjacent (32 B per lane).
template <int R, int W, int U, bool NT, bool PERSISTENT>
__global__ __launch_bounds__(256) void stream(Ptrs p, size_t vecs)
{
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
        const size_t stride = (size_t)gridDim.x * 256;
        for (size_t c = (size_t)blockIdx.x * 256 + threadIdx.x; c + (U - 1) * stride < vecs; c += U * stride) body(c, stride);
    } else {
        const size_t c = (size_t)blockIdx.x * 256 * U + threadIdx.x;
        if (c + (U - 1) * 256 < vecs) body(c, 256);
    }
}

// binary32-style access: two vectors per lane and step, adjacent (32 B per lane) or split (1 KiB apart)
template <int R, int W, bool SPLIT>
__global__ __launch_bounds__(256) void stream_pair(Ptrs p, size_t pairs)
{
    const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
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
    std::sort(ts.begin(), ts.end());
    return ts[2];
}

int main()
{
    const size_t bytes = (size_t)4 * 4096 * 14336 * 2, vecs = bytes / 16;
    Ptrs p;
    for (int i = 0; i < 4; ++i) { void* a; CK(hipMalloc(&a, bytes)); CK(hipMemset(a, 1, bytes)); p.r[i] = (const u32x4*)a; }
    for (int i = 0; i < 4; ++i) { void* a; CK(hipMalloc(&a, bytes)); p.w[i] = (u32x4*)a; }
    int cus = 0; CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
    std::printf("%d compute units; %.1f MB per stream\n", cus, bytes / 1e6);

#define TILED(R, W, U, NT, what) do { unsigned nb = (unsigned)(vecs / (256 * U)); \
        float ms = median_ms([&] { hipLaunchKernelGGL((stream<R, W, U, NT, false>), dim3(nb), dim3(256), 0, 0, p, vecs); }, 20); \
        std::printf("%-34s %dr %dw  tiled U=%d nt=%d          %8.4f ms %6.0f GB/s\n", what, R, W, U, (int)NT, ms, (double)bytes * (R + W) / ms / 1e6); std::fflush(stdout); } while (0)
#define PERS(R, W, U, NT, BPC, what) do { \
        float ms = median_ms([&] { hipLaunchKernelGGL((stream<R, W, U, NT, true>), dim3(cus * BPC), dim3(256), 0, 0, p, vecs); }, 20); \
        std::printf("%-34s %dr %dw  persistent U=%d nt=%d bpc=%-2d %8.4f ms %6.0f GB/s\n", what, R, W, U, (int)NT, BPC, ms, (double)bytes * (R + W) / ms / 1e6); std::fflush(stdout); } while (0)
#define PAIR(R, W, SPLIT, what) do { unsigned nb = (unsigned)((vecs / 2 + 255) / 256); \
        float ms = median_ms([&] { hipLaunchKernelGGL((stream_pair<R, W, SPLIT>), dim3(nb), dim3(256), 0, 0, p, vecs / 2); }, 20); \
        std::printf("%-34s %dr %dw  %-28s %8.4f ms %6.0f GB/s\n", what, R, W, SPLIT ? "2 x 16 B per lane, 1 KiB apart" : "32 B contiguous per lane", ms, (double)bytes * (R + W) / ms / 1e6); std::fflush(stdout); } while (0)

    TILED(1, 0, 1, true,  "read only");
    TILED(0, 1, 1, true,  "write only");
    TILED(1, 1, 1, false, "copy");
    TILED(1, 1, 1, true,  "copy");
    TILED(1, 1, 2, true,  "invact_fwd mix (mask aside)");
    TILED(2, 1, 2, true,  "invact_bwd mix");
    TILED(2, 2, 2, false, "swiglu_invact_fwd mix");
    TILED(2, 2, 2, true,  "swiglu_invact_fwd mix");
    TILED(2, 2, 4, true,  "swiglu_invact_fwd mix");
    TILED(3, 2, 2, false, "swiglu_invact_bwd mix");
    TILED(3, 2, 2, true,  "swiglu_invact_bwd mix");
    TILED(3, 2, 1, true,  "swiglu_invact_bwd mix");
    PERS(2, 2, 2, true, 1, "swiglu_invact_fwd mix");
    PERS(2, 2, 2, true, 2, "swiglu_invact_fwd mix");
    PERS(2, 2, 2, true, 4, "swiglu_invact_fwd mix");
    PERS(2, 2, 2, true, 8, "swiglu_invact_fwd mix");
    PERS(3, 2, 2, true, 1, "swiglu_invact_bwd mix");
    PERS(3, 2, 2, true, 8, "swiglu_invact_bwd mix");
    PAIR(1, 1, false, "binary32 layout, copy");
    PAIR(1, 1, true,  "binary32 layout, copy");
    PAIR(3, 2, false, "binary32 layout, bwd mix");
    PAIR(3, 2, true,  "binary32 layout, bwd mix");
    return 0;
}
