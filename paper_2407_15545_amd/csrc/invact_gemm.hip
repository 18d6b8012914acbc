// Sign-bit variant, the consumer (Section 3.3, "Sign-bit Inverted Activation", and its listing):
// the saved tensor Y_tagged = +-(f(x) - C) is not the activation, so whoever multiplies by the
// activation rebuilds |Y_tagged| + C first.  The listing does that inside the matrix products,
//     forward   out = (Y + C) W^T (+ bias)
//     backward  dW  = dOut^T (Y + C)
// and so do the two kernels here: bfloat16 MFMA GEMMs (gfx950, v_mfma_f32_32x32x16_bf16, binary32
// accumulation) whose loader of the activation operand applies |.| + C to every 16-byte piece on its way
// from global memory to LDS.  The decoded activation never exists in HBM: against invact_sbit_decode
// followed by a library GEMM that saves one read and one write of the activation per product.
//
// Shape of both kernels.  A workgroup of 256 threads (2 x 2 wavefronts) owns a 128 x 128 tile of the
// output; each wavefront a 64 x 64 quarter as 2 x 2 MFMA tiles of 32 x 32.  The contraction runs in steps
// of 64: both operand tiles (128 x 64 bfloat16 each) are loaded with coalesced 128-bit buffer loads into
// registers one step ahead, written to one of two LDS buffers (rows padded to 144 bytes, which spreads the
// 128-bit fragment reads over the banks), and one barrier per step separates the writer of a buffer from
// its readers.  Rows and columns outside the matrices are handled by the buffer extents (loads return 0,
// which the decode turns into C times an operand that is 0; the rows are never stored) and by a column
// test at the store.  Workgroup indices are remapped so that the workgroups an XCD receives (every
// eighth one) are neighbours in the output and share their operand tiles in that XCD's L2.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/invact.h"
#include "invact_constants.h"

namespace {

namespace cst = invact_const;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16   bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16   bf16x2 __attribute__((ext_vector_type(2)));
typedef float    f32x2 __attribute__((ext_vector_type(2)));
typedef float    f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTile = 128;              // output tile edge of a workgroup
constexpr int kStep = 64;               // contraction elements per step
constexpr int kRow = kStep + 8;         // LDS row in elements: 144 bytes
constexpr int kThreads = 256;
constexpr unsigned kLdsBytes = 2 /* buffers */ * 2 /* operands */ * kTile * kRow * 2;

template <int KIND> constexpr float min_of_kind()
{
    return KIND == INVACT_GELU_TANH ? cst::fT_gelu_tanh : KIND == INVACT_GELU_ERF ? cst::fT_gelu_erf : cst::fT_silu;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t whole_buffer(const void* p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi)          // round to nearest even (v_cvt_pk_bf16_f32)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// |y| + C on 8 bfloat16 values: the sum is formed in binary32 and rounded once to bfloat16, exactly as
// invact_sbit_decode forms it.
template <int KIND>
__device__ __forceinline__ u32x4 decode8(u32x4 v)
{
    constexpr float C = min_of_kind<KIND>();
    u32x4 out;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t w = v[j] & 0x7FFF7FFFu;
        out[j] = pack2(__uint_as_float(w << 16) + C, __uint_as_float(w & 0xFFFF0000u) + C);
    }
    return out;
}

// Consecutive workgroup indices land on different XCDs (eight of them).  Give XCD x the x-th eighth of the
// tiles instead, so that tiles which share an operand tile run on the same XCD.  Identity when the number of
// workgroups is not a multiple of 8.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned block, unsigned blocks)
{
    return (blocks % 8u) ? block : (block % 8u) * (blocks / 8u) + block / 8u;
}

// One contraction step of a wavefront: 4 sub-steps of 16, each reading two fragments of either operand
// (lane l: row l % 32 of the 32-row tile, elements 8 (l / 32) .. + 7 of the sub-step) and issuing 2 x 2 MFMAs.
// SWIZZLED: the 16-byte pieces of LDS row R sit at position (piece ^ (R / 8 % 8)), which is how the
// transposing loader of the weight-gradient kernel keeps its scattered writes off each other's banks
// (both wavefront offsets into a tile are multiples of 64 rows, so R / 8 % 8 is that of the row inside it).
template <bool SWIZZLED>
__device__ __forceinline__ void mfma_step(const uint16_t* a_tile, const uint16_t* b_tile, unsigned lane, f32x16 (&acc)[2][2])
{
    const unsigned row = lane & 31u, half = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < kStep / 16; ++kk) {
        bf16x8 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const unsigned R = i * 32 + row;
            const unsigned piece = SWIZZLED ? ((kk * 2 + half) ^ ((R >> 3) & 7u)) : (kk * 2 + half);
            a[i] = *reinterpret_cast<const bf16x8*>(a_tile + R * kRow + piece * 8u);
            b[i] = *reinterpret_cast<const bf16x8*>(b_tile + R * kRow + piece * 8u);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

// out[M][N] = (|y_tagged| + C)[M][K] * w[N][K]^T (+ bias[N]); every matrix row-major, bfloat16; K a multiple of 64.
template <int KIND>
__global__ __launch_bounds__(kThreads) void sbit_linear_kernel(const uint16_t* y_tagged, const uint16_t* w,
                                                               const uint16_t* bias, uint16_t* out,
                                                               unsigned M, unsigned N, unsigned K)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* const a_lds = lds;                                   // [2][kTile][kRow]
    uint16_t* const b_lds = lds + 2 * kTile * kRow;                // [2][kTile][kRow]

    const unsigned n_tiles = (N + kTile - 1) / kTile;
    const unsigned tile = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned m0 = (tile / n_tiles) * kTile, n0 = (tile % n_tiles) * kTile;   // neighbours share the rows of Y

    const unsigned t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const unsigned wm = (wave >> 1) * 64u, wn = (wave & 1u) * 64u;

    // loader: thread t moves the 16-byte piece `piece` of rows r, r + 32, r + 64, r + 96 of both operand tiles
    const unsigned r = t >> 3, piece = t & 7u;
    const __amdgpu_buffer_rsrc_t a_src = whole_buffer(y_tagged, M * K * 2u), b_src = whole_buffer(w, N * K * 2u);
    const unsigned a_off = ((m0 + r) * K + piece * 8u) * 2u, b_off = ((n0 + r) * K + piece * 8u) * 2u;
    const unsigned lds_off = r * kRow + piece * 8u;

    u32x4 ra[4], rb[4];
    auto load = [&](unsigned k0) {
#pragma unroll
        for (unsigned p = 0; p < 4; ++p) {
            // a row outside the matrix starts past the buffer's extent: the hardware returns 0
            const unsigned am = m0 + r + 32u * p, bn = n0 + r + 32u * p;
            ra[p] = __builtin_amdgcn_raw_buffer_load_b128(a_src, (int)(am < M ? a_off + (32u * p * K + k0) * 2u : 0xFFFFFFF0u), 0, 0);
            rb[p] = __builtin_amdgcn_raw_buffer_load_b128(b_src, (int)(bn < N ? b_off + (32u * p * K + k0) * 2u : 0xFFFFFFF0u), 0, 0);
        }
    };
    auto stage = [&](unsigned buf) {
#pragma unroll
        for (unsigned p = 0; p < 4; ++p) {
            *reinterpret_cast<u32x4*>(a_lds + buf * kTile * kRow + 32u * p * kRow + lds_off) = decode8<KIND>(ra[p]);
            *reinterpret_cast<u32x4*>(b_lds + buf * kTile * kRow + 32u * p * kRow + lds_off) = rb[p];
        }
    };

    f32x16 acc[2][2] = {};
    const unsigned steps = K / kStep;
    load(0);
    stage(0);
    __syncthreads();
    for (unsigned s = 0; s < steps; ++s) {
        const unsigned cur = s & 1u;
        if (s + 1 < steps) load((s + 1) * kStep);
        mfma_step<false>(a_lds + cur * kTile * kRow + wm * kRow, b_lds + cur * kTile * kRow + wn * kRow, lane, acc);
        if (s + 1 < steps) stage(cur ^ 1u);
        __syncthreads();
    }

    // MFMA result layout: register q of lane l holds row 8 (q / 4) + 4 (l / 32) + q % 4, column l % 32
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const unsigned col = n0 + wn + j * 32u + (lane & 31u);
        if (col >= N) continue;
        const float b = bias ? __uint_as_float((uint32_t)bias[col] << 16) : 0.0f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const unsigned row = m0 + wm + i * 32u + 8u * (q / 4) + 4u * (lane >> 5) + (q % 4);
                if (row < M) out[(size_t)row * N + col] = (uint16_t)(pack2(acc[i][j][q] + b, 0.0f) & 0xFFFFu);
            }
    }
}

// grad_w[N][K] = grad_out[M][N]^T * (|y_tagged| + C)[M][K]; every matrix row-major, bfloat16; M a multiple of 64,
// N and K multiples of 8.  The contraction index m is the slow one of both operands, so the loader transposes:
// a thread takes the same 16-byte piece (8 consecutive n, or k) of two neighbouring rows m, m + 1 and writes
// eight 32-bit words {row m, row m + 1} into LDS rows n .. n + 7 (k .. k + 7), whose 16-byte pieces are
// swizzled (see mfma_step).  From there on the kernel is the forward one: LDS rows are output rows / columns,
// their elements the contraction.
template <int KIND>
__global__ __launch_bounds__(kThreads) void sbit_linear_wgrad_kernel(const uint16_t* y_tagged, const uint16_t* grad_out,
                                                                     uint16_t* grad_w, unsigned M, unsigned N, unsigned K)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* const g_lds = lds;                                   // [2][kTile (n)][kRow (m)]
    uint16_t* const a_lds = lds + 2 * kTile * kRow;                // [2][kTile (k)][kRow (m)]

    const unsigned k_tiles = (K + kTile - 1) / kTile;
    const unsigned tile = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned n0 = (tile / k_tiles) * kTile, k0 = (tile % k_tiles) * kTile;   // neighbours share the columns of dOut

    const unsigned t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const unsigned wm = (wave >> 1) * 64u, wn = (wave & 1u) * 64u;

    // loader: thread t moves piece `piece` (8 columns) of rows 2 pair, 2 pair + 1 (+ 32) of both operand tiles
    const unsigned pair = t >> 4, piece = t & 15u;
    const __amdgpu_buffer_rsrc_t g_src = whole_buffer(grad_out, M * N * 2u), a_src = whole_buffer(y_tagged, M * K * 2u);
    const bool g_in = n0 + piece * 8u < N, a_in = k0 + piece * 8u < K;      // N and K are multiples of 8: a piece is in or out
    const unsigned g_off = (2u * pair * N + n0 + piece * 8u) * 2u, a_off = (2u * pair * K + k0 + piece * 8u) * 2u;

    u32x4 rg[2][2], ra[2][2];
    auto load = [&](unsigned m0) {
#pragma unroll
        for (unsigned p = 0; p < 2; ++p)
#pragma unroll
            for (unsigned h = 0; h < 2; ++h) {
                const unsigned m = m0 + 32u * p + h;
                rg[p][h] = __builtin_amdgcn_raw_buffer_load_b128(g_src, (int)(g_in ? g_off + m * N * 2u : 0xFFFFFFF0u), 0, 0);
                ra[p][h] = __builtin_amdgcn_raw_buffer_load_b128(a_src, (int)(a_in ? a_off + m * K * 2u : 0xFFFFFFF0u), 0, 0);
            }
    };
    // element e of both rows of a pair as one word: {row m in the low half, row m + 1 in the high half}
    auto pair_word = [](const u32x4& lo, const u32x4& hi, int e) {
        return __builtin_amdgcn_perm(hi[e / 2], lo[e / 2], (e & 1) ? 0x07060302u : 0x05040100u);
    };
    auto stage = [&](unsigned buf) {
#pragma unroll
        for (unsigned p = 0; p < 2; ++p) {
            const u32x4 a0 = decode8<KIND>(ra[p][0]), a1 = decode8<KIND>(ra[p][1]);
            const unsigned mloc = 2u * pair + 32u * p;                       // even: the word holds columns mloc, mloc + 1
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned R = piece * 8u + e;
                const unsigned col = ((((mloc >> 3) ^ (R >> 3)) & 7u) << 3) | (mloc & 7u);
                *reinterpret_cast<uint32_t*>(g_lds + buf * kTile * kRow + R * kRow + col) = pair_word(rg[p][0], rg[p][1], e);
                *reinterpret_cast<uint32_t*>(a_lds + buf * kTile * kRow + R * kRow + col) = pair_word(a0, a1, e);
            }
        }
    };

    f32x16 acc[2][2] = {};
    const unsigned steps = M / kStep;
    load(0);
    stage(0);
    __syncthreads();
    for (unsigned s = 0; s < steps; ++s) {
        const unsigned cur = s & 1u;
        if (s + 1 < steps) load((s + 1) * kStep);
        mfma_step<true>(g_lds + cur * kTile * kRow + wm * kRow, a_lds + cur * kTile * kRow + wn * kRow, lane, acc);
        if (s + 1 < steps) stage(cur ^ 1u);
        __syncthreads();
    }

#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const unsigned col = k0 + wn + j * 32u + (lane & 31u);
        if (col >= K) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const unsigned row = n0 + wm + i * 32u + 8u * (q / 4) + 4u * (lane >> 5) + (q % 4);
                if (row < N) grad_w[(size_t)row * K + col] = (uint16_t)(pack2(acc[i][j][q], 0.0f) & 0xFFFFu);
            }
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launches `kernel` over `tiles` workgroups with the LDS both kernels need (above the 64 KiB a kernel
// gets without asking: the runtime is told once per kernel and device).
template <auto kernel, class... Args>
int launch_tiles(size_t tiles, hipStream_t stream, Args... args)
{
    static std::atomic<uint64_t> prepared{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return INVACT_ERR_HIP;
    if (!(prepared.load(std::memory_order_acquire) >> dev & 1)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)kLdsBytes) != hipSuccess)
            return INVACT_ERR_HIP;
        prepared.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    }
    void* argv[] = {&args...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), dim3((unsigned)tiles), dim3(kThreads), argv, kLdsBytes,
                           stream) == hipSuccess ? INVACT_OK : INVACT_ERR_HIP;
}

constexpr size_t kMaxElems = size_t(1) << 31;      // 32-bit byte offsets inside each bfloat16 matrix

bool fits(size_t rows, size_t cols) { return cols == 0 || rows < kMaxElems / cols || rows * cols < kMaxElems; }

int check_kind_dtype(int kind, int dtype)
{
    if (kind != INVACT_GELU_TANH && kind != INVACT_GELU_ERF && kind != INVACT_SILU) return INVACT_ERR_KIND;
    return dtype == INVACT_BF16 ? INVACT_OK : INVACT_ERR_DTYPE;
}

}  // namespace

extern "C" int invact_sbit_linear_fwd(int kind, int dtype, const void* y_tagged, const void* weight, const void* bias,
                                      void* out, size_t M, size_t N, size_t K, hipStream_t stream)
{
    if (int e = check_kind_dtype(kind, dtype)) return e;
    if (K == 0 || K % kStep != 0 || !fits(M, K) || !fits(N, K) || !fits(M, N)) return INVACT_ERR_SIZE;
    if (M == 0 || N == 0) return INVACT_OK;
    if (!y_tagged || !weight || !out) return INVACT_ERR_NULL;
    if (!aligned16(y_tagged) || !aligned16(weight) || !aligned16(out) || (reinterpret_cast<uintptr_t>(bias) & 1u))
        return INVACT_ERR_ALIGN;
    const size_t tiles = ((M + kTile - 1) / kTile) * ((N + kTile - 1) / kTile);
    const uint16_t *a = static_cast<const uint16_t*>(y_tagged), *b = static_cast<const uint16_t*>(weight),
                   *c = static_cast<const uint16_t*>(bias);
    uint16_t* o = static_cast<uint16_t*>(out);
    const unsigned m = (unsigned)M, n = (unsigned)N, k = (unsigned)K;
    switch (kind) {
    case INVACT_GELU_TANH: return launch_tiles<sbit_linear_kernel<INVACT_GELU_TANH>>(tiles, stream, a, b, c, o, m, n, k);
    case INVACT_GELU_ERF:  return launch_tiles<sbit_linear_kernel<INVACT_GELU_ERF>>(tiles, stream, a, b, c, o, m, n, k);
    default:               return launch_tiles<sbit_linear_kernel<INVACT_SILU>>(tiles, stream, a, b, c, o, m, n, k);
    }
}

extern "C" int invact_sbit_linear_wgrad(int kind, int dtype, const void* y_tagged, const void* grad_out,
                                        void* grad_weight, size_t M, size_t N, size_t K, hipStream_t stream)
{
    if (int e = check_kind_dtype(kind, dtype)) return e;
    if (M == 0 || M % kStep != 0 || N % 8 != 0 || K % 8 != 0 || !fits(M, K) || !fits(N, K) || !fits(M, N))
        return INVACT_ERR_SIZE;
    if (N == 0 || K == 0) return INVACT_OK;
    if (!y_tagged || !grad_out || !grad_weight) return INVACT_ERR_NULL;
    if (!aligned16(y_tagged) || !aligned16(grad_out) || !aligned16(grad_weight)) return INVACT_ERR_ALIGN;
    const size_t tiles = ((N + kTile - 1) / kTile) * ((K + kTile - 1) / kTile);
    const uint16_t *a = static_cast<const uint16_t*>(y_tagged), *g = static_cast<const uint16_t*>(grad_out);
    uint16_t* o = static_cast<uint16_t*>(grad_weight);
    const unsigned m = (unsigned)M, n = (unsigned)N, k = (unsigned)K;
    switch (kind) {
    case INVACT_GELU_TANH: return launch_tiles<sbit_linear_wgrad_kernel<INVACT_GELU_TANH>>(tiles, stream, a, g, o, m, n, k);
    case INVACT_GELU_ERF:  return launch_tiles<sbit_linear_wgrad_kernel<INVACT_GELU_ERF>>(tiles, stream, a, g, o, m, n, k);
    default:               return launch_tiles<sbit_linear_wgrad_kernel<INVACT_SILU>>(tiles, stream, a, g, o, m, n, k);
    }
}
