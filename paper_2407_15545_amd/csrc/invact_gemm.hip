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

constexpr int kStep = 64;               // contraction elements per step
constexpr int kRow = kStep + 8;         // LDS row in elements: 144 bytes

// Shape of a workgroup: WM x WN wavefronts, each owning TM x TN MFMA tiles of 32 x 32.
//   Large  256 x 256 output tile, 8 wavefronts of 128 x 64: 147 KB of LDS, one workgroup per compute unit, two
//          wavefronts per SIMD.  Every operand element staged in LDS feeds 256 output columns (rows), which
//          matters here because the activation operand pays for its decode on the way in.
//   Small  128 x 128, 4 wavefronts of 64 x 64, two workgroups per compute unit: for outputs too small to give
//          every compute unit a large tile.
template <int TM_, int TN_, int WM_, int WN_> struct Shape {
    static constexpr int TM = TM_, TN = TN_, WM = WM_, WN = WN_;
    static constexpr int kThreads = 64 * WM * WN;
    static constexpr int kTileM = 32 * TM * WM, kTileN = 32 * TN * WN;      // rows of the two operand tiles
    static constexpr unsigned kLdsBytes = 2 /* buffers */ * (kTileM + kTileN) * kRow * 2;
};
using Large = Shape<4, 2, 2, 4>;
using Small = Shape<2, 2, 2, 2>;

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
// (a wavefront's offset into a tile is a multiple of 64 rows, so R / 8 % 8 is that of the row inside its part).
template <bool SWIZZLED, int TM, int TN>
__device__ __forceinline__ void mfma_step(const uint16_t* a_tile, const uint16_t* b_tile, unsigned lane, f32x16 (&acc)[TM][TN])
{
    const unsigned row = lane & 31u, half = lane >> 5;
    auto fragment = [&](const uint16_t* tile, int i, int kk) {
        const unsigned R = i * 32 + row;
        const unsigned piece = SWIZZLED ? ((kk * 2 + half) ^ ((R >> 3) & 7u)) : (kk * 2 + half);
        return *reinterpret_cast<const bf16x8*>(tile + R * kRow + piece * 8u);
    };
#pragma unroll
    for (int kk = 0; kk < kStep / 16; ++kk) {
        bf16x8 a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = fragment(a_tile, i, kk);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = fragment(b_tile, j, kk);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

// out[M][N] = (|y_tagged| + C)[M][K] * w[N][K]^T (+ bias[N]); every matrix row-major, bfloat16; K a multiple of 64.
template <int KIND, class S>
__global__ __launch_bounds__(S::kThreads) void sbit_linear_kernel(const uint16_t* y_tagged, const uint16_t* w,
                                                                  const uint16_t* bias, uint16_t* out,
                                                                  unsigned M, unsigned N, unsigned K)
{
    constexpr unsigned kRowsPerPass = S::kThreads / 8;          // 8 threads move one 128-byte operand row
    constexpr unsigned kPassesA = S::kTileM / kRowsPerPass, kPassesB = S::kTileN / kRowsPerPass;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* const a_lds = lds;                                   // [2][kTileM][kRow]
    uint16_t* const b_lds = lds + 2 * S::kTileM * kRow;            // [2][kTileN][kRow]

    const unsigned n_tiles = (N + S::kTileN - 1) / S::kTileN;
    const unsigned tile = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned m0 = (tile / n_tiles) * S::kTileM, n0 = (tile % n_tiles) * S::kTileN;   // neighbours share the rows of Y

    const unsigned t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const unsigned wm = (wave / S::WN) * (32 * S::TM), wn = (wave % S::WN) * (32 * S::TN);

    // loader: thread t moves the 16-byte piece `piece` of rows r, r + kRowsPerPass, ... of both operand tiles
    const unsigned r = t >> 3, piece = t & 7u;
    const __amdgpu_buffer_rsrc_t a_src = whole_buffer(y_tagged, M * K * 2u), b_src = whole_buffer(w, N * K * 2u);
    const unsigned a_off = ((m0 + r) * K + piece * 8u) * 2u, b_off = ((n0 + r) * K + piece * 8u) * 2u;
    const unsigned lds_off = r * kRow + piece * 8u;

    u32x4 ra[kPassesA], rb[kPassesB];
    auto load = [&](unsigned k0) {
        // a row outside the matrix is addressed past the buffer's extent: the hardware returns 0
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p)
            ra[p] = __builtin_amdgcn_raw_buffer_load_b128(
                a_src, (int)(m0 + r + kRowsPerPass * p < M ? a_off + (kRowsPerPass * p * K + k0) * 2u : 0xFFFFFFF0u), 0, 0);
#pragma unroll
        for (unsigned p = 0; p < kPassesB; ++p)
            rb[p] = __builtin_amdgcn_raw_buffer_load_b128(
                b_src, (int)(n0 + r + kRowsPerPass * p < N ? b_off + (kRowsPerPass * p * K + k0) * 2u : 0xFFFFFFF0u), 0, 0);
    };
    auto stage = [&](unsigned buf) {
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p)
            *reinterpret_cast<u32x4*>(a_lds + buf * S::kTileM * kRow + kRowsPerPass * p * kRow + lds_off) = decode8<KIND>(ra[p]);
#pragma unroll
        for (unsigned p = 0; p < kPassesB; ++p)
            *reinterpret_cast<u32x4*>(b_lds + buf * S::kTileN * kRow + kRowsPerPass * p * kRow + lds_off) = rb[p];
    };

    f32x16 acc[S::TM][S::TN] = {};
    const unsigned steps = K / kStep;
    load(0);
    stage(0);
    __syncthreads();
    for (unsigned s = 0; s < steps; ++s) {
        const unsigned cur = s & 1u;
        if (s + 1 < steps) load((s + 1) * kStep);
        mfma_step<false, S::TM, S::TN>(a_lds + cur * S::kTileM * kRow + wm * kRow, b_lds + cur * S::kTileN * kRow + wn * kRow,
                                       lane, acc);
        if (s + 1 < steps) stage(cur ^ 1u);
        __syncthreads();
    }

    // MFMA result layout: register q of lane l holds row 8 (q / 4) + 4 (l / 32) + q % 4, column l % 32
#pragma unroll
    for (int j = 0; j < S::TN; ++j) {
        const unsigned col = n0 + wn + j * 32u + (lane & 31u);
        if (col >= N) continue;
        const float b = bias ? __uint_as_float((uint32_t)bias[col] << 16) : 0.0f;
#pragma unroll
        for (int i = 0; i < S::TM; ++i)
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
template <int KIND, class S>
__global__ __launch_bounds__(S::kThreads) void sbit_linear_wgrad_kernel(const uint16_t* y_tagged, const uint16_t* grad_out,
                                                                        uint16_t* grad_w, unsigned M, unsigned N, unsigned K)
{
    // per operand: 16-byte pieces per row, row pairs one pass of all threads covers, passes per step
    constexpr unsigned kPiecesG = S::kTileM / 8, kPairsG = S::kThreads / kPiecesG, kPassesG = kStep / (2 * kPairsG);
    constexpr unsigned kPiecesA = S::kTileN / 8, kPairsA = S::kThreads / kPiecesA, kPassesA = kStep / (2 * kPairsA);
    static_assert(kPassesG * 2 * kPairsG == kStep && kPassesA * 2 * kPairsA == kStep, "a step is a whole number of passes");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* const g_lds = lds;                                   // [2][kTileM (n)][kRow (m)]
    uint16_t* const a_lds = lds + 2 * S::kTileM * kRow;            // [2][kTileN (k)][kRow (m)]

    const unsigned k_tiles = (K + S::kTileN - 1) / S::kTileN;
    const unsigned tile = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned n0 = (tile / k_tiles) * S::kTileM, k0 = (tile % k_tiles) * S::kTileN;   // neighbours share the columns of dOut

    const unsigned t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const unsigned wm = (wave / S::WN) * (32 * S::TM), wn = (wave % S::WN) * (32 * S::TN);

    // loader: thread t moves one piece (8 columns) of rows 2 pair, 2 pair + 1 (+ 2 kPairs, ...) of either operand tile.
    // A wavefront takes 16 neighbouring pieces of 4 neighbouring row pairs: its 64 scattered 32-bit LDS writes
    // (one element index e at a time) then fall on all 32 banks twice over, which is as good as 256 bytes get.
    const unsigned pair_g = (wave / (kPiecesG / 16)) * 4u + (lane >> 4), piece_g = (lane & 15u) + 16u * (wave % (kPiecesG / 16));
    const unsigned pair_a = (wave / (kPiecesA / 16)) * 4u + (lane >> 4), piece_a = (lane & 15u) + 16u * (wave % (kPiecesA / 16));
    const __amdgpu_buffer_rsrc_t g_src = whole_buffer(grad_out, M * N * 2u), a_src = whole_buffer(y_tagged, M * K * 2u);
    const bool g_in = n0 + piece_g * 8u < N, a_in = k0 + piece_a * 8u < K;  // N and K are multiples of 8: a piece is in or out
    const unsigned g_off = (2u * pair_g * N + n0 + piece_g * 8u) * 2u, a_off = (2u * pair_a * K + k0 + piece_a * 8u) * 2u;

    u32x4 rg[kPassesG][2], ra[kPassesA][2];
    auto load = [&](unsigned m0) {
#pragma unroll
        for (unsigned p = 0; p < kPassesG; ++p)
#pragma unroll
            for (unsigned h = 0; h < 2; ++h)
                rg[p][h] = __builtin_amdgcn_raw_buffer_load_b128(
                    g_src, (int)(g_in ? g_off + (m0 + 2u * kPairsG * p + h) * N * 2u : 0xFFFFFFF0u), 0, 0);
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p)
#pragma unroll
            for (unsigned h = 0; h < 2; ++h)
                ra[p][h] = __builtin_amdgcn_raw_buffer_load_b128(
                    a_src, (int)(a_in ? a_off + (m0 + 2u * kPairsA * p + h) * K * 2u : 0xFFFFFFF0u), 0, 0);
    };
    // Writes the 8 elements of both rows of a pair, as words {row m in the low half, row m + 1 in the high half},
    // into LDS rows 8 piece .. 8 piece + 7 at (swizzled) column mloc.
    auto scatter = [](uint16_t* tile, const u32x4& lo, const u32x4& hi, unsigned piece, unsigned mloc) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const unsigned R = piece * 8u + e;
            const unsigned col = ((((mloc >> 3) ^ (R >> 3)) & 7u) << 3) | (mloc & 7u);
            *reinterpret_cast<uint32_t*>(tile + R * kRow + col) =
                __builtin_amdgcn_perm(hi[e / 2], lo[e / 2], (e & 1) ? 0x07060302u : 0x05040100u);
        }
    };
    auto stage = [&](unsigned buf) {
#pragma unroll
        for (unsigned p = 0; p < kPassesG; ++p)
            scatter(g_lds + buf * S::kTileM * kRow, rg[p][0], rg[p][1], piece_g, 2u * pair_g + 2u * kPairsG * p);
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p)
            scatter(a_lds + buf * S::kTileN * kRow, decode8<KIND>(ra[p][0]), decode8<KIND>(ra[p][1]), piece_a,
                    2u * pair_a + 2u * kPairsA * p);
    };

    f32x16 acc[S::TM][S::TN] = {};
    const unsigned steps = M / kStep;
    load(0);
    stage(0);
    __syncthreads();
    for (unsigned s = 0; s < steps; ++s) {
        const unsigned cur = s & 1u;
        if (s + 1 < steps) load((s + 1) * kStep);
        mfma_step<true, S::TM, S::TN>(g_lds + cur * S::kTileM * kRow + wm * kRow, a_lds + cur * S::kTileN * kRow + wn * kRow,
                                      lane, acc);
        if (s + 1 < steps) stage(cur ^ 1u);
        __syncthreads();
    }

#pragma unroll
    for (int j = 0; j < S::TN; ++j) {
        const unsigned col = k0 + wn + j * 32u + (lane & 31u);
        if (col >= K) continue;
#pragma unroll
        for (int i = 0; i < S::TM; ++i)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const unsigned row = n0 + wm + i * 32u + 8u * (q / 4) + 4u * (lane >> 5) + (q % 4);
                if (row < N) grad_w[(size_t)row * K + col] = (uint16_t)(pack2(acc[i][j][q], 0.0f) & 0xFFFFu);
            }
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launches `kernel` over `tiles` workgroups of shape S (its LDS is above the 64 KiB a kernel gets without
// asking: the runtime is told once per kernel and device).
template <auto kernel, class S, class... Args>
int launch_tiles(size_t tiles, hipStream_t stream, Args... args)
{
    static std::atomic<uint64_t> prepared{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return INVACT_ERR_HIP;
    if (!(prepared.load(std::memory_order_acquire) >> dev & 1)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)S::kLdsBytes) != hipSuccess)
            return INVACT_ERR_HIP;
        prepared.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    }
    void* argv[] = {&args...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), dim3((unsigned)tiles), dim3(S::kThreads), argv,
                           S::kLdsBytes, stream) == hipSuccess ? INVACT_OK : INVACT_ERR_HIP;
}

template <class S> size_t tiles_of(size_t rows, size_t cols)
{
    return ((rows + S::kTileM - 1) / S::kTileM) * ((cols + S::kTileN - 1) / S::kTileN);
}

// The large tile where it still gives every compute unit a workgroup (256 of them), the small one otherwise.
std::atomic<int> g_force_tile{0};                       // 0: choose; 2: small; 4: large (benchmarking)
bool large_tile(size_t rows, size_t cols)
{
    const int forced = g_force_tile.load(std::memory_order_relaxed);
    return forced ? forced == 4 : tiles_of<Large>(rows, cols) >= 256;
}

template <int KIND>
int run_linear(const uint16_t* a, const uint16_t* b, const uint16_t* c, uint16_t* o, unsigned m, unsigned n, unsigned k,
               hipStream_t stream)
{
    if (large_tile(m, n))
        return launch_tiles<sbit_linear_kernel<KIND, Large>, Large>(tiles_of<Large>(m, n), stream, a, b, c, o, m, n, k);
    return launch_tiles<sbit_linear_kernel<KIND, Small>, Small>(tiles_of<Small>(m, n), stream, a, b, c, o, m, n, k);
}

template <int KIND>
int run_wgrad(const uint16_t* a, const uint16_t* g, uint16_t* o, unsigned m, unsigned n, unsigned k, hipStream_t stream)
{
    if (large_tile(n, k))
        return launch_tiles<sbit_linear_wgrad_kernel<KIND, Large>, Large>(tiles_of<Large>(n, k), stream, a, g, o, m, n, k);
    return launch_tiles<sbit_linear_wgrad_kernel<KIND, Small>, Small>(tiles_of<Small>(n, k), stream, a, g, o, m, n, k);
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
    const uint16_t *a = static_cast<const uint16_t*>(y_tagged), *b = static_cast<const uint16_t*>(weight),
                   *c = static_cast<const uint16_t*>(bias);
    uint16_t* o = static_cast<uint16_t*>(out);
    const unsigned m = (unsigned)M, n = (unsigned)N, k = (unsigned)K;
    switch (kind) {
    case INVACT_GELU_TANH: return run_linear<INVACT_GELU_TANH>(a, b, c, o, m, n, k, stream);
    case INVACT_GELU_ERF:  return run_linear<INVACT_GELU_ERF>(a, b, c, o, m, n, k, stream);
    default:               return run_linear<INVACT_SILU>(a, b, c, o, m, n, k, stream);
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
    const uint16_t *a = static_cast<const uint16_t*>(y_tagged), *g = static_cast<const uint16_t*>(grad_out);
    uint16_t* o = static_cast<uint16_t*>(grad_weight);
    const unsigned m = (unsigned)M, n = (unsigned)N, k = (unsigned)K;
    switch (kind) {
    case INVACT_GELU_TANH: return run_wgrad<INVACT_GELU_TANH>(a, g, o, m, n, k, stream);
    case INVACT_GELU_ERF:  return run_wgrad<INVACT_GELU_ERF>(a, g, o, m, n, k, stream);
    default:               return run_wgrad<INVACT_SILU>(a, g, o, m, n, k, stream);
    }
}

// Benchmarking: 0 lets the library choose the tile of the two products above, 2 or 4 forces T (results are the
// same up to the order of the binary32 sums).  Returns its argument, or -1 if it is none of these.
extern "C" int invact_set_linear_tile(int t)
{
    if (t != 0 && t != 2 && t != 4) return -1;
    g_force_tile.store(t, std::memory_order_relaxed);
    return t;
}
