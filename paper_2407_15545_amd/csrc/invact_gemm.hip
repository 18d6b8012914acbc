// Sign-bit variant, the consumer (Section 3.3, "Sign-bit Inverted Activation", and its listing):
// the saved tensor Y_tagged = +-(f(x) - C) is not the activation, so whoever multiplies by the
// activation rebuilds |Y_tagged| + C first.  The listing does that inside the matrix products,
//     forward   out = (Y + C) W^T (+ bias)
//     backward  dW  = dOut^T (Y + C)
//               dX  = (dOut W) * f'(f^-1(Y + C, S))
// and so do the first two kernels here: bfloat16 MFMA GEMMs (gfx950, v_mfma_f32_32x32x16_bf16, binary32
// accumulation) whose loader of the activation operand applies |.| + C to every 16-byte piece on its way
// from global memory to LDS.  The decoded activation never exists in HBM: against invact_sbit_decode
// followed by a library GEMM that saves one read and one write of the activation per product.  The third
// product has nothing to decode on the way in; it multiplies its accumulators by q(|Y_tagged| + C, S) on the way
// out, which saves the write and the read of dOut W that a library GEMM followed by invact_sbit_bwd costs.
//
// Shape of the three kernels.  A workgroup owns a tile of the output (256 x 256 with 8 wavefronts of 128 x 64, or
// one of the other shapes below); each wavefront a block of TM x TN MFMA tiles of 32 x 32.  The contraction
// runs in steps of 64 as a software pipeline of depth two (see contract): operand tiles travel global memory
// -> registers -> (decode) -> one of two LDS buffers -> MFMA fragments, and the work of all four stages is
// spread between the MFMAs of a step.  Rows and columns outside the matrices are handled by the buffer
// extents (loads return 0, stores are dropped).  Workgroup indices are remapped so that the workgroups an XCD
// receives (every eighth one) are neighbours in the output and share their operand tiles in that XCD's L2.
// The weight gradient can also split its contraction over a grid of splits x tiles workgroups, which leave
// binary32 partial tiles in a workspace (the caller's, or a static device array) for a small summing kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <utility>

#include "../../include/invact.h"
#include "invact_constants.h"
#include "invact_math.h"

namespace {

namespace cst = invact_const;

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16   bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16   bf16x2 __attribute__((ext_vector_type(2)));
typedef float    f32x2 __attribute__((ext_vector_type(2)));
typedef float    f32x4 __attribute__((ext_vector_type(4)));
typedef float    f32x16 __attribute__((ext_vector_type(16)));

constexpr int kStep = 64;               // contraction elements per step
constexpr int kRow = kStep + 8;         // LDS row in elements: 144 bytes

// Shape of a workgroup: WM x WN wavefronts, each owning TM x TN MFMA tiles of 32 x 32.
//   Large  256 x 256 output tile, 8 wavefronts of 128 x 64: 147 KB of LDS, one workgroup per compute unit, two
//          wavefronts per SIMD.  Every operand element staged in LDS feeds 256 output columns (rows), which
//          matters here because the activation operand pays for its decode on the way in.
//   Small  128 x 128, 4 wavefronts of 64 x 64, two workgroups per compute unit: for outputs too small to give
//          every compute unit a large tile.
//   Small8 the same tile with 8 wavefronts of 64 x 32: for outputs that give a compute unit one such tile at most.
template <int TM_, int TN_, int WM_, int WN_> struct Shape {
    static constexpr int TM = TM_, TN = TN_, WM = WM_, WN = WN_;
    static constexpr int kThreads = 64 * WM * WN;
    static constexpr int kTileM = 32 * TM * WM, kTileN = 32 * TN * WN;      // rows of the two operand tiles
    static constexpr unsigned kOperandBytes = 2 /* buffers */ * (kTileM + kTileN) * kRow * 2;
    static constexpr unsigned kStagingBytes = WM * WN * (32 * TM) * (32 * TN + 8) * 2;      // the output, on its way out
    static_assert(kStagingBytes <= kOperandBytes, "the output is staged in the operand buffers");
    static constexpr unsigned kLdsBytes = kOperandBytes + kTileN * 4;                       // and the bias behind them
};
using Large = Shape<4, 2, 2, 4>;
using Small = Shape<2, 2, 2, 2>;
using Small8 = Shape<2, 1, 2, 4>;

template <int KIND> constexpr float min_of_kind()
{
    return KIND == INVACT_GELU_TANH ? cst::fT_gelu_tanh : KIND == INVACT_GELU_ERF ? cst::fT_gelu_erf : cst::fT_silu;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t whole_buffer(const void* p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

constexpr unsigned kOutside = 0xFFFFFFF0u;      // a byte offset past the extent of every buffer here

__device__ __forceinline__ uint32_t pack2(float lo, float hi)          // round to nearest even (v_cvt_pk_bf16_f32)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// |y| + C on two (eight) bfloat16 values: the sum is formed in binary32 and rounded once to bfloat16, exactly as
// invact_sbit_decode forms it.
template <int KIND>
__device__ __forceinline__ uint32_t decode2(uint32_t v)
{
    constexpr float C = min_of_kind<KIND>();
    return pack2(__builtin_fabsf(__uint_as_float(v << 16)) + C, __builtin_fabsf(__uint_as_float(v & 0xFFFF0000u)) + C);
}
template <int KIND>
__device__ __forceinline__ u32x4 decode8(u32x4 v)
{
    return u32x4{decode2<KIND>(v[0]), decode2<KIND>(v[1]), decode2<KIND>(v[2]), decode2<KIND>(v[3])};
}

// Consecutive workgroup indices land on different XCDs (eight of them).  Give XCD x the x-th eighth of the
// tiles instead, so that tiles which share an operand tile run on the same XCD.  Identity when the number of
// workgroups is not a multiple of 8.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned block, unsigned blocks)
{
    return (blocks % 8u) ? block : (block % 8u) * (blocks / 8u) + block / 8u;
}

// Row and column of tile `tile` of a rows x cols grid of tiles, walked in bands of kBand rows, column by column
// inside a band: the 32 tiles an XCD works on at a time then form a block of kBand x (32 / kBand) tiles and
// share kBand + 32 / kBand operand panels, where a row-major walk would have them share 1 + 32.
constexpr unsigned kBand = 4;      // 4 and 8 measure alike, 2 and 16 a few per cent lower
struct TileAt { unsigned row, col; };
__device__ __forceinline__ TileAt banded(unsigned tile, unsigned rows, unsigned cols)
{
    const unsigned band = tile / (kBand * cols), within = tile % (kBand * cols);
    const unsigned height = rows - band * kBand < kBand ? rows - band * kBand : kBand;      // the last band may be lower
    return TileAt{band * kBand + within % height, within / height};
}

// Compile-time loops: f(std::integral_constant<int, FIRST>) ... f(std::integral_constant<int, LAST - 1>).
template <int FIRST, int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f)
{
    (f(std::integral_constant<int, FIRST + Is>{}), ...);
}
template <int FIRST, int LAST, class F> __device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (LAST > FIRST) static_for_impl<FIRST>(std::make_integer_sequence<int, LAST - FIRST>{}, f);
}
// The I-th of N equal shares of COUNT items: [share_begin, share_end).
template <int I, int N, int COUNT> constexpr int share_begin = I * COUNT / N;
template <int I, int N, int COUNT> constexpr int share_end = (I + 1) * COUNT / N;

// The contraction loop of both products.  LDS holds two buffers of either operand tile ([rows][kRow], a row is
// a row or column of the output, its elements one step of the contraction); a wavefront accumulates
// acc[i][j] += B-tile j x A-tile i (the MFMA gets the column operand first: see store_accumulators).
//
// A software pipeline of depth two.  During step s a wavefront
//   * multiplies out of buffer s % 2, reading the fragments of sub-step kk + 1 (of four) while the MFMAs of kk run,
//   * writes the operand tiles of step s + 1, which its registers hold since step s - 1, into the other buffer,
//   * and loads the tiles of step s + 2 into the registers this frees, piece by piece, so that every load has a
//     whole step to arrive.
// The loader supplies the last two as tasks: kTasks0, kTasks1, kTasks2 of them for the first three sub-steps,
// task<KK, T>(a_next, b_next, s + 2).  After each MFMA comes its share of the sub-step's other work, and the
// compiler is kept from moving anything across (left alone it gathers the MFMAs, and the matrix unit idles
// while the wavefront decodes and stages).  One barrier per step, before the last sub-step: by then every
// wavefront has read all of buffer s % 2 and written all of the other one, and the last sub-step fetches the
// first fragments of step s + 1.  The steps past the end of the contraction that the pipeline's tail asks for
// are reloads of the last one and are never multiplied.
//
// Two LDS layouts, chosen per operand.  Plain: [rows of the tile][kRow], the elements of a row one step of the contraction; a
// fragment is one 128-bit read per lane (lane l: row l % 32, elements 16 kk + 8 (l / 32) .. + 7).  TRANSPOSED (an
// operand that has the contraction index as its slow one: both of the weight gradient, the weight of the input gradient): [step of the contraction = 64
// rows][rows of the tile + kPadT], as the tiles lie in memory; a fragment is two ds_read_b64_tr_b16 per lane.
// That instruction transposes inside every group of 16 lanes: lane i of a group receives, as its element j, element
// i % 4 of the 8 bytes lane i / 4 + 4 j of the group points at.  So lane r of a group points at contraction row
// 4 t + r / 4 (t = 0, 1: the two reads), tile rows 4 (r % 4) .. + 3 of the group's 16, and lane i ends up with
// contraction rows 4 t .. 4 t + 3 of its own tile row: the 8 consecutive ones an MFMA operand wants.
constexpr unsigned kPadT = 16;          // elements: 4 contraction rows of 32 bytes each then fill all 32 banks once (8: 10 % slower; 24 and, for the large tile, 32: no faster, although 32 takes the remaining bank conflicts away)

template <class S, bool TRANSPOSED_A, bool TRANSPOSED_B, class Loader>
__device__ __forceinline__ void contract(uint16_t* lds, unsigned steps, unsigned wm, unsigned wn, unsigned lane, Loader& loader,
                                         f32x16 (&acc)[S::TM][S::TN])
{
    constexpr unsigned kPitchA = S::kTileM + kPadT, kPitchB = S::kTileN + kPadT;   // TRANSPOSED: elements of an LDS row
    constexpr unsigned kBufA = TRANSPOSED_A ? kStep * kPitchA : S::kTileM * kRow;  // elements of one buffer
    constexpr unsigned kBufB = TRANSPOSED_B ? kStep * kPitchB : S::kTileN * kRow;
    static_assert(2 * (kBufA + kBufB) * 2 <= S::kOperandBytes, "both layouts fit the operand buffers");
    constexpr int kMfmas = S::TM * S::TN, kFrags = S::TM + S::TN;
    static_assert(kStep == 64, "four sub-steps");
    uint16_t *a_cur = lds, *a_nxt = lds + kBufA, *b_cur = lds + 2 * kBufA, *b_nxt = lds + 2 * kBufA + kBufB;

    // fragments, in the order the MFMAs of a sub-step first need them: A 0, B 0 .. TN - 1, A 1 .. TM - 1
    const unsigned row = lane & 31u, half = lane >> 5;
    const unsigned tr_row = 8u * half + ((lane & 15u) >> 2), tr_col = 16u * ((lane >> 4) & 1u) + 4u * (lane & 3u);
    bf16x8 fa[2][S::TM], fb[2][S::TN];
    auto fragment = [&](auto set_c, auto f_c, const uint16_t* a_buf, const uint16_t* b_buf, unsigned kk) {
        constexpr int set = decltype(set_c)::value, f = decltype(f_c)::value;
        constexpr bool of_a = f == 0 || f > S::TN;
        constexpr int index = f == 0 ? 0 : of_a ? f - S::TN : f - 1;
        bf16x8 v;
        if constexpr (of_a ? TRANSPOSED_A : TRANSPOSED_B) {
            typedef short short4_t __attribute__((ext_vector_type(4)));
            typedef __attribute__((address_space(3))) short4_t lds_short4_t;
            constexpr unsigned pitch = of_a ? kPitchA : kPitchB;
            const uint16_t* at = (of_a ? a_buf : b_buf) + (16u * kk + tr_row) * pitch + (of_a ? wm : wn) + index * 32 + tr_col;
            const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)at);
            const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(at + 4u * pitch));
            v = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
            const unsigned R = (of_a ? wm : wn) + index * 32 + row;
            v = *reinterpret_cast<const bf16x8*>((of_a ? a_buf : b_buf) + R * kRow + (kk * 2 + half) * 8u);
        }
        if constexpr (of_a) fa[set][index] = v;
        else fb[set][index] = v;
    };

    loader.prologue(a_cur, b_cur);
    __syncthreads();
    static_for<0, kFrags>([&](auto f) { fragment(std::integral_constant<int, 0>{}, f, a_cur, b_cur, 0); });

    unsigned s = 0;
    auto substep = [&](auto kk_c) {
        constexpr int KK = decltype(kk_c)::value, set = KK & 1;
        using Next = std::integral_constant<int, set ^ 1>;
        static_for<0, kMfmas>([&](auto i_c) {
            constexpr int I = decltype(i_c)::value, i = I / S::TN, j = I % S::TN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
            // one after each of the first MFMAs (more where a sub-step has fewer MFMAs than fragments)
            constexpr int kEach = (kFrags + kMfmas - 1) / kMfmas;
            static_for<(I * kEach < kFrags ? I * kEach : kFrags), ((I + 1) * kEach < kFrags ? (I + 1) * kEach : kFrags)>([&](auto f) {
                if constexpr (KK < 3) fragment(Next{}, f, a_cur, b_cur, KK + 1);
                else fragment(Next{}, f, a_nxt, b_nxt, 0);          // the first ones of the next step
            });
            if constexpr (KK < 3) {
                constexpr int kTasks = KK == 0 ? Loader::kTasks0 : KK == 1 ? Loader::kTasks1 : Loader::kTasks2;
                static_for<share_begin<I, kMfmas, kTasks>, share_end<I, kMfmas, kTasks>>([&](auto t_c) {
                    loader.template task<KK, decltype(t_c)::value>(a_nxt, b_nxt, s + 2);
                });
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    for (; s < steps; ++s) {
        substep(std::integral_constant<int, 0>{});
        substep(std::integral_constant<int, 1>{});
        substep(std::integral_constant<int, 2>{});
        __syncthreads();
        substep(std::integral_constant<int, 3>{});
        uint16_t* x = a_cur; a_cur = a_nxt; a_nxt = x;
        x = b_cur; b_cur = b_nxt; b_nxt = x;
    }
}

// Stores a wavefront's accumulators as bfloat16.  The MFMAs were given the column operand first, so tile (i, j)
// holds, in register q of lane l, the output of row row0 + 32 i + l % 32 and column
// col0 + 32 j + 8 (q / 4) + 4 (l / 32) + q % 4: a lane owns four neighbouring columns of one row.  Where the row
// length is a multiple of 8 the wavefront's 32 TM x 32 TN block goes through LDS (`staging`, private to the
// wavefront, rows of 32 TN + 8 elements) and leaves as 16-byte stores that cover whole 64 TN-byte row segments;
// rows and columns outside the matrix are addressed past the buffer's extent, and the hardware drops them.
// Otherwise single elements are stored.  addend: per column, binary32, in LDS, indexed from col0 (the bias), or nullptr.
template <int TM, int TN>
__device__ __forceinline__ void store_accumulators(const f32x16 (&acc)[TM][TN], uint16_t* out, unsigned rows, unsigned cols,
                                                   unsigned row0, unsigned col0, unsigned lane, const float* addend,
                                                   uint16_t* staging)
{
    constexpr unsigned kStride = 32 * TN + 8;                   // elements
    const unsigned row = lane & 31u, col = 4u * (lane >> 5);
    if (cols % 8u == 0) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const unsigned c = col + 32u * j + 8u * g;
                f32x4 b = {-0.0f, -0.0f, -0.0f, -0.0f};           // the addend that changes nothing, not even a -0
                if (addend) b = *reinterpret_cast<const f32x4*>(addend + c);
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    *reinterpret_cast<u32x2*>(staging + (row + 32u * i) * kStride + c) =
                        u32x2{pack2(acc[i][j][4 * g] + b[0], acc[i][j][4 * g + 1] + b[1]),
                              pack2(acc[i][j][4 * g + 2] + b[2], acc[i][j][4 * g + 3] + b[3])};
            }
        // the same wavefront reads back (LDS serves a wavefront's accesses in order): 4 TN lanes per row, 16 bytes each
        constexpr unsigned kLanesPerRow = 4 * TN, kRowsPerPass = 64 / kLanesPerRow;
        const __amdgpu_buffer_rsrc_t dst = whole_buffer(out, rows * cols * 2u);
        const unsigned r_in = lane / kLanesPerRow, c_in = (lane % kLanesPerRow) * 8u;
#pragma unroll
        for (unsigned p = 0; p < 32u * TM / kRowsPerPass; ++p) {
            const unsigned r = r_in + kRowsPerPass * p;
            const u32x4 v = *reinterpret_cast<const u32x4*>(staging + r * kStride + c_in);
            __builtin_amdgcn_raw_buffer_store_b128(
                v, dst, (int)(row0 + r < rows && col0 + c_in < cols ? ((row0 + r) * cols + col0 + c_in) * 2u : kOutside), 0, 0);
        }
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const unsigned c = col + 32u * j + 8u * (q / 4) + (q % 4);
                if (col0 + c >= cols) continue;
                const float b = addend ? addend[c] : -0.0f;
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    if (row0 + row + 32u * i < rows)
                        out[(size_t)(row0 + row + 32u * i) * cols + col0 + c] = (uint16_t)(pack2(acc[i][j][q] + b, 0.0f) & 0xFFFFu);
            }
    }
}

// Loader of the forward product.  Thread t moves the 16-byte piece t % 8 of rows t / 8, t / 8 + threads / 8, ...
// of both operand tiles (8 threads: one 128-byte row of a step); a row outside the matrix is addressed past
// the buffer's extent, where the hardware returns 0 and reads nothing.  The A pieces (the saved tensor) are
// decoded word by word in the first two sub-steps, the B pieces (the weight) are copied in the third.
template <int KIND, class S> struct LinearLoader {
    static constexpr unsigned kRowsPerPass = S::kThreads / 8;
    static constexpr unsigned kPassesA = S::kTileM / kRowsPerPass, kPassesB = S::kTileN / kRowsPerPass;
    static_assert(kPassesA % 2 == 0, "the A pieces are staged in two halves");
    static constexpr int kTasks0 = 4 * (kPassesA / 2), kTasks1 = kTasks0, kTasks2 = kPassesB;

    __amdgpu_buffer_rsrc_t a_src, b_src;
    unsigned a_off[kPassesA], b_off[kPassesB];      // byte offsets of this thread's pieces at step 0
    unsigned wr;                                    // where this thread writes inside a buffer (elements)
    unsigned steps;
    u32x4 ra[kPassesA], rb[kPassesB];

    __device__ __forceinline__ LinearLoader(const uint16_t* y_tagged, const uint16_t* w, unsigned M, unsigned N, unsigned K,
                                            unsigned m0, unsigned n0, unsigned t)
        : a_src(whole_buffer(y_tagged, M * K * 2u)), b_src(whole_buffer(w, N * K * 2u)), steps(K / kStep)
    {
        const unsigned r = t >> 3, piece = t & 7u;
        wr = r * kRow + piece * 8u;
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p)
            a_off[p] = m0 + r + kRowsPerPass * p < M ? ((m0 + r + kRowsPerPass * p) * K + piece * 8u) * 2u : kOutside;
#pragma unroll
        for (unsigned p = 0; p < kPassesB; ++p)
            b_off[p] = n0 + r + kRowsPerPass * p < N ? ((n0 + r + kRowsPerPass * p) * K + piece * 8u) * 2u : kOutside;
    }
    __device__ __forceinline__ unsigned step_bytes(unsigned step) const { return (step < steps ? step : steps - 1) * (kStep * 2u); }
    __device__ __forceinline__ void load_a(unsigned p, unsigned step)
    {
        ra[p] = __builtin_amdgcn_raw_buffer_load_b128(a_src, (int)a_off[p], (int)step_bytes(step), 0);
    }
    __device__ __forceinline__ void load_b(unsigned p, unsigned step)
    {
        rb[p] = __builtin_amdgcn_raw_buffer_load_b128(b_src, (int)b_off[p], (int)step_bytes(step), 0);
    }
    __device__ __forceinline__ void prologue(uint16_t* a_buf, uint16_t* b_buf)
    {
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p) load_a(p, 0);
#pragma unroll
        for (unsigned p = 0; p < kPassesB; ++p) load_b(p, 0);
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p) {
            *reinterpret_cast<u32x4*>(a_buf + kRowsPerPass * p * kRow + wr) = decode8<KIND>(ra[p]);
            load_a(p, 1);
        }
#pragma unroll
        for (unsigned p = 0; p < kPassesB; ++p) {
            *reinterpret_cast<u32x4*>(b_buf + kRowsPerPass * p * kRow + wr) = rb[p];
            load_b(p, 1);
        }
    }
    template <int KK, int T>
    __device__ __forceinline__ void task(uint16_t* a_nxt, uint16_t* b_nxt, unsigned step)
    {
        if constexpr (KK < 2) {
            constexpr int p = KK * (kPassesA / 2) + T / 4, word = T % 4;
            ra[p][word] = decode2<KIND>(ra[p][word]);
            if constexpr (word == 3) {
                *reinterpret_cast<u32x4*>(a_nxt + kRowsPerPass * p * kRow + wr) = ra[p];
                load_a(p, step);
            }
        } else {
            *reinterpret_cast<u32x4*>(b_nxt + kRowsPerPass * T * kRow + wr) = rb[T];
            load_b(T, step);
        }
    }
};

// out[M][N] = (|y_tagged| + C)[M][K] * w[N][K]^T (+ bias[N]); every matrix row-major, bfloat16; K a multiple of 64.
template <int KIND, class S>
__global__ __launch_bounds__(S::kThreads) void sbit_linear_kernel(const uint16_t* y_tagged, const uint16_t* w,
                                                                  const uint16_t* bias, uint16_t* out,
                                                                  unsigned M, unsigned N, unsigned K)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const unsigned n_tiles = (N + S::kTileN - 1) / S::kTileN;
    const TileAt at = banded(xcd_contiguous(blockIdx.x, gridDim.x), gridDim.x / n_tiles, n_tiles);
    const unsigned m0 = at.row * S::kTileM, n0 = at.col * S::kTileN;
    const unsigned t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const unsigned wm = (wave / S::WN) * (32 * S::TM), wn = (wave % S::WN) * (32 * S::TN);

    f32x16 acc[S::TM][S::TN] = {};
    LinearLoader<KIND, S> loader(y_tagged, w, M, N, K, m0, n0, t);
    contract<S, false, false>(lds, K / kStep, wm, wn, lane, loader, acc);

    // The operand buffers are free once every wavefront is here: each wavefront stages its block of the output in
    // its own part of them; the tile's share of the bias sits behind, as binary32.
    __syncthreads();
    float* const bias_lds = reinterpret_cast<float*>(lds + S::kOperandBytes / 2);
    if (bias) {
        for (unsigned c = t; c < (unsigned)S::kTileN; c += S::kThreads)
            bias_lds[c] = n0 + c < N ? __uint_as_float((uint32_t)bias[n0 + c] << 16) : 0.0f;
        __syncthreads();
    }
    store_accumulators<S::TM, S::TN>(acc, out, M, N, m0 + wm, n0 + wn, lane, bias ? bias_lds + wn : nullptr,
                                     lds + wave * (32 * S::TM) * (32 * S::TN + 8));
}

// Loader of the weight-gradient product.  The contraction index m is the slow one of both operands, and their
// tiles go into LDS as they lie in memory, [64 rows m][columns of the tile + kPadT]: the transposition happens
// in the fragment reads (see contract).  Thread t moves the 16-byte piece t % pieces of rows t / pieces,
// + threads / pieces, ... of either tile (pieces = columns of the tile / 8); N and K are multiples of 8, so a
// piece is inside its matrix or outside, and one outside is addressed past the buffer's extent (zeros, which land
// in rows or columns of the output that are never stored).  The pieces of the saved tensor are decoded word by
// word in the first two sub-steps, those of dOut are copied in the third.
template <int KIND, class S> struct WgradLoader {
    static constexpr unsigned kPiecesG = S::kTileM / 8, kRowsG = S::kThreads / kPiecesG, kPassesG = kStep / kRowsG;
    static constexpr unsigned kPiecesA = S::kTileN / 8, kRowsA = S::kThreads / kPiecesA, kPassesA = kStep / kRowsA;
    static_assert(kPassesG * kRowsG == kStep && kPassesA * kRowsA == kStep, "a step is a whole number of passes");
    static_assert(kPassesA % 2 == 0, "the pieces of the saved tensor are staged in two halves");
    static constexpr unsigned kPitchG = S::kTileM + kPadT, kPitchA = S::kTileN + kPadT;
    static constexpr int kTasks0 = 4 * (kPassesA / 2), kTasks1 = kTasks0, kTasks2 = kPassesG;

    __amdgpu_buffer_rsrc_t g_src, a_src;
    unsigned g_off[kPassesG], a_off[kPassesA];         // byte offsets of this thread's pieces at step 0
    unsigned g_wr, a_wr;                               // where this thread writes inside a buffer (elements)
    unsigned g_step, a_step, steps;                    // bytes from one step to the next
    u32x4 rg[kPassesG], ra[kPassesA];

    // first_step, steps: this workgroup's share of the contraction (rows 64 first_step .. 64 (first_step + steps) - 1 of M)
    __device__ __forceinline__ WgradLoader(const uint16_t* y_tagged, const uint16_t* grad_out, unsigned M, unsigned N, unsigned K,
                                           unsigned n0, unsigned k0, unsigned first_step, unsigned steps_, unsigned t)
        : g_src(whole_buffer(grad_out, M * N * 2u)), a_src(whole_buffer(y_tagged, M * K * 2u)),
          g_step(kStep * N * 2u), a_step(kStep * K * 2u), steps(steps_)
    {
        const unsigned row_g = first_step * kStep + t / kPiecesG, piece_g = t % kPiecesG;
        const unsigned row_a = first_step * kStep + t / kPiecesA, piece_a = t % kPiecesA;
        const bool g_in = n0 + piece_g * 8u < N, a_in = k0 + piece_a * 8u < K;
        g_wr = (t / kPiecesG) * kPitchG + piece_g * 8u;
        a_wr = (t / kPiecesA) * kPitchA + piece_a * 8u;
#pragma unroll
        for (unsigned p = 0; p < kPassesG; ++p) g_off[p] = g_in ? ((row_g + kRowsG * p) * N + n0 + piece_g * 8u) * 2u : kOutside;
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p) a_off[p] = a_in ? ((row_a + kRowsA * p) * K + k0 + piece_a * 8u) * 2u : kOutside;
    }
    __device__ __forceinline__ unsigned clamped(unsigned step) const { return step < steps ? step : steps - 1; }
    __device__ __forceinline__ void load_g(unsigned p, unsigned step)
    {
        rg[p] = __builtin_amdgcn_raw_buffer_load_b128(g_src, (int)g_off[p], (int)(clamped(step) * g_step), 0);
    }
    __device__ __forceinline__ void load_a(unsigned p, unsigned step)
    {
        ra[p] = __builtin_amdgcn_raw_buffer_load_b128(a_src, (int)a_off[p], (int)(clamped(step) * a_step), 0);
    }
    __device__ __forceinline__ void prologue(uint16_t* g_buf, uint16_t* a_buf)
    {
#pragma unroll
        for (unsigned p = 0; p < kPassesG; ++p) load_g(p, 0);
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p) load_a(p, 0);
#pragma unroll
        for (unsigned p = 0; p < kPassesG; ++p) {
            *reinterpret_cast<u32x4*>(g_buf + kRowsG * p * kPitchG + g_wr) = rg[p];
            load_g(p, 1);
        }
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p) {
            *reinterpret_cast<u32x4*>(a_buf + kRowsA * p * kPitchA + a_wr) = decode8<KIND>(ra[p]);
            load_a(p, 1);
        }
    }
    template <int KK, int T>
    __device__ __forceinline__ void task(uint16_t* g_nxt, uint16_t* a_nxt, unsigned step)
    {
        if constexpr (KK < 2) {
            constexpr int p = KK * (kPassesA / 2) + T / 4, word = T % 4;
            ra[p][word] = decode2<KIND>(ra[p][word]);
            if constexpr (word == 3) {
                *reinterpret_cast<u32x4*>(a_nxt + kRowsA * p * kPitchA + a_wr) = ra[p];
                load_a(p, step);
            }
        } else {
            *reinterpret_cast<u32x4*>(g_nxt + kRowsG * T * kPitchG + g_wr) = rg[T];
            load_g(T, step);
        }
    }
};

// grad_w[N][K] = grad_out[M][N]^T * (|y_tagged| + C)[M][K]; every matrix row-major, bfloat16; M a multiple of 64,
// N and K multiples of 8.  LDS rows are steps of the contraction (m), as in memory; the fragment reads transpose.
//
// The contraction can be split: the grid is `splits` x tiles workgroups, workgroup (split, tile) contracts over its
// share of the M / 64 steps, and with splits > 1 it leaves its binary32 accumulators in `partial` instead of
// storing the output: chunk split * tiles + tile, inside it wavefront by wavefront, 16-byte piece by piece in the
// order of the accumulator registers, lane by lane (every store instruction then covers 1 KiB).  wgrad_sum_kernel
// adds the chunks of a tile in the order of the splits and stores the output.  That is for outputs with too few tiles to fill the
// chip and a long contraction (the weight gradient of a layer that is narrow on both sides).
template <int TM, int TN>
__device__ __forceinline__ size_t partial_at(size_t chunk, unsigned waves, unsigned wave, unsigned lane)
{
    return ((chunk * waves + wave) * (TM * TN * 4) * 64u + lane) * 4u;      // in floats; piece q adds 256 q
}

template <int KIND, class S>
__global__ __launch_bounds__(S::kThreads) void sbit_linear_wgrad_kernel(const uint16_t* y_tagged, const uint16_t* grad_out,
                                                                        uint16_t* grad_w, unsigned M, unsigned N, unsigned K,
                                                                        unsigned splits, float* partial)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const unsigned k_tiles = (K + S::kTileN - 1) / S::kTileN, tiles = gridDim.x / splits;
    const unsigned chunk = xcd_contiguous(blockIdx.x, gridDim.x), split = chunk / tiles;
    const TileAt at = banded(chunk % tiles, tiles / k_tiles, k_tiles);
    const unsigned n0 = at.row * S::kTileM, k0 = at.col * S::kTileN;
    const unsigned t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const unsigned wm = (wave / S::WN) * (32 * S::TM), wn = (wave % S::WN) * (32 * S::TN);
    // the M / 64 steps in `splits` shares that differ by one step at most
    const unsigned all_steps = M / kStep, share = all_steps / splits, extra = all_steps % splits;
    const unsigned first_step = split * share + (split < extra ? split : extra), steps = share + (split < extra ? 1u : 0u);

    f32x16 acc[S::TM][S::TN] = {};
    WgradLoader<KIND, S> loader(y_tagged, grad_out, M, N, K, n0, k0, first_step, steps, t);
    contract<S, true, true>(lds, steps, wm, wn, lane, loader, acc);

    if (splits > 1) {
        float* const to = partial + partial_at<S::TM, S::TN>(chunk, S::WM * S::WN, wave, lane);
#pragma unroll
        for (int i = 0; i < S::TM; ++i)
#pragma unroll
            for (int j = 0; j < S::TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<f32x4*>(to + ((i * S::TN + j) * 4 + g) * 256) =
                        f32x4{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        return;
    }
    __syncthreads();       // the operand buffers are free once every wavefront is here: the output is staged there
    store_accumulators<S::TM, S::TN>(acc, grad_w, N, K, n0 + wm, k0 + wn, lane, nullptr,
                                     lds + wave * (32 * S::TM) * (32 * S::TN + 8));
}

// Second pass of a split weight gradient: one wavefront per row of 32 x 32 MFMA tiles of a wavefront of the first
// pass (workgroup (tile * waves + wave) * TM + i) adds those accumulators over the splits, first split first, and
// stores them as the first pass would have.
template <class S>
__global__ __launch_bounds__(64) void wgrad_sum_kernel(const float* partial, uint16_t* grad_w, unsigned N, unsigned K,
                                                       unsigned tiles, unsigned splits)
{
    __shared__ __attribute__((aligned(16))) uint16_t staging[32 * (32 * S::TN + 8)];
    constexpr unsigned kWaves = S::WM * S::WN;
    const unsigned k_tiles = (K + S::kTileN - 1) / S::kTileN;
    const unsigned i = blockIdx.x % S::TM, wave = blockIdx.x / S::TM % kWaves, tile = blockIdx.x / (S::TM * kWaves);
    const unsigned lane = threadIdx.x;
    const TileAt at = banded(tile, tiles / k_tiles, k_tiles);
    const unsigned wm = (wave / S::WN) * (32 * S::TM), wn = (wave % S::WN) * (32 * S::TN);

    f32x16 acc[1][S::TN] = {};
#pragma unroll 4
    for (unsigned split = 0; split < splits; ++split) {
        const float* const from = partial + partial_at<S::TM, S::TN>((size_t)split * tiles + tile, kWaves, wave, lane);
#pragma unroll
        for (int j = 0; j < S::TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(from + ((i * S::TN + j) * 4 + g) * 256));
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[0][j][4 * g + e] += v[e];
            }
    }
    store_accumulators<1, S::TN>(acc, grad_w, N, K, at.row * S::kTileM + wm + 32u * i, at.col * S::kTileN + wn, lane, nullptr, staging);
}

// Loader of the input-gradient product dOut W.  dOut [M][N] has the contraction index n as its fast one and is
// staged like the forward's operands (8 threads per 128-byte row of a step, plain layout); the weight [N][K] has
// it as its slow one and is staged as it lies in memory, like the weight gradient's operands (transposed
// layout).  Nothing is decoded: the tasks are LDS writes and reloads, dOut in the first two sub-steps, the
// weight in the third.  K is a multiple of 8, so a piece of the weight is inside the matrix or outside.
template <class S> struct DgradLoader {
    static constexpr unsigned kRowsPerPassA = S::kThreads / 8, kPassesA = S::kTileM / kRowsPerPassA;
    static constexpr unsigned kPiecesB = S::kTileN / 8, kRowsB = S::kThreads / kPiecesB, kPassesB = kStep / kRowsB;
    static_assert(kPassesB * kRowsB == kStep && kPassesA % 2 == 0, "whole passes; dOut is staged in two halves");
    static constexpr unsigned kPitchB = S::kTileN + kPadT;
    static constexpr int kTasks0 = kPassesA / 2, kTasks1 = kPassesA / 2, kTasks2 = kPassesB;

    __amdgpu_buffer_rsrc_t a_src, b_src;
    unsigned a_off[kPassesA], b_off[kPassesB];        // byte offsets of this thread's pieces at step 0
    unsigned a_wr, b_wr;                              // where this thread writes inside a buffer (elements)
    unsigned b_step, steps;                           // bytes from one step of the weight to the next
    u32x4 ra[kPassesA], rb[kPassesB];

    __device__ __forceinline__ DgradLoader(const uint16_t* grad_out, const uint16_t* w, unsigned M, unsigned N, unsigned K,
                                           unsigned m0, unsigned k0, unsigned t)
        : a_src(whole_buffer(grad_out, M * N * 2u)), b_src(whole_buffer(w, N * K * 2u)), b_step(kStep * K * 2u), steps(N / kStep)
    {
        const unsigned r = t >> 3, piece = t & 7u, row_b = t / kPiecesB, piece_b = t % kPiecesB;
        a_wr = r * kRow + piece * 8u;
        b_wr = row_b * kPitchB + piece_b * 8u;
        const bool b_in = k0 + piece_b * 8u < K;
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p)
            a_off[p] = m0 + r + kRowsPerPassA * p < M ? ((m0 + r + kRowsPerPassA * p) * N + piece * 8u) * 2u : kOutside;
#pragma unroll
        for (unsigned p = 0; p < kPassesB; ++p) b_off[p] = b_in ? ((row_b + kRowsB * p) * K + k0 + piece_b * 8u) * 2u : kOutside;
    }
    __device__ __forceinline__ unsigned clamped(unsigned step) const { return step < steps ? step : steps - 1; }
    __device__ __forceinline__ void load_a(unsigned p, unsigned step)
    {
        ra[p] = __builtin_amdgcn_raw_buffer_load_b128(a_src, (int)a_off[p], (int)(clamped(step) * (kStep * 2u)), 0);
    }
    __device__ __forceinline__ void load_b(unsigned p, unsigned step)
    {
        rb[p] = __builtin_amdgcn_raw_buffer_load_b128(b_src, (int)b_off[p], (int)(clamped(step) * b_step), 0);
    }
    __device__ __forceinline__ void prologue(uint16_t* a_buf, uint16_t* b_buf)
    {
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p) load_a(p, 0);
#pragma unroll
        for (unsigned p = 0; p < kPassesB; ++p) load_b(p, 0);
#pragma unroll
        for (unsigned p = 0; p < kPassesA; ++p) {
            *reinterpret_cast<u32x4*>(a_buf + kRowsPerPassA * p * kRow + a_wr) = ra[p];
            load_a(p, 1);
        }
#pragma unroll
        for (unsigned p = 0; p < kPassesB; ++p) {
            *reinterpret_cast<u32x4*>(b_buf + kRowsB * p * kPitchB + b_wr) = rb[p];
            load_b(p, 1);
        }
    }
    template <int KK, int T>
    __device__ __forceinline__ void task(uint16_t* a_nxt, uint16_t* b_nxt, unsigned step)
    {
        if constexpr (KK < 2) {
            constexpr int p = KK * (kPassesA / 2) + T;
            *reinterpret_cast<u32x4*>(a_nxt + kRowsPerPassA * p * kRow + a_wr) = ra[p];
            load_a(p, step);
        } else {
            *reinterpret_cast<u32x4*>(b_nxt + kRowsB * T * kPitchB + b_wr) = rb[T];
            load_b(T, step);
        }
    }
};

// Multiplies a wavefront's accumulators by q(|y_tagged| + C, sign bit of y_tagged) at their own positions
// (Eqs. (5)-(8), evaluated exactly as invact_sbit_bwd evaluates them).  A lane owns four neighbouring columns
// of a row (see store_accumulators): one 8-byte load of the saved tensor per four accumulators; cols is a
// multiple of 8, so the four are inside the matrix or outside, and outside reads as 0 and is never stored.
template <int KIND, int TM, int TN>
__device__ __forceinline__ void scale_by_q(f32x16 (&acc)[TM][TN], const uint16_t* y_tagged, unsigned rows, unsigned cols,
                                           unsigned row0, unsigned col0, unsigned lane)
{
    constexpr float C = min_of_kind<KIND>();
    const __amdgpu_buffer_rsrc_t src = whole_buffer(y_tagged, rows * cols * 2u);
    const unsigned row = row0 + (lane & 31u), col = col0 + 4u * (lane >> 5);
    u32x2 v[TM][TN][4];                      // every load is under way before the first value is used
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const unsigned r = row + 32u * i, c = col + 32u * j + 8u * g;
                v[i][j][g] = __builtin_amdgcn_raw_buffer_load_b64(src, (int)(r < rows && c < cols ? (r * cols + c) * 2u : kOutside), 0, 0);
            }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t word = v[i][j][g][e / 2];
                    const float t = __uint_as_float(e % 2 ? word & 0xFFFF0000u : word << 16);
                    acc[i][j][4 * g + e] = invact_dev::times_q<KIND, invact_dev::FAST>(
                        acc[i][j][4 * g + e], __builtin_fabsf(t) + C, (__float_as_uint(t) >> 31) != 0);
                }
}

// grad_x[M][K] = (grad_out[M][N] * w[N][K]) * q(|y_tagged| + C, S)[M][K]; every matrix row-major, bfloat16; N a
// multiple of 64, K a multiple of 8.
template <int KIND, class S>
__global__ __launch_bounds__(S::kThreads) void sbit_linear_dgrad_kernel(const uint16_t* y_tagged, const uint16_t* grad_out,
                                                                        const uint16_t* w, uint16_t* grad_x,
                                                                        unsigned M, unsigned N, unsigned K)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const unsigned k_tiles = (K + S::kTileN - 1) / S::kTileN;
    const TileAt at = banded(xcd_contiguous(blockIdx.x, gridDim.x), gridDim.x / k_tiles, k_tiles);
    const unsigned m0 = at.row * S::kTileM, k0 = at.col * S::kTileN;
    const unsigned t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const unsigned wm = (wave / S::WN) * (32 * S::TM), wn = (wave % S::WN) * (32 * S::TN);

    f32x16 acc[S::TM][S::TN] = {};
    DgradLoader<S> loader(grad_out, w, M, N, K, m0, k0, t);
    contract<S, false, true>(lds, N / kStep, wm, wn, lane, loader, acc);

    scale_by_q<KIND, S::TM, S::TN>(acc, y_tagged, M, K, m0 + wm, k0 + wn, lane);
    __syncthreads();       // the operand buffers are free once every wavefront is here: the output is staged there
    store_accumulators<S::TM, S::TN>(acc, grad_x, M, K, m0 + wm, k0 + wn, lane, nullptr,
                                     lds + wave * (32 * S::TM) * (32 * S::TN + 8));
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

// Which shape: the large tile where it still gives every compute unit a workgroup (256 of them); else 128 x 128,
// with 8 wavefronts where there is at most one such workgroup per compute unit (two wavefronts per SIMD hide each
// other's waits: +6 to +15 %), with 4 where there are more (several workgroups per compute unit do that already, and
// the 4-wavefront shape reads a third less from LDS).
std::atomic<int> g_force_tile{0};                       // 0: choose; 2: Small; 3: Small8; 4: Large (benchmarking, tests)
enum class Tile { kLarge, kSmall, kSmall8 };
Tile tile_for(size_t rows, size_t cols)
{
    switch (g_force_tile.load(std::memory_order_relaxed)) {
    case 2: return Tile::kSmall;
    case 3: return Tile::kSmall8;
    case 4: return Tile::kLarge;
    default: break;
    }
    if (tiles_of<Large>(rows, cols) >= 256) return Tile::kLarge;
    return tiles_of<Small>(rows, cols) <= 256 ? Tile::kSmall8 : Tile::kSmall;
}

template <int KIND>
int run_linear(const uint16_t* a, const uint16_t* b, const uint16_t* c, uint16_t* o, unsigned m, unsigned n, unsigned k,
               hipStream_t stream)
{
    switch (tile_for(m, n)) {
    case Tile::kLarge:
        return launch_tiles<sbit_linear_kernel<KIND, Large>, Large>(tiles_of<Large>(m, n), stream, a, b, c, o, m, n, k);
    case Tile::kSmall8:
        return launch_tiles<sbit_linear_kernel<KIND, Small8>, Small8>(tiles_of<Small8>(m, n), stream, a, b, c, o, m, n, k);
    default:
        return launch_tiles<sbit_linear_kernel<KIND, Small>, Small>(tiles_of<Small>(m, n), stream, a, b, c, o, m, n, k);
    }
}

template <int KIND>
int run_dgrad(const uint16_t* a, const uint16_t* g, const uint16_t* w, uint16_t* o, unsigned m, unsigned n, unsigned k,
              hipStream_t stream)
{
    switch (tile_for(m, k)) {
    case Tile::kLarge:
        return launch_tiles<sbit_linear_dgrad_kernel<KIND, Large>, Large>(tiles_of<Large>(m, k), stream, a, g, w, o, m, n, k);
    case Tile::kSmall8:
        return launch_tiles<sbit_linear_dgrad_kernel<KIND, Small8>, Small8>(tiles_of<Small8>(m, k), stream, a, g, w, o, m, n, k);
    default:
        return launch_tiles<sbit_linear_dgrad_kernel<KIND, Small>, Small>(tiles_of<Small>(m, k), stream, a, g, w, o, m, n, k);
    }
}

// How a weight gradient with an N x K output and M / 64 steps of contraction runs: tile shape, number of splits of
// the contraction, and the bytes of binary32 partial sums that needs (0 when it is not split).
std::atomic<int> g_force_splits{0};                     // 0: choose; 1 .. kMaxSplits: force (benchmarking, tests)
constexpr unsigned kMaxSplits = 64;
struct WgradPlan { Tile tile; unsigned splits; size_t tiles, bytes; };
WgradPlan plan_wgrad(size_t M, size_t N, size_t K, bool may_split)
{
    WgradPlan plan{tile_for(N, K), 1, 0, 0};
    const size_t steps = M / kStep;
    const int forced = g_force_splits.load(std::memory_order_relaxed);
    if (may_split && forced > 0) {
        plan.splits = (unsigned)(forced < (int)steps ? forced : steps);
    } else if (may_split && g_force_tile.load(std::memory_order_relaxed) == 0) {
        // Fewer large tiles than compute units (256).  Split so that every compute unit gets one, as long as a part
        // stays kMinSteps long (each part costs a write and a read of 4 bytes per output element); if not even
        // half of them would get a large tile that way, do the same with the small tile.
        constexpr size_t kMinSteps = 16;
        const size_t large = tiles_of<Large>(N, K), small = tiles_of<Small>(N, K), most = steps / kMinSteps;
        if (large < 256) {
            size_t splits = 256 / large < most ? 256 / large : most;
            if (splits > 1 && large * splits >= 128) {
                plan.tile = Tile::kLarge;
            } else {
                splits = small < 256 ? (256 / small < most ? 256 / small : most) : 1;
                if (splits > 1) plan.tile = Tile::kSmall8;
            }
            if (splits > 1) plan.splits = (unsigned)(splits < kMaxSplits ? splits : kMaxSplits);
        }
    }
    size_t tile_elems;
    switch (plan.tile) {
    case Tile::kLarge:  plan.tiles = tiles_of<Large>(N, K), tile_elems = Large::kTileM * Large::kTileN; break;
    case Tile::kSmall8: plan.tiles = tiles_of<Small8>(N, K), tile_elems = Small8::kTileM * Small8::kTileN; break;
    default:            plan.tiles = tiles_of<Small>(N, K), tile_elems = Small::kTileM * Small::kTileN; break;
    }
    plan.bytes = plan.splits > 1 ? plan.splits * plan.tiles * tile_elems * sizeof(float) : 0;
    return plan;
}

template <int KIND, class S>
int run_wgrad_shape(const WgradPlan& plan, const uint16_t* a, const uint16_t* g, uint16_t* o, unsigned m, unsigned n, unsigned k,
                    float* partial, hipStream_t stream)
{
    const unsigned tiles = (unsigned)plan.tiles, splits = plan.splits;
    if (int e = launch_tiles<sbit_linear_wgrad_kernel<KIND, S>, S>(plan.tiles * splits, stream, a, g, o, m, n, k, splits, partial))
        return e;
    if (splits == 1) return INVACT_OK;
    // the launch's own status, not the thread's last-error slot
    const float* from = partial;
    void* argv[] = {&from, &o, &n, &k, const_cast<unsigned*>(&tiles), const_cast<unsigned*>(&splits)};
    return hipLaunchKernel(reinterpret_cast<const void*>(wgrad_sum_kernel<S>), dim3(tiles * S::WM * S::WN * S::TM), dim3(64),
                           argv, 0, stream) == hipSuccess ? INVACT_OK : INVACT_ERR_HIP;
}

template <int KIND>
int run_wgrad(const WgradPlan& plan, const uint16_t* a, const uint16_t* g, uint16_t* o, unsigned m, unsigned n, unsigned k,
              float* partial, hipStream_t stream)
{
    switch (plan.tile) {
    case Tile::kLarge:  return run_wgrad_shape<KIND, Large>(plan, a, g, o, m, n, k, partial, stream);
    case Tile::kSmall8: return run_wgrad_shape<KIND, Small8>(plan, a, g, o, m, n, k, partial, stream);
    default:            return run_wgrad_shape<KIND, Small>(plan, a, g, o, m, n, k, partial, stream);
    }
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

extern "C" int invact_sbit_linear_dgrad(int kind, int dtype, const void* y_tagged, const void* grad_out, const void* weight,
                                        void* grad_x, size_t M, size_t N, size_t K, hipStream_t stream)
{
    if (int e = check_kind_dtype(kind, dtype)) return e;
    if (N == 0 || N % kStep != 0 || K % 8 != 0 || !fits(M, K) || !fits(N, K) || !fits(M, N)) return INVACT_ERR_SIZE;
    if (M == 0 || K == 0) return INVACT_OK;
    if (!y_tagged || !grad_out || !weight || !grad_x) return INVACT_ERR_NULL;
    if (!aligned16(y_tagged) || !aligned16(grad_out) || !aligned16(weight) || !aligned16(grad_x)) return INVACT_ERR_ALIGN;
    const uint16_t *a = static_cast<const uint16_t*>(y_tagged), *g = static_cast<const uint16_t*>(grad_out),
                   *w = static_cast<const uint16_t*>(weight);
    uint16_t* o = static_cast<uint16_t*>(grad_x);
    const unsigned m = (unsigned)M, n = (unsigned)N, k = (unsigned)K;
    switch (kind) {
    case INVACT_GELU_TANH: return run_dgrad<INVACT_GELU_TANH>(a, g, w, o, m, n, k, stream);
    case INVACT_GELU_ERF:  return run_dgrad<INVACT_GELU_ERF>(a, g, w, o, m, n, k, stream);
    default:               return run_dgrad<INVACT_SILU>(a, g, w, o, m, n, k, stream);
    }
}

// Partial sums of invact_sbit_linear_wgrad_static: one array per GPU, allocated with the code object, shared by
// every call on that GPU.  In host code the name is only a handle; scratch_of_device() asks the runtime for the
// array's address on the current device, once per device.
constexpr size_t kScratchBytes = size_t(64) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

std::atomic<void*> g_scratch_at[64];

int scratch_of_device(void** at)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return INVACT_ERR_HIP;
    void* p = g_scratch_at[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return INVACT_ERR_HIP;
        g_scratch_at[dev].store(p, std::memory_order_release);
    }
    *at = p;
    return INVACT_OK;
}

// workspace: the caller's; or, with in_scratch, this GPU's scratch array (workspace and workspace_bytes are ignored)
int wgrad_entry(int kind, int dtype, const void* y_tagged, const void* grad_out, void* grad_weight, size_t M, size_t N, size_t K,
                bool may_split, bool in_scratch, void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (int e = check_kind_dtype(kind, dtype)) return e;
    if (M == 0 || M % kStep != 0 || N % 8 != 0 || K % 8 != 0 || !fits(M, K) || !fits(N, K) || !fits(M, N))
        return INVACT_ERR_SIZE;
    if (N == 0 || K == 0) return INVACT_OK;
    const WgradPlan plan = plan_wgrad(M, N, K, may_split);
    if (plan.bytes > (in_scratch ? kScratchBytes : workspace_bytes) ||
        plan.tiles * plan.splits > 0x7FFFFFFFu / 32u /* workgroups of the summing pass */)
        return INVACT_ERR_SIZE;
    if (!y_tagged || !grad_out || !grad_weight) return INVACT_ERR_NULL;
    if (!aligned16(y_tagged) || !aligned16(grad_out) || !aligned16(grad_weight)) return INVACT_ERR_ALIGN;
    if (plan.bytes && in_scratch) {
        if (int e = scratch_of_device(&workspace)) return e;
    } else if (plan.bytes) {
        if (!workspace) return INVACT_ERR_NULL;
        if (!aligned16(workspace)) return INVACT_ERR_ALIGN;
    }
    const uint16_t *a = static_cast<const uint16_t*>(y_tagged), *g = static_cast<const uint16_t*>(grad_out);
    uint16_t* o = static_cast<uint16_t*>(grad_weight);
    float* const partial = static_cast<float*>(workspace);
    const unsigned m = (unsigned)M, n = (unsigned)N, k = (unsigned)K;
    switch (kind) {
    case INVACT_GELU_TANH: return run_wgrad<INVACT_GELU_TANH>(plan, a, g, o, m, n, k, partial, stream);
    case INVACT_GELU_ERF:  return run_wgrad<INVACT_GELU_ERF>(plan, a, g, o, m, n, k, partial, stream);
    default:               return run_wgrad<INVACT_SILU>(plan, a, g, o, m, n, k, partial, stream);
    }
}

}  // namespace

extern "C" int invact_sbit_linear_wgrad(int kind, int dtype, const void* y_tagged, const void* grad_out,
                                        void* grad_weight, size_t M, size_t N, size_t K, hipStream_t stream)
{
    return wgrad_entry(kind, dtype, y_tagged, grad_out, grad_weight, M, N, K, false, false, nullptr, 0, stream);
}

extern "C" size_t invact_sbit_linear_wgrad_workspace(size_t M, size_t N, size_t K)
{
    if (M == 0 || M % kStep != 0 || N % 8 != 0 || K % 8 != 0 || N == 0 || K == 0 || !fits(N, K)) return 0;
    return plan_wgrad(M, N, K, true).bytes;
}

extern "C" int invact_sbit_linear_wgrad_ws(int kind, int dtype, const void* y_tagged, const void* grad_out,
                                           void* grad_weight, size_t M, size_t N, size_t K, void* workspace,
                                           size_t workspace_bytes, hipStream_t stream)
{
    return wgrad_entry(kind, dtype, y_tagged, grad_out, grad_weight, M, N, K, true, false, workspace, workspace_bytes, stream);
}

extern "C" int invact_sbit_linear_wgrad_static(int kind, int dtype, const void* y_tagged, const void* grad_out,
                                               void* grad_weight, size_t M, size_t N, size_t K, hipStream_t stream)
{
    return wgrad_entry(kind, dtype, y_tagged, grad_out, grad_weight, M, N, K, true, true, nullptr, 0, stream);
}

// Benchmarking and tests: 0 lets the library choose the shape of the two products above, 2, 3 or 4 forces Small,
// Small8 or Large (results are the same up to the order of the binary32 sums).  Returns its argument, or -1 if it is none of these.
extern "C" int invact_set_linear_tile(int t)
{
    if (t != 0 && t != 2 && t != 3 && t != 4) return -1;
    g_force_tile.store(t, std::memory_order_relaxed);
    return t;
}

// Benchmarking and tests: 0 lets invact_sbit_linear_wgrad_ws choose into how many parts it splits the contraction,
// 1 .. 64 forces that number (capped at the number of 64-row steps).  Returns its argument, or -1 if it is out of range.
extern "C" int invact_set_linear_splits(int splits)
{
    if (splits < 0 || splits > (int)kMaxSplits) return -1;
    g_force_splits.store(splits, std::memory_order_relaxed);
    return splits;
}
