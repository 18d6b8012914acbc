// HIP kernels and C ABI of libinvact (gfx950 only).  See include/invact.h for
// the contract of every entry point.
//
// Kernel shape.  All kernels are pure streaming maps, bound by HBM
// bandwidth, so they share one skeleton.  The unit of work of a wavefront is a
// "wave tile" of 64 chunks, a chunk being the elements one lane owns:
//   bfloat16  8 elements per lane (tile of 512): lane L owns elements 8L .. 8L+7,
//             one 128-bit access, and exactly mask byte L of the tile;
//   binary32  4 elements per lane (tile of 256): one 128-bit access per tensor;
//             a lane holds one nibble of mask byte L/2, neighbouring lanes
//             exchange nibbles with one DPP move and the even one stores the
//             byte (reading, both load it).  The forward kernels, whose
//             binary64 arithmetic per element is long, take 8 elements per lane
//             instead (tile of 512, elements 4L.. and 256+4L..: two coalesced
//             accesses; letting a lane own 32 contiguous bytes would cost
//             10-19 % of the bandwidth): eight independent chains hide the
//             latency better (4-5 %), while every other kernel is 2-8 % faster
//             with the smaller footprint per wavefront.
// The canonical little-endian bit stream thus comes out of lane-local shifts,
// whatever the tiling of the kernel that wrote it.
// A lane keeps Op::kShape.unroll chunks in flight: all loads of a step are issued
// before the first store, which is also what makes element-wise in-place use
// (y == x and the like) safe.  The tensor accesses are non-temporal (each byte
// is touched once); mask bytes go through the cache, because the 32 or 64 bytes
// a wavefront touches are a fraction of a cache line.  The elements past the
// last full wave tile (fewer than 512) are handled one element per lane by the first wavefront,
// the mask word being formed by a wave64 ballot there (and zero padding coming
// for free).
//
// Launch shape.  A workgroup is ONE wavefront (four for the kernels that read
// the erfcx table from LDS: see stream_kernel) that handles kShape.unroll wave
// tiles and retires; the hardware dispatcher balances the load.  HBM delivers
// the most when a compute unit has roughly 32 to 96 KiB of loads in flight and
// no more: beyond that the streams of too many wavefronts interleave in the
// memory channels and the rate drops by 5-10 %.  Op::kShape.resident therefore
// caps the number of resident wavefronts per compute unit (below the 32 the
// hardware allows) by giving each workgroup a share of the 160 KiB of LDS that
// it never touches.  Single-wavefront workgroups matter for this: a freed slot
// is refilled at once instead of waiting for the last wavefront of a larger
// workgroup.  The figures in the kShape tables are the measured optima on
// MI355X at 2^24 elements and more; below that the launch is latency-bound
// and the shape makes no difference.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/invact.h"
#include "invact_math.h"

namespace {

using namespace invact_dev;

#ifndef INVACT_LD_AUX
#define INVACT_LD_AUX 2            // nt
#endif
#ifndef INVACT_ST_AUX
#define INVACT_ST_AUX 18           // nt sc1
#endif
#ifndef INVACT_MASK_AUX
#define INVACT_MASK_AUX 0
#endif
#ifndef INVACT_DEFAULT_BLOCKS_PER_CU
#define INVACT_DEFAULT_BLOCKS_PER_CU 0
#endif

// Cache-policy bits of the buffer instructions (the `aux` operand): 1 = sc0, 2 = nt, 16 = sc1.
// Every tensor byte is touched once, so loads carry the non-temporal hint (worth 4-8 % over plain
// loads); stores carry nt and sc1, which on this machine is another 1.5-2 % over nt alone for a
// mix of read and write streams under the occupancy cap the gated kernels use (measured with a
// plain copy kernel of the same stream mix: 3 reads + 2 writes 6.65 -> 6.76 TB/s).
constexpr int kLoadAux = INVACT_LD_AUX, kStoreAux = INVACT_ST_AUX, kMaskAux = INVACT_MASK_AUX;
constexpr int  kDefaultBlocksPerCu = INVACT_DEFAULT_BLOCKS_PER_CU;   // 0: one tile per workgroup
constexpr int  kWaveSlotsPerCu = 32;              // resident wavefronts a compute unit can hold
constexpr int  kWave = 64;                        // lanes of a wavefront

// Launch shape of an operation: wave tiles per wavefront and the cap on resident wavefronts per
// compute unit (none if they would fill the kWaveSlotsPerCu slots anyway).
struct Shape { int unroll, resident; };
template <int DT> constexpr Shape pick(Shape binary32, Shape bfloat16)
{
#ifdef INVACT_UNROLL_ALL                           // build variants for sweeps
    binary32.unroll = bfloat16.unroll = INVACT_UNROLL_ALL;
#endif
    return DT == INVACT_FP32 ? binary32 : bfloat16;
}

typedef float    f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16   bf16x2 __attribute__((ext_vector_type(2)));
typedef float    f32x2 __attribute__((ext_vector_type(2)));

// A wave tile's piece of a tensor as a raw buffer: base = p + offset lives in scalar registers (the
// tile index is the workgroup's), the lane supplies a 32-bit byte offset, and the extent makes the
// hardware drop anything addressed outside the piece.  No 64-bit vector address arithmetic.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_buffer(const void* p, size_t offset, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(p)) + offset, 0, (int)bytes,
                                             0x00020000 /* untyped 32-bit data, no swizzle */);
}
__device__ __forceinline__ u32x4 ld128(__amdgpu_buffer_rsrc_t r, unsigned byte)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte, 0, kLoadAux);
}
__device__ __forceinline__ void st128(__amdgpu_buffer_rsrc_t r, unsigned byte, u32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)byte, 0, kStoreAux);
}
// The mask moves 64 bytes per wavefront and step, half a cache line: it goes through the cache,
// so that the two halves of a line reach HBM as one write.  On the read side the two wavefronts
// that share a line sit on different XCDs (consecutive workgroups do), each with its own L2, so
// the line is fetched twice: 1.2 % more read traffic for the gated backward, which is cheaper than
// keeping the pair on one XCD (measured 0.5-6 % slower).
__device__ __forceinline__ uint32_t ld8(__amdgpu_buffer_rsrc_t r, unsigned byte)
{
    return __builtin_amdgcn_raw_buffer_load_b8(r, (int)byte, 0, kMaskAux);
}
__device__ __forceinline__ void st8(__amdgpu_buffer_rsrc_t r, unsigned byte, uint32_t v)
{
    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)v, r, (int)byte, 0, kMaskAux);
}

// value of the neighbouring lane (lane ^ 1); every lane of the quad must be active
__device__ __forceinline__ uint32_t swap_with_neighbour(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true);
}

// ---------------------------------------------------------------------------
// Storage formats: one chunk (the elements one lane owns in a wave tile) <->
// floats in registers, and the chunk's mask bits <-> memory.  `t` is the wave
// tile (wave-uniform: it comes from the workgroup index), `lane` the lane.
// ---------------------------------------------------------------------------

template <int DT, int ELEMS> struct Storage;        // ELEMS = elements per lane and chunk

// Elements per lane for the streaming-bound operations: one 128-bit access per tensor.
template <int DT> constexpr int lean_elems() { return DT == INVACT_FP32 ? 4 : 8; }

// What the binary32 layouts share: scalar accesses for the tail and the precision-bit tag.
struct Binary32 {
    static constexpr int kPrec = PRECISE;
    static __device__ __forceinline__ float load1(const void* p, size_t i) { return reinterpret_cast<const float*>(p)[i]; }
    static __device__ __forceinline__ void store1(void* p, size_t i, float v) { reinterpret_cast<float*>(p)[i] = v; }
    // precision-bit variant: bit 0 of the stored pattern := the indicator / read it back
    static __device__ __forceinline__ float tag(float v, uint32_t bit)
    {
        return __uint_as_float((__float_as_uint(v) & ~1u) | bit);
    }
    static __device__ __forceinline__ uint32_t lsb(float v) { return __float_as_uint(v) & 1u; }
    static __device__ __forceinline__ void store1_tagged(void* p, size_t i, float v, bool bit) { store1(p, i, tag(v, bit)); }
    static __device__ __forceinline__ bool lsb1(const void* p, size_t i) { return lsb(load1(p, i)); }
};

// binary32, 4 elements per lane: one 128-bit access per tensor and a 256-element wave tile.
template <> struct Storage<INVACT_FP32, 4> : Binary32 {
    struct Raw { u32x4 a; };
    static constexpr int kElems = 4;                    // elements per lane and chunk
    static constexpr int kWaveTile = kWave * kElems;    // elements per wavefront and tile
    static constexpr unsigned kTileBytes = kWaveTile * 4, kMaskBytes = kWaveTile / 8;
    static __device__ __forceinline__ Raw load(const void* p, size_t t, unsigned lane)
    {
        return Raw{ld128(tile_buffer(p, t * kTileBytes, kTileBytes), lane * 16)};
    }
    static __device__ __forceinline__ void unpack(const Raw& r, float (&v)[4])
    {
        for (int j = 0; j < 4; ++j) v[j] = __uint_as_float(r.a[j]);
    }
    static __device__ __forceinline__ void store(void* p, size_t t, unsigned lane, const float (&v)[4])
    {
        st128(tile_buffer(p, t * kTileBytes, kTileBytes), lane * 16,
              u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])});
    }
    // A lane owns the low (even lane) or high (odd lane) nibble of mask byte lane / 2 of the tile.  Writing: the two
    // lanes exchange nibbles with one DPP move and the even one stores the byte.  Reading: both load it.
    static __device__ __forceinline__ void store_mask(uint8_t* mask, size_t t, unsigned lane, uint32_t m)
    {
        const uint32_t other = swap_with_neighbour(m);
        if (!(lane & 1)) st8(tile_buffer(mask, t * kMaskBytes, kMaskBytes), lane >> 1, m | (other << 4));
    }
    static __device__ __forceinline__ uint32_t load_mask(const uint8_t* mask, size_t t, unsigned lane)
    {
        const uint32_t byte = ld8(tile_buffer(mask, t * kMaskBytes, kMaskBytes), lane >> 1);
        return (lane & 1) ? (byte >> 4) : (byte & 0xFu);
    }
    // ind[j] is the indicator of element j as 0.0f or 1.0f (indicator01)
    static __device__ __forceinline__ void store_tagged(void* p, size_t t, unsigned lane, float (&v)[4], const float (&ind)[4])
    {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = tag(v[j], (uint32_t)ind[j]);
        store(p, t, lane, v);
    }
    static __device__ __forceinline__ uint32_t unpack_tagged(const Raw& r, float (&v)[4])
    {
        unpack(r, v);
        uint32_t m = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) m |= lsb(v[j]) << j;
        return m;
    }
};

// binary32, 8 elements per lane: elements 4L .. 4L+3 and 256+4L .. 256+4L+3 of a 512-element wave tile, i.e. two
// coalesced 128-bit accesses (a lane owning 32 contiguous bytes costs 10-19 % of the bandwidth).  A lane then holds
// two nibbles of two different mask bytes; neighbouring lanes swap nibbles with one DPP move so that every lane
// stores (or loads) one byte.  Used where the arithmetic per element is long and more independent chains help.
template <> struct Storage<INVACT_FP32, 8> : Binary32 {
    struct Raw { u32x4 a, b; };
    static constexpr int kElems = 8;
    static constexpr int kWaveTile = kWave * kElems;
    static constexpr unsigned kTileBytes = kWaveTile * 4, kMaskBytes = kWaveTile / 8;
    // v[0..3] = elements 4L.., v[4..7] = elements 256 + 4L.. of the wave tile
    static __device__ __forceinline__ Raw load(const void* p, size_t t, unsigned lane)
    {
        const __amdgpu_buffer_rsrc_t r = tile_buffer(p, t * kTileBytes, kTileBytes);
        return Raw{ld128(r, lane * 16), ld128(r, 1024 + lane * 16)};
    }
    static __device__ __forceinline__ void unpack(const Raw& r, float (&v)[8])
    {
        for (int j = 0; j < 4; ++j) { v[j] = __uint_as_float(r.a[j]); v[4 + j] = __uint_as_float(r.b[j]); }
    }
    static __device__ __forceinline__ void store(void* p, size_t t, unsigned lane, const float (&v)[8])
    {
        const __amdgpu_buffer_rsrc_t r = tile_buffer(p, t * kTileBytes, kTileBytes);
        st128(r, lane * 16, u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])});
        st128(r, 1024 + lane * 16, u32x4{__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])});
    }
    // Bits 0-3 of m belong to byte L/2 of the tile (low nibble for even L), bits
    // 4-7 to byte 32 + L/2.  Even lanes end up with the first byte of the pair,
    // odd lanes with the second.
    static __device__ __forceinline__ unsigned mask_byte(unsigned lane) { return ((lane & 1) ? 32 : 0) + (lane >> 1); }
    static __device__ __forceinline__ void store_mask(uint8_t* mask, size_t t, unsigned lane, uint32_t m)
    {
        const uint32_t other = swap_with_neighbour(m);
        const uint32_t byte = (lane & 1) ? (((other >> 4) & 0xFu) | (m & 0xF0u))
                                         : ((m & 0xFu) | ((other & 0xFu) << 4));
        st8(tile_buffer(mask, t * kMaskBytes, kMaskBytes), mask_byte(lane), byte);
    }
    static __device__ __forceinline__ uint32_t load_mask(const uint8_t* mask, size_t t, unsigned lane)
    {
        const uint32_t own = ld8(tile_buffer(mask, t * kMaskBytes, kMaskBytes), mask_byte(lane));
        const uint32_t other = swap_with_neighbour(own);
        return (lane & 1) ? ((other >> 4) | (own & 0xF0u)) : ((own & 0xFu) | ((other & 0xFu) << 4));
    }
    static __device__ __forceinline__ void store_tagged(void* p, size_t t, unsigned lane, float (&v)[8], const float (&ind)[8])
    {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = tag(v[j], (uint32_t)ind[j]);
        store(p, t, lane, v);
    }
    static __device__ __forceinline__ uint32_t unpack_tagged(const Raw& r, float (&v)[8])
    {
        unpack(r, v);
        uint32_t m = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) m |= lsb(v[j]) << j;
        return m;
    }
};

// bfloat16, 8 elements per lane: one 128-bit access per tensor, and exactly mask byte L of the 512-element wave tile.
template <> struct Storage<INVACT_BF16, 8> {
    struct Raw { u32x4 w; };
    static constexpr int kPrec = FAST;
    static constexpr int kElems = 8;                    // elements per lane and chunk
    static constexpr int kWaveTile = kWave * kElems;    // elements per wavefront and tile
    static constexpr unsigned kTileBytes = kWaveTile * 2, kMaskBytes = kWaveTile / 8;
    static __device__ __forceinline__ Raw load(const void* p, size_t t, unsigned lane)
    {
        return Raw{ld128(tile_buffer(p, t * kTileBytes, kTileBytes), lane * 16)};
    }
    static __device__ __forceinline__ void unpack(const Raw& r, float (&v)[8])
    {
        for (int j = 0; j < 4; ++j) {
            v[2 * j]     = __uint_as_float(r.w[j] << 16);
            v[2 * j + 1] = __uint_as_float(r.w[j] & 0xFFFF0000u);
        }
    }
    // round to nearest even (v_cvt_pk_bf16_f32)
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
    }
    static __device__ __forceinline__ void store(void* p, size_t t, unsigned lane, const float (&v)[8])
    {
        st128(tile_buffer(p, t * kTileBytes, kTileBytes), lane * 16,
              u32x4{pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])});
    }
    static __device__ __forceinline__ void store_mask(uint8_t* mask, size_t t, unsigned lane, uint32_t m)
    {
        st8(tile_buffer(mask, t * kMaskBytes, kMaskBytes), lane, m);
    }
    static __device__ __forceinline__ uint32_t load_mask(const uint8_t* mask, size_t t, unsigned lane)
    {
        return ld8(tile_buffer(mask, t * kMaskBytes, kMaskBytes), lane);
    }
    static __device__ __forceinline__ float load1(const void* p, size_t i)
    {
        return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(p)[i] << 16);
    }
    static __device__ __forceinline__ void store1(void* p, size_t i, float v)
    {
        reinterpret_cast<uint16_t*>(p)[i] = (uint16_t)(pack2(v, 0.0f) & 0xFFFFu);
    }
    // precision-bit variant: bit 0 of each stored 16-bit pattern := bit j of m / read it back
    // (ind[j] is the indicator of element j as 0.0f or 1.0f: the two tag bits of a word are one exact binary32 sum)
    static __device__ __forceinline__ void store_tagged(void* p, size_t t, unsigned lane, float (&v)[8], const float (&ind)[8])
    {
        u32x4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t bits = (uint32_t)fmaf(ind[2 * j + 1], 65536.0f, ind[2 * j]);
            w[j] = (pack2(v[2 * j], v[2 * j + 1]) & 0xFFFEFFFEu) | bits;
        }
        st128(tile_buffer(p, t * kTileBytes, kTileBytes), lane * 16, w);
    }
    static __device__ __forceinline__ uint32_t unpack_tagged(const Raw& r, float (&v)[8])
    {
        unpack(r, v);
        uint32_t m = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) m |= ((r.w[j] & 1u) << (2 * j)) | (((r.w[j] >> 16) & 1u) << (2 * j + 1));
        return m;
    }
    static __device__ __forceinline__ void store1_tagged(void* p, size_t i, float v, bool bit)
    {
        reinterpret_cast<uint16_t*>(p)[i] = (uint16_t)((pack2(v, 0.0f) & 0xFFFEu) | (uint32_t)bit);
    }
    static __device__ __forceinline__ bool lsb1(const void* p, size_t i) { return reinterpret_cast<const uint16_t*>(p)[i] & 1u; }
};

// The indicator [x < T] of all elements of a chunk, packed (element j -> bit j), without compares and
// selects: (T - x) 2^25 is at least 2 for every binary32 x below T (T lies in [-2, -1/2], where
// neighbouring values are at least 2^-24 apart) and at most 0 otherwise, so clamping it to [0, 1] gives
// exactly 1.0 or 0.0 -- a fused multiply-add with the clamp modifier, which also turns a NaN into 0 and
// -inf into 1 -- and sum_j 2^j [x_j < T] is exact in binary32.  Two full-rate instructions per element
// instead of compare + select + or.
template <int KIND>
__device__ __forceinline__ float indicator01(float x)                  // [x < T] as 0.0f or 1.0f
{
    constexpr float kBig = 33554432.0f;                                // 2^25
    return med3(fmaf(x, -kBig, KindConst<KIND>::T * kBig), 0.0f, 1.0f);
}
template <int KIND, int N>
__device__ __forceinline__ uint32_t indicator_bits(const float (&v)[N])
{
    float sum = indicator01<KIND>(v[0]);
#pragma unroll
    for (int j = 1; j < N; ++j) sum = fmaf(indicator01<KIND>(v[j]), (float)(1u << j), sum);
    return (uint32_t)sum;
}

enum MaskMode { MASK_NONE = 0, MASK_WRITE = 1, MASK_READ = 2 };

// ---------------------------------------------------------------------------
// The element-wise operations.  Each has
//   In      -- the raw registers of one chunk of every input stream
//   load    -- fill In for the lane's chunk of wave tile t
//   run     -- compute and store that chunk
//   scalar  -- the same for the single element i (tail); takes / returns the mask bit
// ---------------------------------------------------------------------------

template <int KIND, int DT>
struct FwdOp {                       // y = f(x), s = [x < T]
    using S = Storage<DT, 8>;
    const void* x; void* y; uint8_t* mask;
    struct In { typename S::Raw x; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const { in.x = S::load(x, t, lane); }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float v[S::kElems]; S::unpack(in.x, v);
        const uint32_t m = indicator_bits<KIND>(v);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) v[j] = act<KIND, S::kPrec>(v[j]);
        S::store(y, t, lane, v);
        S::store_mask(mask, t, lane, m);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool) const
    {
        float v = S::load1(x, i);
        S::store1(y, i, act<KIND, S::kPrec>(v));
        return v < KindConst<KIND>::T;
    }
    static constexpr int kMask = MASK_WRITE;
    static constexpr bool kMillsTable = KIND == GELU_ERF && S::kPrec == PRECISE   /* erfcx comes from the LDS table */;
    static constexpr bool kMillsFar = false;
    static constexpr Shape kShape = pick<DT>({2, 32}, {1, 32});   // {tiles, resident cap}: binary32, bfloat16
};

template <int KIND, int DT>
struct BwdOp {                       // grad_x = grad_y * q(y, s)
    using S = Storage<DT, lean_elems<DT>()>;
    const void* y; const uint8_t* mask; const void* gy; void* gx;
    struct In { typename S::Raw y, g; uint32_t m; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const
    {
        in.y = S::load(y, t, lane); in.g = S::load(gy, t, lane); in.m = S::load_mask(mask, t, lane);
    }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float a[S::kElems], g[S::kElems]; S::unpack(in.y, a); S::unpack(in.g, g);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) g[j] = times_q<KIND, S::kPrec>(g[j], a[j], (in.m >> j) & 1u);
        S::store(gx, t, lane, g);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool bit) const
    {
        S::store1(gx, i, times_q<KIND, S::kPrec>(S::load1(gy, i), S::load1(y, i), bit));
        return bit;
    }
    static constexpr int kMask = MASK_READ;
    static constexpr bool kMillsTable = false, kMillsFar = false;
    static constexpr Shape kShape = pick<DT>({1, 24}, {1, 32});   // {tiles, resident cap}: binary32, bfloat16
};

template <int KIND, int DT>
struct GluFwdOp {                    // act = f(gate), s = [gate < T], h = f(gate) * up
    using S = Storage<DT, lean_elems<DT>()>;
    const void* gate; const void* up; void* act_out; void* h; uint8_t* mask;
    struct In { typename S::Raw g, u; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const
    {
        in.g = S::load(gate, t, lane); in.u = S::load(up, t, lane);
    }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float v[S::kElems], u[S::kElems]; S::unpack(in.g, v); S::unpack(in.u, u);
        const uint32_t m = indicator_bits<KIND>(v);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) act_times<KIND, S::kPrec>(v[j], u[j], v[j], u[j]);
        S::store(act_out, t, lane, v);
        S::store(h, t, lane, u);
        S::store_mask(mask, t, lane, m);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool) const
    {
        float v = S::load1(gate, i), u = S::load1(up, i), a, p;
        act_times<KIND, S::kPrec>(v, u, a, p);
        S::store1(act_out, i, a);
        S::store1(h, i, p);
        return v < KindConst<KIND>::T;
    }
    static constexpr int kMask = MASK_WRITE;
    static constexpr bool kMillsTable = KIND == GELU_ERF && S::kPrec == PRECISE   /* erfcx comes from the LDS table */;
    static constexpr bool kMillsFar = true;       // h = f(gate) * up needs f(gate) where it is far below binary32's range
    // {tiles, resident cap}: binary32, bfloat16; the binary32 erf form has arithmetic enough to want every slot
    static constexpr Shape kShape = pick<DT>({1, kMillsTable ? 32 : 16}, {1, 16});
};

template <int KIND, int DT>
struct GluBwdOp {                    // grad_up = grad_h * act ; grad_gate = grad_h * up * q(act, s)
    using S = Storage<DT, lean_elems<DT>()>;
    const void* act_in; const void* up; const uint8_t* mask; const void* gh; void* ggate; void* gup;
    struct In { typename S::Raw a, u, g; uint32_t m; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const
    {
        in.a = S::load(act_in, t, lane); in.u = S::load(up, t, lane); in.g = S::load(gh, t, lane);
        in.m = S::load_mask(mask, t, lane);
    }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float a[S::kElems], u[S::kElems], g[S::kElems]; S::unpack(in.a, a); S::unpack(in.u, u); S::unpack(in.g, g);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) {
            float gate_grad = times_q<KIND, S::kPrec>(g[j], u[j], a[j], (in.m >> j) & 1u);
            a[j] = g[j] * a[j];                  // grad_up
            u[j] = gate_grad;                    // grad_gate
        }
        S::store(gup, t, lane, a);
        S::store(ggate, t, lane, u);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool bit) const
    {
        float a = S::load1(act_in, i), u = S::load1(up, i), g = S::load1(gh, i);
        S::store1(gup, i, g * a);
        S::store1(ggate, i, times_q<KIND, S::kPrec>(g, u, a, bit));
        return bit;
    }
    static constexpr int kMask = MASK_READ;
    static constexpr bool kMillsTable = false, kMillsFar = false;
    static constexpr Shape kShape = pick<DT>({1, 16}, {1, 16});   // {tiles, resident cap}: binary32, bfloat16
};

// Precision-bit variant: no mask tensor, the indicator travels in bit 0 of y.
template <int KIND, int DT>
struct PbitFwdOp {                   // y = f(x) with bit 0 := [x < T]
    using S = Storage<DT, 8>;
    const void* x; void* y;
    struct In { typename S::Raw x; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const { in.x = S::load(x, t, lane); }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float v[S::kElems], ind[S::kElems]; S::unpack(in.x, v);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) { ind[j] = indicator01<KIND>(v[j]); v[j] = act<KIND, S::kPrec>(v[j]); }
        S::store_tagged(y, t, lane, v, ind);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool) const
    {
        float v = S::load1(x, i);
        S::store1_tagged(y, i, act<KIND, S::kPrec>(v), v < KindConst<KIND>::T);
        return false;
    }
    static constexpr int kMask = MASK_NONE;
    static constexpr bool kMillsTable = KIND == GELU_ERF && S::kPrec == PRECISE   /* erfcx comes from the LDS table */;
    static constexpr bool kMillsFar = false;
    static constexpr Shape kShape = pick<DT>({2, 32}, {1, 32});   // {tiles, resident cap}: binary32, bfloat16
};

template <int KIND, int DT>
struct PbitBwdOp {                   // s = bit 0 of y; grad_x = grad_y * q(y, s)
    using S = Storage<DT, lean_elems<DT>()>;
    const void* y; const void* gy; void* gx;
    struct In { typename S::Raw y, g; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const
    {
        in.y = S::load(y, t, lane); in.g = S::load(gy, t, lane);
    }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float a[S::kElems], g[S::kElems];
        const uint32_t m = S::unpack_tagged(in.y, a);
        S::unpack(in.g, g);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) g[j] = times_q<KIND, S::kPrec>(g[j], a[j], (m >> j) & 1u);
        S::store(gx, t, lane, g);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool) const
    {
        S::store1(gx, i, times_q<KIND, S::kPrec>(S::load1(gy, i), S::load1(y, i), S::lsb1(y, i)));
        return false;
    }
    static constexpr int kMask = MASK_NONE;
    static constexpr bool kMillsTable = false, kMillsFar = false;
    static constexpr Shape kShape = pick<DT>({1, 24}, {1, 32});   // {tiles, resident cap}: binary32, bfloat16
};

// Sign-bit variant: no mask tensor; the saved tensor is f(x) - min f, which is never negative, with
// the indicator in its sign bit.  Whoever consumes it adds the minimum back.
template <int KIND, int DT>
struct SbitFwdOp {                   // y_tagged = +-(f(x) - C), sign bit := [x < T]
    using S = Storage<DT, 8>;
    const void* x; void* yt;
    struct In { typename S::Raw x; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const { in.x = S::load(x, t, lane); }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float v[S::kElems]; S::unpack(in.x, v);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) v[j] = act_minus_min_signed<KIND, S::kPrec>(v[j]);
        S::store(yt, t, lane, v);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool) const
    {
        S::store1(yt, i, act_minus_min_signed<KIND, S::kPrec>(S::load1(x, i)));
        return false;
    }
    static constexpr int kMask = MASK_NONE;
    static constexpr bool kMillsTable = KIND == GELU_ERF && S::kPrec == PRECISE   /* erfcx comes from the LDS table */;
    static constexpr bool kMillsFar = false;
    static constexpr Shape kShape = pick<DT>({2, 32}, {1, 32});   // {tiles, resident cap}: binary32, bfloat16
};

template <int KIND, int DT>
struct SbitDecodeOp {                // y = |y_tagged| + C
    using S = Storage<DT, lean_elems<DT>()>;
    const void* yt; void* y;
    struct In { typename S::Raw y; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const { in.y = S::load(yt, t, lane); }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float v[S::kElems]; S::unpack(in.y, v);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) v[j] = fabsf(v[j]) + KindConst<KIND>::fT;
        S::store(y, t, lane, v);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool) const
    {
        S::store1(y, i, fabsf(S::load1(yt, i)) + KindConst<KIND>::fT);
        return false;
    }
    static constexpr int kMask = MASK_NONE;
    static constexpr bool kMillsTable = false, kMillsFar = false;
    static constexpr Shape kShape = pick<DT>({2, 20}, {1, 32});   // {tiles, resident cap}: binary32, bfloat16
};

template <int KIND, int DT>
struct SbitBwdOp {                   // s = sign bit of y_tagged; grad_x = grad_y * q(|y_tagged| + C, s)
    using S = Storage<DT, lean_elems<DT>()>;
    const void* yt; const void* gy; void* gx;
    struct In { typename S::Raw y, g; };
    __device__ __forceinline__ void load(In& in, size_t t, unsigned lane) const
    {
        in.y = S::load(yt, t, lane); in.g = S::load(gy, t, lane);
    }
    static __device__ __forceinline__ float one(float g, float t)
    {
        return times_q<KIND, S::kPrec>(g, fabsf(t) + KindConst<KIND>::fT, (__float_as_uint(t) >> 31) != 0);
    }
    __device__ __forceinline__ void run(const In& in, size_t t, unsigned lane) const
    {
        float a[S::kElems], g[S::kElems];
        S::unpack(in.y, a);
        S::unpack(in.g, g);
#pragma unroll
        for (int j = 0; j < S::kElems; ++j) g[j] = one(g[j], a[j]);
        S::store(gx, t, lane, g);
    }
    __device__ __forceinline__ bool scalar(size_t i, bool) const
    {
        S::store1(gx, i, one(S::load1(gy, i), S::load1(yt, i)));
        return false;
    }
    static constexpr int kMask = MASK_NONE;
    static constexpr bool kMillsTable = false, kMillsFar = false;
    static constexpr Shape kShape = pick<DT>({1, 24}, {1, 32});   // {tiles, resident cap}: binary32, bfloat16
};

// ---------------------------------------------------------------------------
// Skeleton
// ---------------------------------------------------------------------------

// A workgroup is one wavefront -- or four, for the operations that read the erfcx table: they share one copy
// of it in LDS, which costs each of them a quarter of the copying.  PERSISTENT: the grid strides over the wave
// tiles (a fixed number of workgroups per compute unit).  Otherwise every wavefront handles kUnroll consecutive
// wave tiles and retires, and the dispatcher balances the load.  The tile index comes from the workgroup (and
// wavefront) index, so every branch below is wave-uniform (the neighbour swap of the binary32 mask needs whole
// quads) and tile addresses stay in scalar registers.
template <class Op> constexpr int kGroupWaves = Op::kMillsTable ? 4 : 1;

template <class Op, bool PERSISTENT>
__global__ __launch_bounds__(kWave * kGroupWaves<Op>) void stream_kernel(const Op op, const size_t n)
{
    constexpr int kUnroll = Op::kShape.unroll;
    constexpr size_t kWaveTile = Op::S::kWaveTile;
    constexpr unsigned kWaves = kGroupWaves<Op>;
    const size_t wave_tiles = n / kWaveTile;
    const unsigned lane = threadIdx.x % kWave;
    // which wavefront of the grid this is (uniform over the wavefront: make the compiler see it)
    const size_t wave = kWaves == 1 ? (size_t)blockIdx.x
                                    : (size_t)blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    if constexpr (Op::kMillsTable) fill_mills_table<Op::kMillsFar>(threadIdx.x, kWave * kWaves);

    if constexpr (PERSISTENT) {
        const size_t stride = (size_t)gridDim.x * kWaves;
        size_t t = wave;
        for (; t + (kUnroll - 1) * stride < wave_tiles; t += kUnroll * stride) {
            typename Op::In in[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) op.load(in[u], t + u * stride, lane);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) op.run(in[u], t + u * stride, lane);
        }
        for (; t < wave_tiles; t += stride) {
            typename Op::In in;
            op.load(in, t, lane);
            op.run(in, t, lane);
        }
    } else {
        const size_t t = wave * kUnroll;
        if (t + kUnroll <= wave_tiles) {
            typename Op::In in[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) op.load(in[u], t + u, lane);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) op.run(in[u], t + u, lane);
        } else {
            for (int u = 0; u < kUnroll; ++u) {
                if (t + u < wave_tiles) {
                    typename Op::In in;
                    op.load(in, t + u, lane);
                    op.run(in, t + u, lane);
                }
            }
        }
    }

    // Tail: elements [kWaveTile wave_tiles, n), one per lane, by the first wavefront.
    // Whole 64-bit mask words are written (read), so the zero padding of the
    // last word comes from the ballot itself.
    if (wave == 0) {
        for (size_t base = wave_tiles * kWaveTile; base < n; base += 64) {
            const size_t i = base + lane;
            if constexpr (Op::kMask == MASK_WRITE) {
                bool bit = false;
                if (i < n) bit = op.scalar(i, false);
                const uint64_t word = __builtin_amdgcn_ballot_w64(bit);
                if (lane == 0) reinterpret_cast<uint64_t*>(op.mask)[base / 64] = word;
            } else if constexpr (Op::kMask == MASK_READ) {
                const uint64_t word = reinterpret_cast<const uint64_t*>(op.mask)[base / 64];
                if (i < n) op.scalar(i, (word >> lane) & 1u);
            } else {
                if (i < n) op.scalar(i, false);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------

std::atomic<int> g_blocks_per_cu{kDefaultBlocksPerCu};
std::atomic<int> g_cu_count[64];            // per device, 0 = not queried yet
std::atomic<int> g_resident_override{0};     // 0: every operation uses its own kShape.resident
constexpr unsigned kLdsPerCu = 160 * 1024;

int cu_count()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = g_cu_count[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        g_cu_count[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Bytes of (unused) dynamic LDS that keep at most `resident` wavefronts of a
// kernel on one compute unit (whole workgroups, where a workgroup is several);
// the kernel is told once per device that it may be launched with that much.
template <class Op>
unsigned occupancy_cap_lds(int resident)
{
    if (resident <= 0 || resident >= kWaveSlotsPerCu) return 0;   // the hardware's own limit
    static std::atomic<uint64_t> prepared{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (!(prepared.load(std::memory_order_acquire) >> dev & 1)) {
        // what the kernel declares itself (the erfcx table) counts against the same 160 KiB
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(stream_kernel<Op, false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)(kLdsPerCu - (Op::kMillsTable ? (unsigned)kMillsTableBytes<Op::kMillsFar> : 0u))) != hipSuccess)
            return 0;
        prepared.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    }
    const unsigned groups = (unsigned)resident / kGroupWaves<Op> ? (unsigned)resident / kGroupWaves<Op> : 1u;
    const unsigned share = kLdsPerCu / groups, own = Op::kMillsTable ? (unsigned)kMillsTableBytes<Op::kMillsFar> : 0u;
    return share > own ? share - own : 0;
}

// Enqueues one launch and reports THIS launch's status: the runtime's return value, not the
// thread's last-error slot, which may still hold (and would clear) an error of the caller's own work.
template <class Op>
int enqueue(void (*kernel)(Op, size_t), unsigned blocks, unsigned threads, unsigned lds, hipStream_t stream,
            Op op, size_t n)
{
    void* args[] = {&op, &n};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), dim3(blocks), dim3(threads), args, lds, stream)
               == hipSuccess ? INVACT_OK : INVACT_ERR_HIP;
}

template <class Op>
int launch(const Op& op, size_t n, hipStream_t stream)
{
    constexpr int kUnroll = Op::kShape.unroll;
    const size_t wave_tiles = n / Op::S::kWaveTile;
    const int per_cu = g_blocks_per_cu.load(std::memory_order_relaxed);
    if (per_cu == 0) {
        constexpr size_t per_block = (size_t)kUnroll * kGroupWaves<Op>;
        size_t blocks = (wave_tiles + per_block - 1) / per_block;
        if (blocks == 0) blocks = 1;                          // the tail still needs a wavefront
        if (blocks > 0x7FFFFFFFu) return INVACT_ERR_SIZE;
        const int forced = g_resident_override.load(std::memory_order_relaxed);
        const unsigned lds = occupancy_cap_lds<Op>(forced ? forced : Op::kShape.resident);
        return enqueue(stream_kernel<Op, false>, (unsigned)blocks, kWave * kGroupWaves<Op>, lds, stream, op, n);
    } else {
        size_t blocks = (wave_tiles + kGroupWaves<Op> - 1) / kGroupWaves<Op>;
        const size_t cap = (size_t)cu_count() * (size_t)per_cu;
        if (blocks > cap) blocks = cap;
        if (blocks == 0) blocks = 1;
        return enqueue(stream_kernel<Op, true>, (unsigned)blocks, kWave * kGroupWaves<Op>, 0, stream, op, n);
    }
}

// Runs fn<KIND, DT>() for the run-time (kind, dtype) pair.
template <class F>
int dispatch(int kind, int dtype, F&& fn)
{
#define INVACT_CASE(K, D) if (kind == K && dtype == D) return fn(std::integral_constant<int, K>{}, std::integral_constant<int, D>{});
    INVACT_CASE(INVACT_GELU_TANH, INVACT_FP32) INVACT_CASE(INVACT_GELU_TANH, INVACT_BF16)
    INVACT_CASE(INVACT_GELU_ERF,  INVACT_FP32) INVACT_CASE(INVACT_GELU_ERF,  INVACT_BF16)
    INVACT_CASE(INVACT_SILU,      INVACT_FP32) INVACT_CASE(INVACT_SILU,      INVACT_BF16)
#undef INVACT_CASE
    return INVACT_ERR_KIND;
}

int check_common(int kind, int dtype, size_t n)
{
    if (kind != INVACT_GELU_TANH && kind != INVACT_GELU_ERF && kind != INVACT_SILU) return INVACT_ERR_KIND;
    if (dtype != INVACT_FP32 && dtype != INVACT_BF16) return INVACT_ERR_DTYPE;
    if (n > SIZE_MAX - 63) return INVACT_ERR_SIZE;
    return INVACT_OK;
}

int check_data(std::initializer_list<const void*> data)
{
    for (const void* p : data) if (p == nullptr) return INVACT_ERR_NULL;
    for (const void* p : data) if (!aligned(p, 16)) return INVACT_ERR_ALIGN;
    return INVACT_OK;
}

int check_ptrs(std::initializer_list<const void*> data, const void* mask)
{
    for (const void* p : data) if (p == nullptr) return INVACT_ERR_NULL;
    if (mask == nullptr) return INVACT_ERR_NULL;
    for (const void* p : data) if (!aligned(p, 16)) return INVACT_ERR_ALIGN;
    if (!aligned(mask, 8)) return INVACT_ERR_ALIGN;
    return INVACT_OK;
}

}  // namespace

extern "C" {

size_t invact_mask_bytes(size_t n) { return 8 * (n / 64 + (n % 64 != 0)); }

const char* invact_strerror(int status)
{
    switch (status) {
    case INVACT_OK:        return "success";
    case INVACT_ERR_KIND:  return "unknown activation kind";
    case INVACT_ERR_DTYPE: return "unknown dtype";
    case INVACT_ERR_NULL:  return "null pointer argument";
    case INVACT_ERR_ALIGN: return "pointer not aligned (16 bytes for tensors, 8 for the mask)";
    case INVACT_ERR_SIZE:  return "size not accepted: too large, not the multiple the entry point asks for, or a workspace too small";
    case INVACT_ERR_HIP:   return "HIP runtime error at kernel launch";
    }
    return "unknown status";
}

int invact_set_blocks_per_cu(int blocks_per_cu)
{
    if (blocks_per_cu < 0 || blocks_per_cu > 64) return -1;
    g_blocks_per_cu.store(blocks_per_cu == 0 ? kDefaultBlocksPerCu : blocks_per_cu, std::memory_order_relaxed);
    return blocks_per_cu;
}

int invact_set_resident_blocks(int blocks)
{
    if (blocks < 0 || blocks > 32) return -1;
    g_resident_override.store(blocks, std::memory_order_relaxed);
    return blocks;
}

int invact_fwd(int kind, int dtype, const void* x, void* y, void* mask, size_t n, hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_ptrs({x, y}, mask)) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(FwdOp<K.value, D.value>{x, y, static_cast<uint8_t*>(mask)}, n, stream);
    });
}

int invact_bwd(int kind, int dtype, const void* y, const void* mask, const void* grad_y,
               void* grad_x, size_t n, hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_ptrs({y, grad_y, grad_x}, mask)) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(BwdOp<K.value, D.value>{y, static_cast<const uint8_t*>(mask), grad_y, grad_x}, n, stream);
    });
}

int geglu_invact_fwd(int kind, int dtype, const void* gate, const void* up, void* act, void* h,
                     void* mask, size_t n, hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_ptrs({gate, up, act, h}, mask)) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(GluFwdOp<K.value, D.value>{gate, up, act, h, static_cast<uint8_t*>(mask)}, n, stream);
    });
}

int geglu_invact_bwd(int kind, int dtype, const void* act, const void* up, const void* mask,
                     const void* grad_h, void* grad_gate, void* grad_up, size_t n, hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_ptrs({act, up, grad_h, grad_gate, grad_up}, mask)) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(GluBwdOp<K.value, D.value>{act, up, static_cast<const uint8_t*>(mask), grad_h,
                                                 grad_gate, grad_up}, n, stream);
    });
}

int invact_pbit_fwd(int kind, int dtype, const void* x, void* y, size_t n, hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_data({x, y})) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(PbitFwdOp<K.value, D.value>{x, y}, n, stream);
    });
}

int invact_pbit_bwd(int kind, int dtype, const void* y, const void* grad_y, void* grad_x, size_t n,
                    hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_data({y, grad_y, grad_x})) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(PbitBwdOp<K.value, D.value>{y, grad_y, grad_x}, n, stream);
    });
}

int invact_sbit_fwd(int kind, int dtype, const void* x, void* y_tagged, size_t n, hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_data({x, y_tagged})) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(SbitFwdOp<K.value, D.value>{x, y_tagged}, n, stream);
    });
}

int invact_sbit_decode(int kind, int dtype, const void* y_tagged, void* y, size_t n, hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_data({y_tagged, y})) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(SbitDecodeOp<K.value, D.value>{y_tagged, y}, n, stream);
    });
}

int invact_sbit_bwd(int kind, int dtype, const void* y_tagged, const void* grad_y, void* grad_x, size_t n,
                    hipStream_t stream)
{
    if (int e = check_common(kind, dtype, n)) return e;
    if (n == 0) return INVACT_OK;
    if (int e = check_data({y_tagged, grad_y, grad_x})) return e;
    return dispatch(kind, dtype, [&](auto K, auto D) {
        return launch(SbitBwdOp<K.value, D.value>{y_tagged, grad_y, grad_x}, n, stream);
    });
}

int swiglu_invact_fwd(int dtype, const void* gate, const void* up, void* act, void* h, void* mask,
                      size_t n, hipStream_t stream)
{
    return geglu_invact_fwd(INVACT_SILU, dtype, gate, up, act, h, mask, n, stream);
}

int swiglu_invact_bwd(int dtype, const void* act, const void* up, const void* mask, const void* grad_h,
                      void* grad_gate, void* grad_up, size_t n, hipStream_t stream)
{
    return geglu_invact_bwd(INVACT_SILU, dtype, act, up, mask, grad_h, grad_gate, grad_up, n, stream);
}

}  // extern "C"
