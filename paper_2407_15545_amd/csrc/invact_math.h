// Device-side arithmetic of the Inverted-Activations kernels (gfx950).
//
// Two precision policies exist for the forward activation:
//   FAST    -- binary32 throughout, hardware exp2 / rcp / sqrt (each within one
//              ulp) and short polynomials; far more accurate than a bfloat16
//              store can show.  Used when the storage dtype is bfloat16.
//   PRECISE -- everything up to one final rounding in binary64 (a little over half
//              the binary32 rate on this chip): 2^t from an exact split of t and a
//              polynomial, reciprocals from a binary32 seed and one Newton step,
//              erfcx from a table of short polynomials in LDS.  Used when the
//              storage dtype is binary32, where a binary32 exponent argument alone
//              would cost 5-70 ulp in the left tail.
// The backward approximation q (Eqs. (5)-(8)) is evaluated in binary32 for both
// dtypes; for binary32 storage its product with the gradient is rounded once.
//
// Rough cost model measured on MI355X (lanes per clock and compute unit):
// v_add/mul/fma_f32 ~100, other VALU incl. binary64 fma/mul/add and conversions
// ~60, v_exp/rcp/sqrt_f32 ~31, v_rcp_f64 ~16.
#pragma once

#include <hip/hip_runtime.h>
#include <float.h>

#include "invact_constants.h"

namespace invact_dev {

enum Kind { GELU_TANH = 0, GELU_ERF = 1, SILU = 2 };
enum Prec { FAST = 0, PRECISE = 1 };

namespace cst = invact_const;

__device__ __forceinline__ float hw_exp2(float v) { return __builtin_amdgcn_exp2f(v); }   // v_exp_f32
__device__ __forceinline__ float hw_rcp(float v)  { return __builtin_amdgcn_rcpf(v); }    // v_rcp_f32
__device__ __forceinline__ float hw_sqrt(float v) { return __builtin_amdgcn_sqrtf(v); }   // v_sqrt_f32
// median of three: clamps v to [lo, hi]; a NaN comes out as lo
__device__ __forceinline__ float med3(float v, float lo, float hi) { return __builtin_amdgcn_fmed3f(v, lo, hi); }

constexpr float  kLog2e       = 1.44269504088896340736f;
constexpr double kLog2eD      = 1.44269504088896340736;
constexpr double kLn2D        = 0.69314718055994530942;
constexpr double kSqrt2OverPi = 0.79788456080286535588;   // sqrt(2/pi)
constexpr double kGeluCubic   = 0.044715;
constexpr double kInvSqrt2    = 0.70710678118654752440;

// The branch threshold T (minimiser of f) and f(T), rounded to binary32.
template <int KIND> struct KindConst;
template <> struct KindConst<GELU_TANH> { static constexpr float T = cst::T_gelu_tanh, fT = cst::fT_gelu_tanh; };
template <> struct KindConst<GELU_ERF>  { static constexpr float T = cst::T_gelu_erf,  fT = cst::fT_gelu_erf; };
template <> struct KindConst<SILU>      { static constexpr float T = cst::T_silu,      fT = cst::fT_silu; };

// All three activations are written as
//     f(x) = max(x, -0) - |u|,   u = x * P(-|x|),
// with P the gate evaluated on the negative side (sigmoid(-|z|) or Phi(-|x|)):
// for x < 0 this is u itself, for x >= 0 it is x - x P(-|x|) = x P(|x|).  One
// formula, no select, and -inf, -0 and +inf come out as -0, -0 and +inf.

// ---------------------------------------------------------------------------
// Forward, FAST
// ---------------------------------------------------------------------------

// x * sigmoid(-|z|) from th = -|z| log2(e) / 2.  With Eh = exp(-|z|/2) the gate
// is Eh^2 / (1 + Eh^2); the product is taken as (x Eh) * (Eh r) so that no
// factor is subnormal while the result is still a normal number (x ~ -90 for
// SiLU).  A NaN x arrives through th.
__device__ __forceinline__ float x_gate_fast(float x, float th)
{
    float Eh = hw_exp2(th);
    float r  = hw_rcp(fmaf(Eh, Eh, 1.0f));
    return (med3(x, -FLT_MAX, FLT_MAX) * Eh) * (Eh * r);
}

template <int KIND>
__device__ __forceinline__ float act_fast(float x)
{
    float u;
    if constexpr (KIND == SILU) {
        u = x_gate_fast(x, -fabsf(x) * (0.5f * kLog2e));
    } else if constexpr (KIND == GELU_TANH) {
        // z = 2u', u' = sqrt(2/pi) (x + 0.044715 x^3):  |z| log2(e) / 2 = |x (k1 + k2 x^2)|
        constexpr float k1 = (float)(kSqrt2OverPi * kLog2eD);
        constexpr float k2 = (float)(kSqrt2OverPi * kLog2eD * kGeluCubic);
        u = x_gate_fast(x, -fabsf(x * fmaf(k2, x * x, k1)));
    } else {
        // Phi(-|x|) = erfc(z) / 2 = erfcx(z) exp(-z^2) / 2 with z = |x| / sqrt 2; the result is
        // max(x, -0) - |x| Phi(-|x|) as one fused multiply-add.  |x| is clamped so that an infinite x meets
        // Phi = 0 as a finite factor; a NaN x arrives through w.
        constexpr float pz = (float)(cst::erfcx_fast_p * kInvSqrt2);
        constexpr int deg = sizeof(cst::erfcx_fast) / sizeof(cst::erfcx_fast[0]) - 1;
        float w = hw_rcp(fmaf(pz, fabsf(x), 1.0f));
        float g = 0.5f * cst::erfcx_fast[deg];
#pragma unroll
        for (int k = deg - 1; k >= 0; --k) g = fmaf(g, w, 0.5f * cst::erfcx_fast[k]);
        float E = hw_exp2((x * x) * (-0.5f * kLog2e));            // exp(-z^2)
        return fmaf(-med3(fabsf(x), 0.0f, FLT_MAX), (g * w) * E, med3(x, -0.0f, fabsf(x)));
    }
    // max(x, -0) as the median of (x, -0, |x|): one instruction (a median against the constant +inf is
    // rewritten by the compiler into a maximum preceded by a canonicalising v_max x, x).  A NaN x comes through u.
    return med3(x, -0.0f, fabsf(x)) - fabsf(u);
}

// ---------------------------------------------------------------------------
// Forward, PRECISE
// ---------------------------------------------------------------------------

// erfcx by table, for the erf form with binary32 storage.  G(x) = Phi(-x) exp(x^2 / 2) = erfcx(x / sqrt 2) / 2 is
// smooth and slowly varying, so on [0, 14.5) -- beyond, x Phi(-x) is below half the smallest binary32 subnormal --
// 116 intervals of width 1/8 with a degree-4 polynomial each reach 3e-9.  The interval index and the position
// inside it come from 8 |x| with one conversion and one v_fract_f32, both exact, and the five coefficients from
// LDS: 10 slow-rate instructions less per element than the reciprocal-based fit (1 / (1 + p z) to 2^-30 needs a
// Newton step in binary64, and its polynomial twice the degree).  A row is two 128-bit reads: c0 and c1 in
// binary64, and c2, c3, c4, whose terms are below G / 64, in binary32 (c2 + t (c3 + t c4) is evaluated in
// binary32, at the full rate, the rest in binary64); LDS traffic is what this costs, so the row is kept short,
// and its two halves live in two arrays of 16-byte entries: lanes that read different rows then spread over
// all eight groups of four banks.
// Every workgroup copies its part of the table from global memory (3712 or 5120 bytes, L2-resident) into its LDS before its first
// element: a twentieth of the kernel's time with one wavefront per workgroup, which is why these kernels run four.
// Two lengths: FAR = false, 116 rows, |x| < 14.5, for the kernels that store f(x) alone; FAR = true, all 160 rows,
// |x| < 20, for the gated forward, whose product f(gate) * up can still be a binary32 number where f(gate) alone
// has long rounded to -0 (|up| goes up to 3.4e38; beyond -20 even that product is below half a subnormal).
static __device__ __attribute__((aligned(16))) const uint32_t g_mills_table[cst::mills_rows * 8] = { INVACT_MILLS_TABLE };
template <bool FAR> constexpr int kMillsRows = FAR ? cst::mills_rows : cst::mills_rows_near;
template <bool FAR> constexpr int kMillsTableBytes = kMillsRows<FAR> * 32;
template <bool FAR> constexpr float kMillsClamp = FAR ? 19.99f : 14.49f;          // 8 * clamp < rows

typedef uint32_t mills_piece_t __attribute__((ext_vector_type(4)));      // (c0, c1) or (c2, c3, c4, -) of a row

template <bool FAR>
__device__ __forceinline__ mills_piece_t* mills_lds()
{
    __shared__ mills_piece_t table[kMillsRows<FAR> * 2];
    return table;
}

// The whole workgroup (`threads` of them, `thread` = threadIdx.x) fills the LDS copy: the first kMillsRows<FAR>
// entries of either half of the table.
template <bool FAR>
__device__ __forceinline__ void fill_mills_table(unsigned thread, unsigned threads)
{
    const mills_piece_t* src = reinterpret_cast<const mills_piece_t*>(g_mills_table);
    mills_piece_t* dst = mills_lds<FAR>();
    constexpr unsigned R = kMillsRows<FAR>;
    for (unsigned k = thread; k < 2u * R; k += threads) dst[k] = src[k < R ? k : k - R + cst::mills_rows];
    __syncthreads();
}

// 2^(a b) for a binary64 product t = a b in [-30000, 0]:  t = n + f with n = round(t), |f| <= 1/2,
// 2^f by a degree-6 polynomial (relative error 2.6e-9: the hardware exponential's 0.78 ulp of binary32
// would be the largest error of the whole forward; its last two steps in binary64), and the scaling by 2^n
// exact (v_ldexp_f64, no subnormal binary32 intermediate).  n comes from adding 1.5 * 2^52: the sum
// is rounded to an integer, and since the low 32 bits of that constant's significand are zero the
// low word of the sum is n itself in two's complement.  Both uses of the product are fused
// (fma(a, b, .)), so the product is never rounded on its own and costs no instruction.  A NaN gives NaN.
__device__ __forceinline__ double exp2_neg(double a, double b)
{
    constexpr double kRound = 6755399441055744.0;        // 1.5 * 2^52
    double s = fma(a, b, kRound);
    double f = fma(a, b, kRound - s);                    // kRound - s = -n exactly
    // the terms from f^2 on are below 0.07 of the result: binary32 is enough for them (a tenth of an ulp of the
    // result), at the full rate and a fraction of the power of binary64
    const float ff = (float)f;
    float q = (float)cst::exp2_precise[6];
#pragma unroll
    for (int k = 5; k >= 2; --k) q = fmaf(q, ff, (float)cst::exp2_precise[k]);
    const double p = fma(fma((double)q, f, cst::exp2_precise[1]), f, cst::exp2_precise[0]);
    return ldexp(p, __double2loint(s));
}

// 1 / d for d in [1, 16], to about 2^-44: binary32 seed, one Newton step in binary64.
__device__ __forceinline__ double rcp_newton(double d)
{
    double r = (double)hw_rcp((float)d);
    return r * fma(-d, r, 2.0);
}

// The gate on the negative side in binary64: P = sigmoid(-|z|) or Phi(-|x|), and the clamped x it was computed
// from (|x| is clamped where P is exactly 0 anyway, so that an infinite x meets that 0 as a finite factor).
// The clamp drops a NaN; act_precise lets it through by its other operand.
struct Gate { double P; float xc; };

template <int KIND, bool FAR = false>
__device__ __forceinline__ Gate gate_precise(float x)
{
    Gate out;
    if constexpr (KIND == SILU) {
        out.xc = med3(x, -2048.0f, 2048.0f);                   // beyond, the gate underflows to 0 anyway
        double E  = exp2_neg(-fabs((double)out.xc), kLog2eD);
        out.P = E * rcp_newton(1.0 + E);
    } else if constexpr (KIND == GELU_TANH) {
        constexpr double a = 2.0 * kSqrt2OverPi * kLog2eD, b = a * kGeluCubic;
        out.xc = med3(x, -64.0f, 64.0f);
        double xd = (double)out.xc;
        double E  = exp2_neg(-fabs(xd), fma(b, xd * xd, a));     // a, b > 0
        out.P = E * rcp_newton(1.0 + E);
    } else {
        // G from the table (see above), times exp(-x^2 / 2).  Beyond the clamp x Phi(-x) rounds to -0 or leaves x
        // as it is, with the clamped P as with the true one.
        static_assert(kMillsClamp<FAR> * cst::mills_per_unit < kMillsRows<FAR>, "the clamp keeps the row index inside the table");
        out.xc = med3(x, -kMillsClamp<FAR>, kMillsClamp<FAR>);
        double xd = (double)out.xc;
        float m = fabsf(out.xc) * (float)cst::mills_per_unit;
        const mills_piece_t* row = mills_lds<FAR>() + (unsigned)m;                       // truncation: the interval
        const float tf = __builtin_amdgcn_fractf(m);                                // position inside it, exact
        typedef double double2_t __attribute__((ext_vector_type(2)));
        typedef float float4_t __attribute__((ext_vector_type(4)));
        const double2_t lo = __builtin_bit_cast(double2_t, row[0]);                 // c0, c1
        const float4_t hi = __builtin_bit_cast(float4_t, row[kMillsRows<FAR>]);     // c2, c3, c4, -
        const float q = fmaf(fmaf(hi[2], tf, hi[1]), tf, hi[0]);
        const double t = (double)tf, c0 = lo[0], c1 = lo[1];
        double g = fma(fma((double)q, t, c1), t, c0);
        out.P = g * exp2_neg(xd * (-0.5 * kLog2eD), xd);
    }
    return out;
}

// f(x) - minus = (max(x, -0) - minus) - |x| P in binary64, one fused multiply-add: what the gated product
// (minus = 0) and the sign-bit variant (minus = min f) start from.
template <int KIND, bool FAR = false>
__device__ __forceinline__ double act_precise(float x, double minus = 0.0)
{
    Gate g = gate_precise<KIND, FAR>(x);
    // max(x, -0) as a select, which lets a NaN x through where a maximum would drop it: the result is then a
    // NaN, and a quiet one (the conversions quiet it), so that the precision-bit variant, which rewrites bit 0 of
    // the stored pattern, cannot turn the signalling NaNs 0x7F800001 / 0xFF800001 into infinities
    const float positive_part = (x < 0.0f) ? -0.0f : x;
    return fma(-fabs((double)g.xc), g.P, (double)positive_part - minus);
}


// f(x) rounded once to binary32.
template <int KIND, int PREC>
__device__ __forceinline__ float act(float x)
{
    if constexpr (PREC == FAST) return act_fast<KIND>(x);
    else return (float)act_precise<KIND>(x);
}

// f(gate) and f(gate) * up, each rounded once (the product is formed from the
// unrounded activation).
template <int KIND, int PREC>
__device__ __forceinline__ void act_times(float gate, float up, float& a, float& h)
{
    if constexpr (PREC == FAST) {
        a = act_fast<KIND>(gate);
        h = a * up;
    } else {
        double ad = act_precise<KIND, true>(gate);         // the far table: see g_mills_table
        a = (float)ad;
        h = (float)(ad * (double)up);
    }
}

// Sign-bit variant (Section 3.3): f(x) - C with C = f(T) the minimum of f, clamped at 0 (the
// difference is negative only by the rounding of C), rounded once to binary32, with its sign bit
// set to the indicator [x < T].  A NaN x gives a NaN.
template <int KIND, int PREC>
__device__ __forceinline__ float act_minus_min_signed(float x)
{
    constexpr float C = KindConst<KIND>::fT;
    float v;
    if constexpr (PREC == FAST) {
        float d = act_fast<KIND>(x) - C;
        v = (d < 0.0f) ? 0.0f : d;                      // keeps a NaN
    } else {
        // max(x, -0) - C is exact in binary64 wherever it matters (for |x| > 2^28 the result rounds to x anyway),
        // so f(x) - C still sees one rounding before the store.  The clamp comes after it, as a select that keeps
        // a NaN; the difference is never a negative zero (the fused multiply-add rounds an exact, non-zero value
        // of at least 2^-110, or gives +0), so a sign bit cannot survive it.
        v = (float)act_precise<KIND>(x, (double)C);
        v = (v < 0.0f) ? 0.0f : v;
    }
    // |v| = v for every number here; for a NaN it clears the sign the NaN came with, so that the stored sign bit
    // is the indicator (0 for a NaN) for every input.  A source modifier of the select: no instruction.
    return (x < KindConst<KIND>::T) ? -v : __builtin_fabsf(v);
}

// ---------------------------------------------------------------------------
// Backward: q(y, s) ~ f'(f^-1(y)), Eqs. (5)-(8)
// ---------------------------------------------------------------------------

// 2^(log2(e) c3 (c4 - yt)^3) by Horner's rule on the expanded cubic.
__device__ __forceinline__ float cubic_exp2(const float (&t)[4], float yt)
{
    return hw_exp2(fmaf(fmaf(fmaf(t[3], yt, t[2]), yt, t[1]), yt, t[0]));
}

// The pieces of q one evaluation produces:
//   ql     q_left(y)                                        (Eq. (5) / Eq. (7))
//   qr     q_right(y), summed so that the terms which cancel near y = f(T)
//          (where q_right passes through zero) meet in fused operations
//   small  q_right(y) - 1, i.e. h (GELU) or h (1 - y) (SiLU), with a relative
//          error of a few ulp of ITSELF: the better representation once |small|
//          is well below 1 (q near or above 1)
// Clamps are NaN-dropping medians (one instruction each), so a NaN y leaves qr
// finite; ql is NaN for a NaN y (through the 2y term / the + y term), and the
// callers select ql whenever y is NaN.  yt is clamped to [0, 64]: the
// exponential factor is exactly 0 beyond, and +inf must not meet that 0.
struct QParts { float ql, qr, small; };

template <int KIND, int PREC>
__device__ __forceinline__ QParts q_parts(float y, bool left)
{
    constexpr float fT = KindConst<KIND>::fT;
    QParts out;
    if constexpr (KIND == SILU) {
        const auto& L = cst::silu_left;
        const auto& R = cst::silu_right;
        (void)left;
        float yc = med3(y, 64.0f, -fabsf(y));        // min(y, 64) as a median the compiler leaves alone (cf. act_fast)
        float yt = med3(y - fT, 0.0f, 64.0f);
        float sq = hw_sqrt(yt);
        // Eq. (8) as 1 + h (1 - y), h = (c0 + r) E
        float E = cubic_exp2(cst::silu_right_exp2, yt);
        float r = fmaf(R[2], yt, R[1] * sq);
        float h = fmaf(r, E, R[0] * E);
        out.qr    = fmaf(-yc, h, fmaf(r, E, fmaf(R[0], E, 1.0f)));
        out.small = h * (1.0f - yc);
        // Eq. (7): (c0 + c1 sqrt(yt) + c2 yt + c3 yt^2) (1 - y) + y   (y itself: a NaN must show here)
        float A = fmaf(yt, fmaf(L[3], yt, L[2]), fmaf(L[1], sq, L[0]));
        out.ql = fmaf(A, 1.0f - y, y);
    } else {
        const auto& L = cst::gelu_left;
        const auto& R = cst::gelu_right;
        // Each element needs one of sqrt(y + c1) (Eq. (5)) and sqrt(y - f(T))
        // (Eq. (6)): pick the addend by the branch bit and take one root.
        float arg = med3(y + (left ? L[1] : -fT), 0.0f, 64.0f);
        float sq  = hw_sqrt(arg);
        // Eq. (6): 1 + (c0 + c1 sqrt(yt) + c2 yt) E, with yt = arg
        float E = cubic_exp2(cst::gelu_right_exp2, arg);
        if constexpr (PREC == FAST) {
            // 1 + (c0 + c1 sqrt(yt) + c2 yt) E as written: three operations; the rounding of the bracket is far
            // below a bfloat16 ulp even where the sum passes through zero
            out.qr    = fmaf(fmaf(R[2], arg, fmaf(R[1], sq, R[0])), E, 1.0f);
            out.small = 0.0f;                                   // not used
        } else {
            // the same sum with E multiplied in first: the partial sums stay below 1,
            // where binary32 is twice as fine as at c1 sqrt(yt) ~ 1
            float sE = sq * E, c2y = R[2] * arg;
            out.qr    = fmaf(R[1], sE, fmaf(c2y, E, fmaf(R[0], E, 1.0f)));
            out.small = fmaf(R[1], sE, fmaf(c2y, E, R[0] * E));
        }
        // Eq. (5): c0 sqrt(y + c1) (2y + c2 sqrt(-y)) (|c3 y^2 + |c4 y + c5| + c6| + c7)
        // The factor 2 of the middle bracket goes to c0 (exact: the results are the same bit for bit), which
        // saves the doubling of y; with bfloat16 storage c0 goes on into the last bracket (its constants are
        // rounded once more, which costs an ulp of binary32), which saves a product.
        float s2 = hw_sqrt(med3(-y, 0.0f, FLT_MAX));
        float B  = fmaf(0.5f * L[2], s2, y);
        if constexpr (PREC == FAST) {
            constexpr float k = 2.0f * L[0];                    // positive: it passes through both absolute values
            float inner = fabsf(fmaf(k * L[4], y, k * L[5]));
            float outer = fabsf(fmaf(k * L[3], y * y, inner) + k * L[6]) + k * L[7];
            out.ql = sq * B * outer;
        } else {
            float inner = fabsf(fmaf(L[4], y, L[5]));
            float outer = fabsf(fmaf(L[3], y * y, inner) + L[6]) + L[7];
            out.ql = ((2.0f * L[0]) * sq) * B * outer;
        }
    }
    return out;
}

// The product of q(y, s) with the incoming gradient.
//
// FAST (bfloat16 storage): plain products; every rounding is far below the
// store's.
// PRECISE (binary32 storage): q is kept as base + delta with
//   (base, delta) = (ql, 0) on the left branch,
//                   (qr, 0) on the right branch while |small| >= 1/4,
//                   (1, small) otherwise,
// and the product with g is rounded once.  Where q is near 1 a rounded q would
// by itself cost half an ulp of the two the result may be off by.

// grad * q  (invact_bwd)
template <int KIND, int PREC>
__device__ __forceinline__ float times_q(float g, float y, bool left)
{
    QParts p = q_parts<KIND, PREC>(y, left);
    const bool take_left = left || (y != y);                   // a NaN y must give NaN: ql carries it
    if constexpr (PREC == FAST) {
        return g * (take_left ? p.ql : p.qr);
    } else {
        const bool direct = take_left || !(fabsf(p.small) < 0.25f);
        float base  = take_left ? p.ql : (direct ? p.qr : 1.0f);
        float delta = direct ? 0.0f : p.small;
        // the small term from a g clamped to the finite range (the same g unless it is infinite): an infinite g
        // times a delta of 0 would turn the infinity of the first term into a NaN; a NaN g stays one through it
        return fmaf(g, base, med3(g, -FLT_MAX, FLT_MAX) * delta);
    }
}

// (a * b) * q  (gated backward: a = grad_h, b = up)
template <int KIND, int PREC>
__device__ __forceinline__ float times_q(float a, float b, float y, bool left)
{
    QParts p = q_parts<KIND, PREC>(y, left);
    const bool take_left = left || (y != y);
    float g = a * b;
    if constexpr (PREC == FAST) {
        return g * (take_left ? p.ql : p.qr);
    } else {
        const bool direct = take_left || !(fabsf(p.small) < 0.25f);
        float base  = take_left ? p.ql : (direct ? p.qr : 1.0f);
        float delta = direct ? 0.0f : p.small;
        float e = fmaf(a, b, -g);                              // a b = g + e exactly,
        e = (fabsf(g) <= FLT_MAX) ? e : 0.0f;                  // unless the product is infinite (or a NaN, which g carries)
        return fmaf(g, base, fmaf(med3(g, -FLT_MAX, FLT_MAX), delta, e * (base + delta)));     // clamped g: see above
    }
}

}  // namespace invact_dev
