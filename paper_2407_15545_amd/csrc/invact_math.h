// Device-side arithmetic of the Inverted-Activations kernels (gfx950).
//
// Everything here works on binary32 values in registers.  Two precision
// policies exist for the forward activation:
//   FAST    -- hardware exp2 / rcp / sqrt (1 ulp each) and short polynomials;
//              far more accurate than a bfloat16 store can show.  Used when
//              the storage dtype is bfloat16.
//   PRECISE -- arguments and the final combination in binary64, the
//              transcendental itself still the binary32 hardware unit fed
//              with a hi + lo split argument; about 1.6 ulp worst case.  Used
//              when the storage dtype is binary32.
// The backward approximation q (Eqs. (5)-(8)) is evaluated the same way for
// both dtypes: its absolute error is what matters there.
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
__device__ __forceinline__ float clamp_finite(float v)                                    // NaN -> -FLT_MAX
{
    return __builtin_amdgcn_fmed3f(v, -FLT_MAX, FLT_MAX);
}

constexpr float kLog2e      = 1.44269504088896340736f;
constexpr double kLog2eD    = 1.44269504088896340736;
constexpr double kLn2D      = 0.69314718055994530942;
constexpr double kSqrt2OverPi = 0.79788456080286535588;   // sqrt(2/pi)
constexpr double kGeluCubic = 0.044715;
constexpr double kInvSqrt2  = 0.70710678118654752440;

// The branch threshold T (minimiser of f) and f(T), rounded to binary32.
template <int KIND> struct KindConst;
template <> struct KindConst<GELU_TANH> { static constexpr float T = cst::T_gelu_tanh, fT = cst::fT_gelu_tanh; };
template <> struct KindConst<GELU_ERF>  { static constexpr float T = cst::T_gelu_erf,  fT = cst::fT_gelu_erf; };
template <> struct KindConst<SILU>      { static constexpr float T = cst::T_silu,      fT = cst::fT_silu; };

// ---------------------------------------------------------------------------
// Forward, FAST
// ---------------------------------------------------------------------------

// x * sigmoid(z) given th = -|z| log2(e) / 2 (sign(z) = sign(x)).
// With Eh = exp(-|z|/2):  sigmoid(|z|) = 1 / (1 + Eh^2),  sigmoid(-|z|) = Eh^2 / (1 + Eh^2).
// The product is taken as (x Eh) * (Eh r) so that no factor is subnormal
// while the result is still a normal number (x ~ -90 for SiLU).
__device__ __forceinline__ float x_sigmoid_fast(float x, float th)
{
    float Eh = hw_exp2(th);
    float r  = hw_rcp(fmaf(Eh, Eh, 1.0f));
    float m  = (x < 0.0f) ? Eh : 1.0f;
    float a  = clamp_finite(x) * m;          // -inf * 0 must not make a NaN; NaN x comes back through r
    return a * (r * m);
}

template <int KIND>
__device__ __forceinline__ float act_fast(float x)
{
    if constexpr (KIND == SILU) {
        return x_sigmoid_fast(x, -fabsf(x) * (0.5f * kLog2e));
    } else if constexpr (KIND == GELU_TANH) {
        // z = 2u, u = sqrt(2/pi) (x + 0.044715 x^3):  |z| log2(e) / 2 = |x (k1 + k2 x^2)|
        constexpr float k1 = (float)(kSqrt2OverPi * kLog2eD);
        constexpr float k2 = (float)(kSqrt2OverPi * kLog2eD * kGeluCubic);
        float inner = x * fmaf(k2, x * x, k1);
        return x_sigmoid_fast(x, -fabsf(inner));
    } else {
        // x Phi(x), Phi(-|x|) = erfc(z)/2 = erfcx(z) exp(-z^2) / 2 with z = |x| / sqrt 2
        constexpr float pz = (float)(cst::erfcx_fast_p * kInvSqrt2);
        float ax = fabsf(x);
        float w  = hw_rcp(fmaf(pz, ax, 1.0f));
        float g  = 0.5f * cst::erfcx_fast[5];
#pragma unroll
        for (int k = 4; k >= 0; --k) g = fmaf(g, w, 0.5f * cst::erfcx_fast[k]);
        g *= w;                                                   // erfcx(z) / 2
        float E = hw_exp2((x * x) * (-0.5f * kLog2e));            // exp(-z^2)
        float u = (clamp_finite(x) * g) * E;                      // x Phi(-|x|) sign-carrying
        return (x < 0.0f) ? u : x - u;                            // x (1 - Phi(-|x|)) for x >= 0
    }
}

// ---------------------------------------------------------------------------
// Forward, PRECISE
// ---------------------------------------------------------------------------

// exp2 of a binary64 argument t <= 0 through the binary32 unit:
// 2^t = 2^hi * 2^lo,  hi = fl32(t),  2^lo = 1 + lo ln2 (|lo| < 2^-24 |t|).
// Returns a binary64 value with the relative error of v_exp_f32 (1 ulp of
// binary32) and no error from the argument.  `bias` is added to the
// exponent so that the caller can keep the result normal.
__device__ __forceinline__ double exp2_split(double t, float bias)
{
    float hi = (float)t;
    float lo = (float)(t - (double)hi);
    float e  = hw_exp2(hi + bias);
    return (double)e * (1.0 + kLn2D * (double)lo);
}

// 1 / d for d in [1, 2], to ~2^-45: binary32 seed and one Newton step in binary64.
__device__ __forceinline__ double rcp_newton(double d)
{
    double r = (double)hw_rcp((float)d);
    return r * (2.0 - d * r);
}

// x * sigmoid(z) with t = -|z| log2(e) given in binary64; result in binary64
// (relative error about 2^-23.3 from the hardware exp2, nothing else).
__device__ __forceinline__ double x_sigmoid_precise(float x, double t)
{
    // E = exp(-|z|) scaled by 2^64 when it would be subnormal in binary32
    t = (t < -300.0) ? -300.0 : t;                 // keeps fl32(t) finite; NaN stays NaN
    const bool tiny = t < -120.0;
    double E = exp2_split(t, tiny ? 64.0f : 0.0f);
    double Eu = tiny ? 0.0 : E;                    // unscaled value, only needed in 1 + E
    double r = rcp_newton(1.0 + Eu);
    double xd = (double)clamp_finite(x);
    double y = (x < 0.0f) ? xd * E * r * (tiny ? 0x1p-64 : 1.0) : xd * r;
    return (x == INFINITY) ? (double)x : y;
}

template <int KIND>
__device__ __forceinline__ double act_precise(float x)
{
    if constexpr (KIND == SILU) {
        return x_sigmoid_precise(x, -fabs((double)x) * kLog2eD);
    } else if constexpr (KIND == GELU_TANH) {
        double xd = (double)x;
        double z2 = xd * (2.0 * kSqrt2OverPi * kLog2eD + (2.0 * kSqrt2OverPi * kLog2eD * kGeluCubic) * (xd * xd));
        return x_sigmoid_precise(x, -fabs(z2));
    } else {
        if (fabsf(x) == INFINITY) return (x > 0.0f) ? (double)x : -0.0;
        double ax = fabs((double)x);
        double z  = ax * kInvSqrt2;
        // w = 1 / (1 + p z) in (0, 1]; seed + Newton as above (the denominator is not in [1,2]
        // but the binary32 seed is good to 2^-22 for any normal argument)
        double d = 1.0 + cst::erfcx_precise_p * z;
        double w = (double)hw_rcp((float)d);
        w = w * (2.0 - d * w);
        double g = cst::erfcx_precise[10];
#pragma unroll
        for (int k = 9; k >= 0; --k) g = g * w + cst::erfcx_precise[k];
        g *= w;                                                    // erfcx(z)
        double t = -(z * z) * kLog2eD;                             // log2 of exp(-z^2)
        const bool tiny = t < -100.0;
        double E = exp2_split(t < -300.0 ? -300.0 : t, tiny ? 64.0f : 0.0f);
        double xd = (double)clamp_finite(x);
        double u = xd * (0.5 * g) * E;                             // x erfc(z) / 2 (scaled if tiny)
        if (tiny) u *= 0x1p-64;
        return (x < 0.0f) ? u : (double)x - u;
    }
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
        double ad = act_precise<KIND>(gate);
        a = (float)ad;
        h = (float)(ad * (double)up);
    }
}

// ---------------------------------------------------------------------------
// Backward: q(y, s) ~ f'(f^-1(y)), Eqs. (5)-(8)
// ---------------------------------------------------------------------------

__device__ __forceinline__ float clamp0(float v) { return (v < 0.0f) ? 0.0f : v; }   // NaN stays NaN

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
//          error of a few ulp of ITSELF: the better representation once |small| is
//          well below 1 (q near or above 1)
struct QParts { float ql, qr, small; };

template <int KIND>
__device__ __forceinline__ QParts q_parts(float y)
{
    constexpr float fT = KindConst<KIND>::fT;
    QParts out;
    if constexpr (KIND == SILU) {
        const auto& L = cst::silu_left;
        const auto& R = cst::silu_right;
        float yc = (y > 64.0f) ? 64.0f : y;          // E == 0 beyond yt = 64; keeps NaN, tames +inf
        float yt = clamp0(yc - fT);
        float sq = hw_sqrt(yt);
        // Eq. (8) as 1 + h (1 - y), h = (c0 + r) E
        float E = cubic_exp2(cst::silu_right_exp2, yt);
        float r = fmaf(R[2], yt, R[1] * sq);
        float h = fmaf(r, E, R[0] * E);
        out.qr    = fmaf(-yc, h, fmaf(r, E, fmaf(R[0], E, 1.0f)));
        out.small = h * (1.0f - yc);
        // Eq. (7): (c0 + c1 sqrt(yt) + c2 yt + c3 yt^2) (1 - y) + y
        float A = fmaf(yt, fmaf(L[3], yt, L[2]), fmaf(L[1], sq, L[0]));
        out.ql = fmaf(A, 1.0f - yc, yc);
    } else {
        const auto& L = cst::gelu_left;
        const auto& R = cst::gelu_right;
        // Eq. (6): 1 + (c0 + c1 sqrt(yt) + c2 yt) E.  E is exactly 0 beyond yt = 64,
        // so y is clamped there (keeps +inf from producing inf * 0).
        float yc = (y > 64.0f) ? 64.0f : y;
        float yt = clamp0(yc - fT);
        float E  = cubic_exp2(cst::gelu_right_exp2, yt);
        float r  = fmaf(R[2], yt, R[1] * hw_sqrt(yt));
        out.qr    = fmaf(r, E, fmaf(R[0], E, 1.0f));
        out.small = fmaf(r, E, R[0] * E);
        // Eq. (5): c0 sqrt(y + c1) (2y + c2 sqrt(-y)) (|c3 y^2 + |c4 y + c5| + c6| + c7).
        // NaN reaches the result through the 2y term, so fmax may drop it here.
        float s1 = hw_sqrt(fmaxf(y + L[1], 0.0f));
        float s2 = hw_sqrt(fmaxf(-y, 0.0f));
        float B  = fmaf(L[2], s2, y + y);
        float inner = fabsf(fmaf(L[4], y, L[5]));
        float outer = fabsf(fmaf(L[3], y * y, inner) + L[6]) + L[7];
        out.ql = (L[0] * s1) * B * outer;
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
    QParts p = q_parts<KIND>(y);
    if constexpr (PREC == FAST) {
        return g * (left ? p.ql : p.qr);
    } else {
        const bool direct = left || !(fabsf(p.small) < 0.25f);
        float base  = left ? p.ql : (direct ? p.qr : 1.0f);
        float delta = direct ? 0.0f : p.small;
        return fmaf(g, base, g * delta);
    }
}

// (a * b) * q  (gated backward: a = grad_h, b = up)
template <int KIND, int PREC>
__device__ __forceinline__ float times_q(float a, float b, float y, bool left)
{
    QParts p = q_parts<KIND>(y);
    float g = a * b;
    if constexpr (PREC == FAST) {
        return g * (left ? p.ql : p.qr);
    } else {
        const bool direct = left || !(fabsf(p.small) < 0.25f);
        float base  = left ? p.ql : (direct ? p.qr : 1.0f);
        float delta = direct ? 0.0f : p.small;
        float e = fmaf(a, b, -g);                              // a b = g + e exactly
        return fmaf(g, base, fmaf(g, delta, e * (base + delta)));
    }
}

}  // namespace invact_dev
