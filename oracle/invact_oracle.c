/*
 * CPU oracle for the Inverted-Activations element-wise path (arXiv 2407.15545).
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must
 * compute; it is slow, scalar, IEEE double and shares nothing with the HIP
 * code.  Only the test-suite, the smoke check and the benchmark's CPU-baseline
 * leg may call it.  The product path never does.
 *
 * Parts (each cites the passage of the paper it follows):
 *   O1  exact forward y = f(x)                      Method, Eq. (1), Eq. (3)
 *   O2  branch indicator s = [x < T] and bit pack   Eq. (4) and the paragraph after it
 *   O3  exact f'(x) and the branch-wise inverse     Method, "Inverted Activation"; Fig. 2
 *   O4  the closed-form approximation q(y, s)       Eqs. (5)-(8), Appendix "Approximation Coefficients"
 *   forward / backward of the layer                 Listing "forward-backward" (Algorithm 1)
 *   SwiGLU / GeGLU gated variants                   Experiments, "GeGLU" block; Limitations
 *   precision-bit variant                           Method, "Precision Bit Inverted Activation" and its listing
 *   sign-bit variant, and its consumer (Y + C) W     Method, "Sign-bit Inverted Activation" and its listing
 *
 * Pin status.  O1, O2, O3 are pinned by identities, library routines and brute
 * force (tests/test_oracle_*.py).  O4 is "parity unpinned": the paper prints
 * neither a worked example nor an error bound for q, so q is pinned only
 * indirectly (it must approximate f'(f^-1(y)) region by region, planted
 * mistakes must break that, and it must reproduce independently computed
 * point values kept under tests/golden/).
 *
 * Readings of the paper taken here (the paper is silent or garbled on each):
 *   - The two SiLU coefficient tables of the appendix are printed under the
 *     wrong labels: the 5-coefficient table belongs to the exponential form
 *     (Eq. 8, x >= T) and the 4-coefficient table to the polynomial form
 *     (Eq. 7, x < T).
 *   - The tanh form of GELU uses the GELU formulas and coefficients with its
 *     own T and f(T); the literal c1 of Eq. (5) is kept.
 *   - Every square-root argument is clamped at zero ((v < 0) ? 0 : v, which
 *     lets NaN through).
 *   - All coefficients, T and f(T) used by q and by the indicator are the
 *     binary32 roundings of the printed / computed values, held in double,
 *     so that a binary32 kernel evaluates the very same function.
 *   - x == T gives s = 0; NaN gives s = 0; f(-inf) = -0 with s = 1;
 *     q(+inf, s = 0) = 1.
 *   - Eq. (8), (1 + h)(1 - y) + y, is evaluated in the algebraically equal
 *     form 1 + h (1 - y): as printed it cancels to 0 for y > 2^53 even in
 *     double.
 *   - Sign-bit variant: C is the binary32-rounded f(T); f(x) - C is clamped
 *     at zero, rounded once to the storage dtype, and the sign bit is set on
 *     the stored pattern; the consumer's Y + C is one binary32 addition, and
 *     the backward evaluates q there.
 *   - Sign-bit listing, gradient of the layer's input: printed as the incoming
 *     gradient times f'(f^-1(Y + C, S)); the incoming gradient has the shape of
 *     the linear layer's output, so the factor meant is the gradient at the
 *     activation's output, dOut W: dX = (dOut W) * q(Y + C, S).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { KIND_GELU_TANH = 0, KIND_GELU_ERF = 1, KIND_SILU = 2, KIND_COUNT = 3 };
enum { DTYPE_FP32 = 0, DTYPE_BF16 = 1 };

/* ------------------------------------------------------------------ */
/* O1: exact forward                                                   */
/* ------------------------------------------------------------------ */

/* Logistic function and its complement without cancellation. */
static double sigmoid(double z)  { return 1.0 / (1.0 + exp(-z)); }
static double sigmoidc(double z) { return 1.0 / (1.0 + exp(z)); }   /* 1 - sigmoid(z) */

/* Inner argument of the tanh form: u = sqrt(2/pi) (x + 0.044715 x^3). */
static double tanh_arg(double x)
{
    return sqrt(2.0 / M_PI) * (x + 0.044715 * x * x * x);
}

/* GELU, erf form: x Phi(x) with Phi(x) = erfc(-x / sqrt 2) / 2. */
static double gelu_erf(double x)
{
    if (isinf(x)) return x > 0 ? x : -0.0;
    return 0.5 * x * erfc(-x / sqrt(2.0));
}

/* GELU, tanh form: x (1 + tanh u) / 2 = x sigmoid(2u)  (the right-hand side
 * is the same number without the cancellation of 1 + tanh u for u << 0). */
static double gelu_tanh(double x)
{
    if (isinf(x)) return x > 0 ? x : -0.0;
    return x * sigmoid(2.0 * tanh_arg(x));
}

/* SiLU: x sigmoid(x). */
static double silu(double x)
{
    if (isinf(x)) return x > 0 ? x : -0.0;
    return x * sigmoid(x);
}

double oracle_f_scalar(int kind, double x)
{
    switch (kind) {
    case KIND_GELU_TANH: return gelu_tanh(x);
    case KIND_GELU_ERF:  return gelu_erf(x);
    case KIND_SILU:      return silu(x);
    }
    return NAN;
}

/* ------------------------------------------------------------------ */
/* O3: exact derivative                                                */
/* ------------------------------------------------------------------ */

double oracle_df_scalar(int kind, double x)
{
    if (isnan(x)) return x;
    if (isinf(x)) return x > 0 ? 1.0 : 0.0;
    switch (kind) {
    case KIND_GELU_ERF: {
        /* Phi(x) + x phi(x) */
        double Phi = 0.5 * erfc(-x / sqrt(2.0));
        double phi = exp(-0.5 * x * x) / sqrt(2.0 * M_PI);
        return Phi + x * phi;
    }
    case KIND_GELU_TANH: {
        /* d/dx [x g(x)], g = sigmoid(2u):  g + x * 2 g (1 - g) u'(x) */
        double u  = tanh_arg(x);
        double du = sqrt(2.0 / M_PI) * (1.0 + 3.0 * 0.044715 * x * x);
        double g  = sigmoid(2.0 * u);
        double gc = sigmoidc(2.0 * u);
        if (g == 0.0 || gc == 0.0) return g;      /* saturated: f' is 0 or 1 */
        return g + x * (2.0 * g * gc * du);
    }
    case KIND_SILU: {
        /* sigma (1 + x (1 - sigma)) */
        double g  = sigmoid(x);
        double gc = sigmoidc(x);
        return g == 0.0 ? 0.0 : g * (1.0 + x * gc);
    }
    }
    return NAN;
}

/* ------------------------------------------------------------------ */
/* T = argmin f, f(T), and their binary32 roundings                    */
/* ------------------------------------------------------------------ */

static double T_exact[KIND_COUNT], fT_exact[KIND_COUNT];
static double T_f32[KIND_COUNT],   fT_f32[KIND_COUNT];
static int    consts_ready = 0;

static double as_f32(double v) { return (double)(float)v; }

/* T is the only zero of f' on [-2, -0.5] (f' < 0 left of it, > 0 right). */
static void init_consts(void)
{
    if (consts_ready) return;
    for (int k = 0; k < KIND_COUNT; ++k) {
        double lo = -2.0, hi = -0.5;
        for (int it = 0; it < 200; ++it) {
            double mid = 0.5 * (lo + hi);
            if (mid == lo || mid == hi) break;
            if (oracle_df_scalar(k, mid) < 0.0) lo = mid; else hi = mid;
        }
        /* lo and hi are now neighbours; keep the one with the smaller |f'| */
        double t = fabs(oracle_df_scalar(k, lo)) <= fabs(oracle_df_scalar(k, hi)) ? lo : hi;
        T_exact[k]  = t;
        fT_exact[k] = oracle_f_scalar(k, t);
        T_f32[k]    = as_f32(t);
        fT_f32[k]   = as_f32(fT_exact[k]);
    }
    consts_ready = 1;
}

double oracle_T(int kind)       { init_consts(); return T_exact[kind]; }
double oracle_fT(int kind)      { init_consts(); return fT_exact[kind]; }
double oracle_T_f32(int kind)   { init_consts(); return T_f32[kind]; }
double oracle_fT_f32(int kind)  { init_consts(); return fT_f32[kind]; }

/* ------------------------------------------------------------------ */
/* O3: exact branch-wise inverse                                       */
/* ------------------------------------------------------------------ */

/* x with f(x) = y on (-inf, T] if s else on [T, inf), by bisection until the
 * bracket is two neighbouring doubles (no Newton step: it could not improve
 * on that).  NaN for a y the branch does not reach. */
double oracle_finv_scalar(int kind, double y, int s)
{
    init_consts();
    double T = T_exact[kind], fT = fT_exact[kind];
    if (isnan(y)) return y;
    if (y < fT) return NAN;
    if (y == fT) return T;
    double lo, hi;                       /* f(lo) on one side of y, f(hi) on the other */
    if (s) {
        if (y > 0.0) return NAN;
        if (y == 0.0) return -INFINITY;
        lo = -1.0e4; hi = T;             /* f decreasing: f(lo) = -0 > y > f(hi) = fT */
        for (int it = 0; it < 400; ++it) {
            double mid = 0.5 * (lo + hi);
            if (mid == lo || mid == hi) break;
            if (oracle_f_scalar(kind, mid) > y) lo = mid; else hi = mid;
        }
    } else {
        if (isinf(y)) return y;
        if (y == 0.0) return 0.0;                 /* f(0) = 0 on the right branch */
        lo = T; hi = (y > 0.0 ? y : 0.0) + 1.0;   /* f(x) <= x for x >= 0, f(x) >= x - 1 */
        for (int it = 0; it < 400; ++it) {
            double mid = 0.5 * (lo + hi);
            if (mid == lo || mid == hi) break;
            if (oracle_f_scalar(kind, mid) < y) lo = mid; else hi = mid;
        }
    }
    /* of the two neighbours keep the one whose image is nearer to y */
    return fabs(oracle_f_scalar(kind, lo) - y) <= fabs(oracle_f_scalar(kind, hi) - y) ? lo : hi;
}

/* ------------------------------------------------------------------ */
/* O4: the paper's approximation of f'(f^-1(y))                        */
/* ------------------------------------------------------------------ */

/* Appendix "Approximation Coefficients", as printed. */
static const double GELU_LEFT[8] = {
    +1.6311011311381, +0.16997246666667, -0.06261728, +1.2947087,
    +1.98055565, +0.22730362, -0.038978495, +1.3295193 };
static const double GELU_RIGHT[5] = {
    -1.383717971214795, +1.558420184350027, +0.044045748018110,
    +0.032146736769376, -2.119885089843949 };
/* printed under the label q^right; used by the polynomial form, Eq. (7) */
static const double SILU_LEFT[4] = {
    +0.217177007595768, -0.507684370508263, +0.079631397669175, +0.357494204859375 };
/* printed under the label q^left; used by the exponential form, Eq. (8) */
static const double SILU_RIGHT[5] = {
    -1.310856402130980, +0.848589647031652, -0.162990512595109,
    +0.002696163985044, -5.770613302664509 };

static double clamp0(double v) { return (v < 0.0) ? 0.0 : v; }

/* Coefficients can be overridden (tests plant mistakes this way). */
typedef struct {
    double gelu_left[8], gelu_right[5], silu_left[4], silu_right[5];
} coeff_set;

static void default_coeffs(coeff_set *c)
{
    for (int i = 0; i < 8; ++i) c->gelu_left[i]  = as_f32(GELU_LEFT[i]);
    for (int i = 0; i < 5; ++i) c->gelu_right[i] = as_f32(GELU_RIGHT[i]);
    for (int i = 0; i < 4; ++i) c->silu_left[i]  = as_f32(SILU_LEFT[i]);
    for (int i = 0; i < 5; ++i) c->silu_right[i] = as_f32(SILU_RIGHT[i]);
}

void oracle_default_coeffs(double *out22)
{
    coeff_set c; default_coeffs(&c);
    memcpy(out22, &c, sizeof c);
}

/* Eq. (6) / inner part of Eq. (8): h = (c0 + c1 sqrt(yt) + c2 yt) exp(c3 (c4 - yt)^3) */
static double exp_form(const double *c, double yt)
{
    double d = c[4] - yt;
    return (c[0] + c[1] * sqrt(yt) + c[2] * yt) * exp(c[3] * d * d * d);
}

static double q_with_fT(const coeff_set *cs, int kind, double fT, double y, int s)
{
    if (kind == KIND_SILU) {
        double yt = clamp0(y - fT);
        if (s) {                                                   /* Eq. (7) */
            const double *c = cs->silu_left;
            double a = c[0] + c[1] * sqrt(yt) + c[2] * yt + c[3] * yt * yt;
            return a * (1.0 - y) + y;
        }
        if (isinf(y) && y > 0) return 1.0;
        return 1.0 + exp_form(cs->silu_right, yt) * (1.0 - y);     /* Eq. (8) */
    }
    if (s) {                                                       /* Eq. (5) */
        const double *c = cs->gelu_left;
        double inner = fabs(c[4] * y + c[5]);
        double outer = fabs(c[3] * y * y + inner + c[6]) + c[7];
        return c[0] * sqrt(clamp0(y + c[1])) * (2.0 * y + c[2] * sqrt(clamp0(-y))) * outer;
    }
    if (isinf(y) && y > 0) return 1.0;
    return 1.0 + exp_form(cs->gelu_right, clamp0(y - fT));         /* Eq. (6) */
}

static double q_with(const coeff_set *cs, int kind, double y, int s)
{
    return q_with_fT(cs, kind, fT_f32[kind], y, s);
}

double oracle_q_scalar(int kind, double y, int s)
{
    init_consts();
    coeff_set c; default_coeffs(&c);
    return q_with(&c, kind, y, s);
}

/* ------------------------------------------------------------------ */
/* Rounding to the storage grid                                        */
/* ------------------------------------------------------------------ */

/* Nearest value (ties to even) with p significand bits and binary32's
 * exponent range: p = 24 is binary32, p = 8 is bfloat16. */
static double round_grid(double v, int p)
{
    if (isnan(v) || isinf(v) || v == 0.0) return v;
    int e;
    frexp(v, &e);                         /* |v| = m 2^e, m in [0.5, 1) */
    int qexp = e - p;                     /* exponent of the quantum */
    if (qexp < -126 - (p - 1)) qexp = -126 - (p - 1);   /* subnormal spacing */
    double r = ldexp(nearbyint(ldexp(v, -qexp)), qexp);
    if (fabs(r) >= ldexp(1.0, 128)) r = copysign(INFINITY, v);
    return r;
}

double oracle_round_scalar(int dtype, double v)
{
    return round_grid(v, dtype == DTYPE_BF16 ? 8 : 24);
}

/* ------------------------------------------------------------------ */
/* Array entry points                                                  */
/* ------------------------------------------------------------------ */

void oracle_f(int kind, const double *x, double *y, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) y[i] = oracle_f_scalar(kind, x[i]);
}

void oracle_df(int kind, const double *x, double *d, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) d[i] = oracle_df_scalar(kind, x[i]);
}

void oracle_finv(int kind, const double *y, const uint8_t *s, double *x, size_t n)
{
    init_consts();
#pragma omp parallel for schedule(dynamic, 1024)
    for (size_t i = 0; i < n; ++i) x[i] = oracle_finv_scalar(kind, y[i], s[i]);
}

void oracle_q(int kind, const double *y, const uint8_t *s, double *q, size_t n)
{
    init_consts();
    coeff_set c; default_coeffs(&c);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) q[i] = q_with(&c, kind, y[i], s[i]);
}

/* Same as oracle_q with caller-supplied constants: 22 coefficients in the
 * order gelu_left[8], gelu_right[5], silu_left[4], silu_right[5], and the
 * value used for f(T).  Tests use it to plant mistakes and to evaluate q
 * with the unrounded constants. */
void oracle_q_coeffs(int kind, const double *coeffs22, double fT, const double *y,
                     const uint8_t *s, double *q, size_t n)
{
    init_consts();
    coeff_set c; memcpy(&c, coeffs22, sizeof c);
    for (size_t i = 0; i < n; ++i) q[i] = q_with_fT(&c, kind, fT, y[i], s[i]);
}

/* The appendix's coefficients exactly as printed (not rounded to binary32). */
void oracle_printed_coeffs(double *out22)
{
    memcpy(out22,      GELU_LEFT,  sizeof GELU_LEFT);
    memcpy(out22 + 8,  GELU_RIGHT, sizeof GELU_RIGHT);
    memcpy(out22 + 13, SILU_LEFT,  sizeof SILU_LEFT);
    memcpy(out22 + 17, SILU_RIGHT, sizeof SILU_RIGHT);
}

void oracle_round(int dtype, const double *v, double *out, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) out[i] = oracle_round_scalar(dtype, v[i]);
}

/* O2.  s[i] = [x[i] < T]; bit (i mod 8) of byte (i div 8), which is bit
 * (i mod 64) of little-endian 64-bit word (i div 64).  `mask` holds
 * 8 ceil(n/64) bytes; bits past n are 0. */
void oracle_indicator(int kind, const double *x, uint8_t *s, size_t n)
{
    init_consts();
    double T = T_f32[kind];
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) s[i] = (x[i] < T) ? 1 : 0;
}

size_t oracle_mask_bytes(size_t n) { return 8 * ((n + 63) / 64); }

void oracle_pack(const uint8_t *s, uint8_t *mask, size_t n)
{
    size_t nbytes = oracle_mask_bytes(n);
#pragma omp parallel for schedule(static)
    for (size_t b = 0; b < nbytes; ++b) {
        uint8_t byte = 0;
        for (size_t j = 0; j < 8; ++j) {
            size_t i = 8 * b + j;
            if (i < n && s[i]) byte |= (uint8_t)(1u << j);
        }
        mask[b] = byte;
    }
}

/* pack [v[i] < T] without an intermediate array */
static void pack_less_than(const double *v, double T, uint8_t *mask, size_t n)
{
    size_t nbytes = oracle_mask_bytes(n);
#pragma omp parallel for schedule(static)
    for (size_t b = 0; b < nbytes; ++b) {
        uint8_t byte = 0;
        for (size_t j = 0; j < 8; ++j) {
            size_t i = 8 * b + j;
            if (i < n && v[i] < T) byte |= (uint8_t)(1u << j);
        }
        mask[b] = byte;
    }
}

void oracle_unpack(const uint8_t *mask, uint8_t *s, size_t n)
{
    for (size_t i = 0; i < n; ++i) s[i] = (mask[i / 8] >> (i % 8)) & 1;
}

/* Algorithm 1, forward: S = X < T, Y = f(X).  y_exact is f(x) in double,
 * y_stored its rounding to the storage dtype (what the layer saves and
 * returns). */
void oracle_invact_fwd(int kind, int dtype, const double *x, double *y_exact,
                       double *y_stored, uint8_t *mask, size_t n)
{
    init_consts();
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        y_exact[i]  = oracle_f_scalar(kind, x[i]);
        y_stored[i] = oracle_round_scalar(dtype, y_exact[i]);
    }
    pack_less_than(x, T_f32[kind], mask, n);
}

/* Algorithm 1, backward: dX = dY * q(Y, S) (unrounded double). */
void oracle_invact_bwd(int kind, const double *y, const uint8_t *mask,
                       const double *grad_y, double *grad_x, size_t n)
{
    init_consts();
    coeff_set c; default_coeffs(&c);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        int s = (mask[i / 8] >> (i % 8)) & 1;
        grad_x[i] = grad_y[i] * q_with(&c, kind, y[i], s);
    }
}

/* Gated block, forward: a = f(gate), s = [gate < T], h = a * up.
 * The block saves a (rounded), up and the mask. */
void oracle_glu_fwd(int kind, int dtype, const double *gate, const double *up,
                    double *a_exact, double *a_stored, double *h_exact,
                    uint8_t *mask, size_t n)
{
    init_consts();
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        a_exact[i]  = oracle_f_scalar(kind, gate[i]);
        a_stored[i] = oracle_round_scalar(dtype, a_exact[i]);
        h_exact[i]  = a_exact[i] * up[i];
    }
    pack_less_than(gate, T_f32[kind], mask, n);
}

/* Gated block, backward from the saved a, up, mask:
 * grad_up = grad_h * a ; grad_gate = grad_h * up * q(a, s). */
void oracle_glu_bwd(int kind, const double *a, const double *up, const uint8_t *mask,
                    const double *grad_h, double *grad_gate, double *grad_up, size_t n)
{
    init_consts();
    coeff_set c; default_coeffs(&c);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        int s = (mask[i / 8] >> (i % 8)) & 1;
        grad_up[i]   = grad_h[i] * a[i];
        grad_gate[i] = grad_h[i] * up[i] * q_with(&c, kind, a[i], s);
    }
}

/* ------------------------------------------------------------------ */
/* Precision-bit variant                                               */
/* ------------------------------------------------------------------ */

/* Position of the lowest significand bit of the storage format inside the
 * binary32 pattern of a stored value (a bfloat16 is the upper half of one). */
static uint32_t lsb_mask(int dtype) { return dtype == DTYPE_BF16 ? 0x00010000u : 0x00000001u; }

/* Y = (Y & ~1) | S on the storage format's bit pattern. */
double oracle_tag_lsb(int dtype, double stored, int s)
{
    float f = (float)stored;              /* exact: stored lies on the grid */
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    bits = (bits & ~lsb_mask(dtype)) | (s ? lsb_mask(dtype) : 0u);
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* S = Y & 1 */
int oracle_read_lsb(int dtype, double stored)
{
    float f = (float)stored;
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    return (bits & lsb_mask(dtype)) != 0;
}

/* Forward: S = X < T; Y = f(X) rounded to the storage dtype; lowest bit of Y := S.
 * The tagged Y is both what the layer returns and what it saves. */
void oracle_pbit_fwd(int kind, int dtype, const double *x, double *y_exact, double *y_stored, size_t n)
{
    init_consts();
    double T = T_f32[kind];
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        y_exact[i]  = oracle_f_scalar(kind, x[i]);
        y_stored[i] = oracle_tag_lsb(dtype, oracle_round_scalar(dtype, y_exact[i]), x[i] < T);
    }
}

/* Backward: S = Y & 1; dX = dY * q(Y, S), with Y the saved (tagged) value. */
void oracle_pbit_bwd(int kind, int dtype, const double *y, const double *grad_y, double *grad_x, size_t n)
{
    init_consts();
    coeff_set c; default_coeffs(&c);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i)
        grad_x[i] = grad_y[i] * q_with(&c, kind, y[i], oracle_read_lsb(dtype, y[i]));
}

/* ------------------------------------------------------------------ */
/* Sign-bit variant (Section 3.3, "Sign-bit Inverted Activation", and  */
/* its listing)                                                        */
/* ------------------------------------------------------------------ */

/* Forward: S = X < T; Y = f(X) - C with C = min f = f(T) (here the binary32-
 * rounded f(T), like every constant), so Y >= 0 up to that rounding (clamp0
 * takes care of the rest); Y is rounded to the storage dtype and its sign bit
 * is set to S.  The tagged Y is what the layer saves; what it hands to the
 * next layer is Y + C (oracle_sbit_decode). */
void oracle_sbit_fwd(int kind, int dtype, const double *x, double *v_exact, double *y_tagged, size_t n)
{
    init_consts();
    double T = T_f32[kind], C = fT_f32[kind];
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        v_exact[i] = clamp0(oracle_f_scalar(kind, x[i]) - C);
        double mag = oracle_round_scalar(dtype, v_exact[i]);
        y_tagged[i] = (x[i] < T) ? -fabs(mag) : fabs(mag);          /* sign bit := S (a NaN keeps S = 0) */
    }
}

/* What the consumer of the saved tensor computes first: S = sign bit, Y = |Y| + C. */
void oracle_sbit_decode(int kind, int dtype, const double *y_tagged, double *y_exact, double *y_stored, size_t n)
{
    init_consts();
    double C = fT_f32[kind];
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        y_exact[i]  = fabs(y_tagged[i]) + C;                         /* exact in double */
        y_stored[i] = oracle_round_scalar(dtype, y_exact[i]);
    }
}

/* Backward: S = sign bit of the saved Y; Y + C formed in binary32 (one rounding:
 * the working precision of the kernels' registers); dX = dY * q(Y + C, S). */
void oracle_sbit_bwd(int kind, const double *y_tagged, const double *grad_y, double *grad_x, size_t n)
{
    init_consts();
    coeff_set c; default_coeffs(&c);
    double C = fT_f32[kind];
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        int s = signbit(y_tagged[i]) != 0 && !isnan(y_tagged[i]);
        double y = oracle_round_scalar(DTYPE_FP32, fabs(y_tagged[i]) + C);
        grad_x[i] = grad_y[i] * q_with(&c, kind, y, s);
    }
}

/* The consumer in the paper's listing, forward: out = (Y + C) W^T (+ bias).  Y + C is what
 * oracle_sbit_decode stores: the sum rounded to the storage dtype, which is what a matrix unit fed
 * with that dtype multiplies.  y_tagged is [M][K], w is [N][K] (the layout of a linear layer's weight),
 * bias is [N] or NULL, out is [M][N]; plain sums in double. */
void oracle_sbit_linear(int kind, int dtype, const double *y_tagged, const double *w, const double *bias,
                        double *out, size_t M, size_t N, size_t K)
{
    init_consts();
    double C = fT_f32[kind];
#pragma omp parallel for schedule(static)
    for (size_t m = 0; m < M; ++m)
        for (size_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (size_t k = 0; k < K; ++k)
                acc += oracle_round_scalar(dtype, fabs(y_tagged[m * K + k]) + C) * w[n * K + k];
            out[m * N + n] = bias ? acc + bias[n] : acc;
        }
}

/* The same listing, backward: dW = dOut^T (Y + C), with Y + C as above.  grad_out is [M][N],
 * grad_w is [N][K]. */
void oracle_sbit_linear_wgrad(int kind, int dtype, const double *y_tagged, const double *grad_out,
                              double *grad_w, size_t M, size_t N, size_t K)
{
    init_consts();
    double C = fT_f32[kind];
#pragma omp parallel for schedule(static)
    for (size_t n = 0; n < N; ++n)
        for (size_t k = 0; k < K; ++k) {
            double acc = 0.0;
            for (size_t m = 0; m < M; ++m)
                acc += grad_out[m * N + n] * oracle_round_scalar(dtype, fabs(y_tagged[m * K + k]) + C);
            grad_w[n * K + k] = acc;
        }
}

/* The same listing, backward, the gradient of the layer's input: the gradient that reaches the
 * activation's output is dOut W (the adjoint of the forward product; the listing prints the factor
 * as the incoming gradient alone), and the activation's own backward multiplies it by
 * f'(f^-1(Y + C, S)), i.e. by q as oracle_sbit_bwd evaluates it: dX = (dOut W) * q(Y + C, S).
 * grad_out is [M][N], w is [N][K], grad_x is [M][K]; plain sums in double, nothing rounded. */
void oracle_sbit_linear_dgrad(int kind, const double *y_tagged, const double *grad_out, const double *w,
                              double *grad_x, size_t M, size_t N, size_t K)
{
    init_consts();
    coeff_set c; default_coeffs(&c);
    double C = fT_f32[kind];
#pragma omp parallel for schedule(static)
    for (size_t m = 0; m < M; ++m)
        for (size_t k = 0; k < K; ++k) {
            double acc = 0.0;
            for (size_t n = 0; n < N; ++n)
                acc += grad_out[m * N + n] * w[n * K + k];
            double yt = y_tagged[m * K + k];
            int s = signbit(yt) != 0 && !isnan(yt);
            double y = oracle_round_scalar(DTYPE_FP32, fabs(yt) + C);
            grad_x[m * K + k] = acc * q_with(&c, kind, y, s);
        }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
