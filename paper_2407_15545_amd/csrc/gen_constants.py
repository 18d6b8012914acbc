#!/usr/bin/env python3
"""Writes invact_constants.h: every numeric constant the HIP kernels use.

Run by hand when a constant changes (python gen_constants.py > invact_constants.h);
the header is committed.  Independent of the CPU oracle: nothing here is
imported from or shared with it.

  * T, f(T): minimiser of each activation (Eq. (4): the point that separates
    the two monotone halves), found with 50-digit arithmetic.
  * The coefficients of Eqs. (5)-(8) as printed in the appendix "Approximation
    Coefficients" (the two SiLU tables are printed under each other's labels:
    the five-entry table goes with the exponential form).
  * The cubic exponent c3 (c4 - y~)^3 log2(e) of Eqs. (6) and (8) expanded in
    powers of y~ (all four terms have the same sign, so Horner's rule in
    binary32 loses nothing and needs one rounding fewer near y~ = 0).
  * A polynomial fit of erfcx(z) = exp(z^2) erfc(z) in w = 1 / (1 + p z), used
    by the erf form of GELU with bfloat16 storage:  erfcx(z) ~ w * sum_k a_k w^k on z in [0, 10];
    for binary32 storage a table of degree-4 polynomials of erfcx(x / sqrt 2) / 2 on intervals of width 1/8
    (two coefficients in binary64, three in binary32: 32 bytes a row).
  * A polynomial fit of 2^f on |f| <= 0.501 for the binary32-storage forward
    (the hardware exponential's 0.78 ulp would be the largest error there).
"""
import struct

import mpmath as mp
import numpy as np
import scipy.special as sp
from numpy.polynomial import chebyshev as C, polynomial as P

mp.mp.dps = 50


def f32(v):
    return float(np.float32(v))


def minimiser(kind):
    x = mp.mpf
    if kind == "silu":
        f = lambda t: t / (1 + mp.exp(-t))
    elif kind == "gelu_erf":
        f = lambda t: t * mp.erfc(-t / mp.sqrt(2)) / 2
    else:
        f = lambda t: t / (1 + mp.exp(-2 * mp.sqrt(2 / mp.pi) * (t + x("0.044715") * t ** 3)))
    T = mp.findroot(lambda t: mp.diff(f, t), x("-1.0"))
    return T, f(T)


def erfcx_fit(p, deg, zmax=10.0):
    """Chebyshev interpolant of erfcx(z)/w in w on [1/(1+p zmax), 1], as monomials in w."""
    wmin = 1 / (1 + p * zmax)
    k = np.arange(4 * deg + 8)
    t = np.cos(np.pi * (k + 0.5) / k.size)
    w = 0.5 * (1 + wmin) + 0.5 * (1 - wmin) * t
    z = (1 / w - 1) / p
    cheb = C.chebfit(t, sp.erfcx(z) / w, deg)
    a, b = 2 / (1 - wmin), -(1 + wmin) / (1 - wmin)      # t = a w + b
    mono, pw = np.zeros(1), np.ones(1)
    for ck in C.cheb2poly(cheb):
        mono = P.polyadd(mono, ck * pw)
        pw = P.polymul(pw, np.array([b, a]))
    zz = np.linspace(0, zmax, 400001)
    ww = 1 / (1 + p * zz)
    err = np.abs(P.polyval(ww, mono) * ww / sp.erfcx(zz) - 1).max()
    return mono, err


def mills_table(rows, per_unit):
    """G(x) = Phi(-x) exp(x^2 / 2) = erfcx(x / sqrt 2) / 2 on [0, rows / per_unit) as one degree-4 polynomial per
    interval of width 1 / per_unit: row i holds the monomial coefficients in t = per_unit x - i in [0, 1), c0 and
    c1 in binary64 and c2, c3, c4 in binary32 (their terms are below G / 64, so binary32 is enough for them: the
    kernel evaluates c2 + t (c3 + t c4) in binary32 and the rest in binary64).
    Returns (rows of (c0, c1, c2, c3, c4), max relative error of that mixed evaluation)."""
    deg = 4
    G = lambda x: 0.5 * sp.erfcx(x / np.sqrt(2.0))
    k = np.arange(4 * deg + 8)
    node = np.cos(np.pi * (k + 0.5) / k.size)                  # Chebyshev nodes on [-1, 1]; t = (node + 1) / 2
    table, worst = [], 0.0
    for i in range(rows):
        cheb = C.chebfit(node, G((i + 0.5 * (node + 1)) / per_unit), deg)
        mono, pw = np.zeros(1), np.ones(1)
        for ck in C.cheb2poly(cheb):                           # node = 2 t - 1
            mono = P.polyadd(mono, ck * pw)
            pw = P.polymul(pw, np.array([-1.0, 2.0]))
        row = (float(mono[0]), float(mono[1]), f32(mono[2]), f32(mono[3]), f32(mono[4]))
        tt = np.linspace(0.0, 1.0, 4001)
        t32 = tt.astype(np.float32)
        q = (np.float32(row[4]) * t32 + np.float32(row[3])).astype(np.float32)
        q = (q * t32 + np.float32(row[2])).astype(np.float32)
        g = (q.astype(np.float64) * tt + row[1]) * tt + row[0]
        worst = max(worst, np.abs(g / G((i + tt) / per_unit) - 1).max())
        table.append(row)
    return table, worst


def exp2_fit(deg, half=0.501):
    """Chebyshev interpolant of 2^f on [-half, half] as monomials in f, and its max relative error."""
    k = np.arange(4 * deg + 8)
    t = np.cos(np.pi * (k + 0.5) / k.size)
    vals = np.array([float(mp.power(2, mp.mpf(float(v)) * half)) for v in t])
    mono = C.cheb2poly(C.chebfit(t, vals, deg)) / half ** np.arange(deg + 1)     # t = f / half
    ff = np.linspace(-half, half, 200001)
    exact = np.array([float(mp.power(2, mp.mpf(float(v)))) for v in ff[::100]])
    err = np.abs(P.polyval(ff[::100], mono) / exact - 1).max()
    return mono, err


GELU_LEFT = [1.6311011311381, 0.16997246666667, -0.06261728, 1.2947087,
             1.98055565, 0.22730362, -0.038978495, 1.3295193]
GELU_RIGHT = [-1.383717971214795, 1.558420184350027, 0.044045748018110,
              0.032146736769376, -2.119885089843949]
SILU_LEFT = [0.217177007595768, -0.507684370508263, 0.079631397669175, 0.357494204859375]
SILU_RIGHT = [-1.310856402130980, 0.848589647031652, -0.162990512595109,
              0.002696163985044, -5.770613302664509]


def arr(name, vals, typ="float", suffix="f"):
    # binary32 constants are rounded HERE and printed with 9 significant digits, which
    # round-trip; printing the unrounded value with 9 digits can land on the wrong neighbour
    body = ", ".join(f"{v:.17g}{suffix}" if suffix == "" else f"{f32(v):.9g}{suffix}" for v in vals)
    return f"static constexpr {typ} {name}[{len(vals)}] = {{ {body} }};"


def cubic(c3, c4):
    """t(y~) = c3 (c4 - y~)^3 log2(e) = t0 + y~ (a1 + y~ (a2 + y~ a3)), from the binary32 c3, c4."""
    K = f32(c3) * float(mp.log(mp.e, 2))
    c = f32(c4)
    return [K * c ** 3, -3 * K * c ** 2, 3 * K * c, -K]


def main():
    out = ["// Generated by gen_constants.py -- do not edit by hand.",
           "#pragma once", "", "namespace invact_const {", ""]
    for kind in ("gelu_tanh", "gelu_erf", "silu"):
        T, fT = minimiser(kind)
        out.append(f"// {kind}: T = {mp.nstr(T, 20)}, f(T) = {mp.nstr(fT, 20)}")
        out.append(f"static constexpr float T_{kind} = {f32(T):.9g}f;")
        out.append(f"static constexpr float fT_{kind} = {f32(fT):.9g}f;")
    out.append("")
    out.append("// Eq. (5)"); out.append(arr("gelu_left", GELU_LEFT))
    out.append("// Eq. (6)"); out.append(arr("gelu_right", GELU_RIGHT))
    out.append("// Eq. (7) (table printed under the label q^right)"); out.append(arr("silu_left", SILU_LEFT))
    out.append("// Eq. (8) (table printed under the label q^left)"); out.append(arr("silu_right", SILU_RIGHT))
    out.append("")
    out.append("// log2(e) c3 (c4 - y~)^3 = t[0] + y~ (t[1] + y~ (t[2] + y~ t[3]))")
    out.append(arr("gelu_right_exp2", cubic(GELU_RIGHT[3], GELU_RIGHT[4])))
    out.append(arr("silu_right_exp2", cubic(SILU_RIGHT[3], SILU_RIGHT[4])))
    out.append("")
    # degree 3: 2.6e-4 is 13 % of half a bfloat16 ulp (the stored value stays within 0.57 ulp of f(x)),
    # and every fma less shows in the speed of the bfloat16 forward
    mono, err = erfcx_fit(0.42, 3)
    out.append(f"// erfcx(z) ~ w (a0 + a1 w + ... ), w = 1/(1 + {0.42} z); max rel. error {err:.2e} on [0, 10]")
    out.append("static constexpr float erfcx_fast_p = 0.42f;")
    out.append(arr("erfcx_fast", mono))
    # binary32 storage: erfcx from a table of short polynomials (held in LDS by the kernels): 116 intervals of
    # width 1/8 cover every |x| whose result is not yet +-0 or x itself in binary32; the gated forward, whose
    # product f(gate) * up can still be a binary32 number where f(gate) alone no longer is (|up| up to 3.4e38),
    # uses 160 (beyond x = -20, |x Phi(x)| * 3.4e38 is below half the smallest subnormal)
    rows, near_rows, per_unit = 160, 116, 8
    table, err = mills_table(rows, per_unit)
    out.append(f"// Phi(-x) exp(x^2/2) on [{0}, {rows / per_unit}): row i = coefficients in t = {per_unit} x - i of a degree-4 fit "
               f"on [i/{per_unit}, (i+1)/{per_unit}); max rel. error {err:.2e}.")
    out.append("// 32-bit words: for every row c0 and c1 as binary64 (low word first); then for every row c2, c3, c4 as binary32")
    out.append("// and one word of padding (two arrays of 16-byte entries).")
    out.append(f"static constexpr int mills_rows = {rows}, mills_rows_near = {near_rows}, mills_per_unit = {per_unit};")
    out.append(f"#define INVACT_MILLS_TABLE \\")
    for i, row in enumerate(table):
        words = struct.unpack("<4I", struct.pack("<dd", row[0], row[1]))
        out.append("    " + ", ".join(f"0x{w:08x}u" for w in words) + ", \\")
    for i, row in enumerate(table):
        words = struct.unpack("<4I", struct.pack("<fffI", row[2], row[3], row[4], 0))
        out.append("    " + ", ".join(f"0x{w:08x}u" for w in words) + ("," if i + 1 < rows else "") + " \\")
    out.append("")
    mono, err = exp2_fit(6)
    out.append(f"// 2^f ~ e0 + e1 f + ... on |f| <= 0.501; max rel. error {err:.2e}")
    out.append(arr("exp2_precise", mono, "double", ""))
    out.append("")
    out.append("}  // namespace invact_const")
    print("\n".join(out))


if __name__ == "__main__":
    main()
