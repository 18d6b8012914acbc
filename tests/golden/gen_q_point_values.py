#!/usr/bin/env python3
"""Regenerates q_point_values.txt: point values of the approximation q(y, s) of Eqs. (5)-(8), computed with
40-digit arithmetic (mpmath) straight from the printed formulas and the coefficients of the appendix
"Approximation Coefficients" exactly as printed (not rounded to binary32), at y = f(x) with f and the
minimiser T exact.  Imports nothing from the oracle or from the GPU library.

    python tests/golden/gen_q_point_values.py > tests/golden/q_point_values.txt

Reading taken for SiLU: the appendix prints a five-number table under the label "left" and a four-number one
under "right", but Eq. (7) (left) has four coefficients and Eq. (8) (right) five, so the five-number table goes
with Eq. (8) and the four-number table with Eq. (7).
"""
import mpmath as mp

mp.mp.dps = 40
M = mp.mpf

GELU_LEFT = [M(v) for v in ("1.6311011311381", "0.16997246666667", "-0.06261728", "1.2947087",
                            "1.98055565", "0.22730362", "-0.038978495", "1.3295193")]
GELU_RIGHT = [M(v) for v in ("-1.383717971214795", "1.558420184350027", "0.044045748018110",
                             "0.032146736769376", "-2.119885089843949")]
SILU_FIVE = [M(v) for v in ("-1.310856402130980", "0.848589647031652", "-0.162990512595109",
                            "0.002696163985044", "-5.770613302664509")]
SILU_FOUR = [M(v) for v in ("0.217177007595768", "-0.507684370508263", "0.079631397669175", "0.357494204859375")]

F = {"gelu_erf": lambda x: x * mp.erfc(-x / mp.sqrt(2)) / 2,
     "silu": lambda x: x / (1 + mp.exp(-x))}


def minimiser(kind):
    return mp.findroot(lambda t: mp.diff(F[kind], t), M(-1))


def exp_form(c, yt):
    """1 + (c0 + c1 sqrt(y~) + c2 y~) exp(c3 (c4 - y~)^3): the bracket of Eq. (6) and of Eq. (8)."""
    return 1 + (c[0] + c[1] * mp.sqrt(yt) + c[2] * yt) * mp.exp(c[3] * (c[4] - yt) ** 3)


def q(kind, branch, y, fT):
    yt = y - fT
    if kind == "gelu_erf":
        if branch == "left":                                                       # Eq. (5)
            c = GELU_LEFT
            return c[0] * mp.sqrt(y + c[1]) * (2 * y + c[2] * mp.sqrt(-y)) * \
                (abs(c[3] * y ** 2 + abs(c[4] * y + c[5]) + c[6]) + c[7])
        return exp_form(GELU_RIGHT, yt)                                            # Eq. (6)
    if branch == "left":                                                           # Eq. (7)
        c = SILU_FOUR
        return (c[0] + c[1] * mp.sqrt(yt) + c[2] * yt + c[3] * yt ** 2) * (1 - y) + y
    return exp_form(SILU_FIVE, yt) * (1 - y) + y                                   # Eq. (8)


POINTS = [("gelu_erf", "right", "0"), ("gelu_erf", "right", "1"), ("gelu_erf", "right", "T"),
          ("gelu_erf", "left", "-1"), ("gelu_erf", "left", "-2"),
          ("silu", "right", "0"), ("silu", "right", "1"), ("silu", "right", "T"),
          ("silu", "left", "-2"), ("silu", "left", "-20")]

HEADER = """# Point values of the approximation q(y, s), Eqs. (5)-(8) with the coefficients
# of the appendix "Approximation Coefficients" exactly as printed (not rounded to
# binary32), y = f(x) and f(T) exact.  The paper prints no worked example; these
# six-digit values were computed with 40-digit arithmetic by a party other than
# the oracle's author before the oracle existed, under the reading that the two
# SiLU tables are printed under each other's labels; gen_q_point_values.py (mpmath,
# nothing of the oracle) reproduces them.  "T" in the x column means the minimiser of f.
# kind      branch  x      q"""


def rows():
    out = []
    for kind, branch, xs in POINTS:
        T = minimiser(kind)
        x = T if xs == "T" else M(xs)
        value = q(kind, branch, F[kind](x), F[kind](T))
        out.append((kind, branch, xs, mp.nstr(value, 6, strip_zeros=False, min_fixed=-10, max_fixed=10)))
    return out


if __name__ == "__main__":
    print(HEADER)
    for kind, branch, xs, value in rows():
        print(f"{kind:<11s} {branch:<7s} {xs:<6s} {value}")
