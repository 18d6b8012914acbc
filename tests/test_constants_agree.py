"""The kernels' constants (csrc/invact_constants.h, written by csrc/gen_constants.py) and
the oracle's (computed inside invact_oracle.c) are derived independently; "the same
approximation" needs them to be the same binary32 numbers."""
import os
import re

import numpy as np

import oracle as O

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                      "paper_2407_15545_amd", "csrc", "invact_constants.h")


def header_floats(name, text):
    m = re.search(name + r"(?:\[\d+\])? = \{? ?([^;}]*?) ?\}?;", text)
    return [np.float32(v.strip().rstrip("f")) for v in m.group(1).split(",")]


def test_header_constants_equal_the_oracles():
    text = open(HEADER).read()
    c = O.default_coeffs()
    groups = {"gelu_left": c[0:8], "gelu_right": c[8:13], "silu_left": c[13:17], "silu_right": c[17:22]}
    for name, want in groups.items():
        got = header_floats(name, text)
        assert [float(g) for g in got] == [float(w) for w in want], name
    for kind in ("gelu_tanh", "gelu_erf", "silu"):
        assert float(header_floats("T_" + kind, text)[0]) == O.T(kind, f32=True), kind
        assert float(header_floats("fT_" + kind, text)[0]) == O.fT(kind, f32=True), kind


def test_expanded_cubic_is_the_cubic():
    # t[0] + y (t[1] + y (t[2] + y t[3])) == log2(e) c3 (c4 - y)^3 with the binary32 c3, c4
    text = open(HEADER).read()
    c = O.default_coeffs()
    for name, right in (("gelu_right_exp2", c[8:13]), ("silu_right_exp2", c[17:22])):
        t = [float(v) for v in header_floats(name, text)]
        y = np.linspace(0, 30, 3001)
        horner = t[0] + y * (t[1] + y * (t[2] + y * t[3]))
        exact = np.log2(np.e) * right[3] * (right[4] - y) ** 3
        assert np.all(np.abs(horner - exact) <= 1.5e-7 * np.abs(exact) + 3e-8)
        assert all(v < 0 for v in t)        # one sign: Horner's rule cannot cancel
