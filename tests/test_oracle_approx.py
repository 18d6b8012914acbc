"""Pins of the oracle's approximation q(y, s) (Eqs. (5)-(8)) and of the layer
forward / backward built on it (Algorithm 1, gated block).

The paper prints neither a worked example nor an error bound for q, so q is
"parity unpinned" in the strict sense.  What pins it here:
  * it must approximate the exact f'(f^-1(y)) -- which is pinned independently
    in test_oracle_exact.py -- within per-region bounds;
  * point values computed by another party (tests/golden/q_point_values.txt);
  * limits that follow from the formulas;
  * planted mistakes (a dropped term, a flipped sign, swapped coefficients, the
    SiLU tables used as labelled, edits of the C source) must each break one of
    the above.
"""
import os
import re
import shutil
import subprocess

import mpmath as mp
import numpy as np
import pytest

import oracle as O
import synth

KINDS = ["gelu_tanh", "gelu_erf", "silu"]
KID = O.KINDS

# max |q - f'| allowed per x-interval: (kind, branch) -> [(x_lo, x_hi, bound)].
# "T" stands for the minimiser.  The approximation is worst just right of T
# (about 2e-2 for GELU) and a few 1e-3 elsewhere.
def regions(kind, T):
    if kind == "silu":
        return {1: [(-40, -5, 1.0e-3), (-5, -1.5, 3.0e-4), (-1.5, T, 1.1e-3)],
                0: [(T, -1.0, 2.3e-3), (-1.0, 0, 1.2e-3), (0, 2, 2.5e-4), (2, 3, 3.5e-4),
                    (3, 8, 3.5e-3), (8, 40, 1.9e-3)]}
    left_near = 1.6e-3 if kind == "gelu_erf" else 9.5e-3     # tanh form reuses the erf-fitted constants
    return {1: [(-40, -10, 1e-9), (-10, -5, 1.0e-4), (-5, -3, 8.5e-4), (-3, -0.9, 2.3e-3),
                (-0.9, T, left_near)],
            0: [(T, -0.7, 2.3e-2), (-0.7, -0.55, 1.8e-2), (-0.55, 0, 4.7e-3), (0, 5, 3.0e-3),
                (5, 8, 1e-5), (8, 40, 1e-9)]}


class Lib:
    """Thin functional view of one compiled oracle (the real one or a mutant)."""

    def __init__(self, lib):
        self.lib = lib

    def f(self, kind, x):
        x = np.ascontiguousarray(x, np.float64); y = np.empty_like(x)
        self.lib.oracle_f(KID[kind], x, y, x.size)
        return y

    def df(self, kind, x):
        x = np.ascontiguousarray(x, np.float64); y = np.empty_like(x)
        self.lib.oracle_df(KID[kind], x, y, x.size)
        return y

    def q(self, kind, y, s, coeffs=None, fT=None):
        y = np.ascontiguousarray(y, np.float64)
        s = np.ascontiguousarray(np.broadcast_to(np.uint8(s), y.shape), np.uint8)
        out = np.empty_like(y)
        if coeffs is None and fT is None:
            self.lib.oracle_q(KID[kind], y, s, out, y.size)
        else:
            c = np.empty(22); self.lib.oracle_default_coeffs(c)
            c = c if coeffs is None else np.ascontiguousarray(coeffs, np.float64)
            t = self.lib.oracle_fT_f32(KID[kind]) if fT is None else fT
            self.lib.oracle_q_coeffs(KID[kind], c, t, y, s, out, y.size)
        return out

    def printed(self):
        c = np.empty(22); self.lib.oracle_printed_coeffs(c); return c


def q_pin_failures(L, golden_rows, coeffs=None):
    """Run every pin of q against oracle view L; return the list of failures."""
    bad = []
    for kind in KINDS:
        T = L.lib.oracle_T(KID[kind])
        for s, regs in regions(kind, T).items():
            for lo, hi, bound in regs:
                x = np.linspace(lo, hi, 4001)
                err = np.abs(L.q(kind, L.f(kind, x), s, coeffs=coeffs) - L.df(kind, x))
                if not np.all(err <= bound):
                    bad.append(f"{kind} s={s} x in [{lo:.3g},{hi:.3g}]: {np.nanmax(err):.3g} > {bound:.3g}")
        # limits: q_right -> 1; exact 1 at +inf
        big = L.q(kind, np.array([60.0, 1e3, 1e30, np.inf]), 0, coeffs=coeffs)
        if not np.all(np.abs(big - 1.0) <= 1e-12):
            bad.append(f"{kind} q_right(large y) = {big}")
    # GELU left: zero at y = 0-, never positive on [f(T), 0]
    for kind in ("gelu_erf", "gelu_tanh"):
        fT = L.lib.oracle_fT(KID[kind])
        y = np.linspace(fT, 0.0, 20001)
        ql = L.q(kind, y, 1, coeffs=coeffs)
        if not (abs(L.q(kind, np.array([-0.0]), 1, coeffs=coeffs)[0]) == 0 and np.all(ql <= 0)):
            bad.append(f"{kind} q_left sign / zero at 0-")
    # point values (unrounded constants unless the caller planted its own)
    for kind, branch, xs, qs in golden_rows:
        T = L.lib.oracle_T(KID[kind])
        x = T if xs == "T" else float(xs)
        c = L.printed() if coeffs is None else coeffs
        got = L.q(kind, L.f(kind, np.array([x])), 1 if branch == "left" else 0,
                  coeffs=c, fT=L.lib.oracle_fT(KID[kind]))[0]
        digits = len(qs.split(".")[1])
        if abs(got - float(qs)) > 0.6 * 10.0 ** -digits:
            bad.append(f"{kind} {branch} x={xs}: {got} vs {qs}")
    return bad


@pytest.fixture(scope="module")
def rows(golden):
    return golden("q_point_values.txt")


def test_q_passes_every_pin(rows):
    assert q_pin_failures(Lib(O.lib()), rows) == []


def test_q_rounded_constants_stay_close_to_printed(rows):
    # the binary32-rounded constants change q only where sqrt has a steep slope
    L = Lib(O.lib())
    for kind in KINDS:
        T, fT = O.T(kind), O.fT(kind)
        for s, lo, hi in ((1, -30.0, T - 1e-2), (0, T + 1e-2, 30.0)):
            x = np.linspace(lo, hi, 20001)
            y = L.f(kind, x)
            a = L.q(kind, y, s)
            b = L.q(kind, y, s, coeffs=L.printed(), fT=fT)
            assert np.max(np.abs(a - b)) < 1e-5


# ---------------------------------------------------------------- planted mistakes: constants

def coefficient_mutants():
    base = O.printed_coeffs()
    names = [f"gelu_left.c{i}" for i in range(8)] + [f"gelu_right.c{i}" for i in range(5)] + \
            [f"silu_left.c{i}" for i in range(4)] + [f"silu_right.c{i}" for i in range(5)]
    out = []
    for i, nm in enumerate(names):
        z = base.copy(); z[i] = 0.0; out.append((f"drop {nm}", z))
        f = base.copy(); f[i] = -f[i]; out.append((f"flip {nm}", f))
    groups = [(0, 8), (8, 13), (13, 17), (17, 22)]
    for a, b in groups:
        for i in range(a, b - 1):
            w = base.copy(); w[i], w[i + 1] = w[i + 1], w[i]
            out.append((f"swap {names[i]} <-> {names[i + 1]}", w))
    return out


@pytest.mark.parametrize("name,coeffs", coefficient_mutants(), ids=[m[0] for m in coefficient_mutants()])
def test_planted_coefficient_mistake_is_caught(name, coeffs, rows):
    assert q_pin_failures(Lib(O.lib()), rows, coeffs=coeffs), f"pins did not notice: {name}"


def test_silu_tables_as_labelled_are_off_by_order_one():
    # Reading: the appendix prints the two SiLU tables under each other's labels.
    # Used as labelled, Eq. (7) would get five numbers for four slots and Eq. (8)
    # four for five; whichever way they are forced in, the error is O(1).
    c = O.printed_coeffs()
    five, four = c[17:22].copy(), c[13:17].copy()
    wrong = c.copy()
    wrong[13:17] = five[:4]                      # Eq. (7) with the table labelled "left"
    wrong[17:22] = np.append(four, 0.0)          # Eq. (8) with the table labelled "right"
    L = Lib(O.lib())
    T = O.T("silu")
    xl, xr = np.linspace(-10, T, 2001), np.linspace(T, 10, 2001)
    el = np.abs(L.q("silu", L.f("silu", xl), 1, coeffs=wrong) - L.df("silu", xl)).max()
    er = np.abs(L.q("silu", L.f("silu", xr), 0, coeffs=wrong) - L.df("silu", xr)).max()
    assert el > 0.5 and er > 0.1
    # and the 4-coefficient table's c0 is sigma(T), as Eq. (7) needs at y~ = 0
    assert abs(four[0] - 1.0 / (1.0 + np.exp(-T))) < 1e-3
    # GELU-left c1 is -f(T) of the erf form, not of the tanh form
    assert abs(c[1] + O.fT("gelu_erf")) < 2e-6 < abs(c[1] + O.fT("gelu_tanh"))


# ---------------------------------------------------------------- planted mistakes: source

SOURCE_MUTANTS = [
    ("eq7/8 (1 - y) -> (1 + y), first", r"return a \* \(1\.0 - y\) \+ y;", "return a * (1.0 + y) + y;"),
    ("eq7 drops + y", r"return a \* \(1\.0 - y\) \+ y;", "return a * (1.0 - y);"),
    ("eq8 (1 - y) -> (1 + y)", r"silu_right, yt\) \* \(1\.0 - y\)", "silu_right, yt) * (1.0 + y)"),
    ("eq8 drops the factor (1 - y)", r"silu_right, yt\) \* \(1\.0 - y\)", "silu_right, yt)"),
    ("exp form: c4 - yt -> yt - c4", r"double d = c\[4\] - yt;", "double d = yt - c[4];"),
    ("exp form: cube -> square", r"c\[3\] \* d \* d \* d", "c[3] * d * d"),
    ("exp form: sign of exponent", r"exp\(c\[3\] \* d", "exp(-c[3] * d"),
    ("exp form: sqrt dropped", r"c\[1\] \* sqrt\(yt\) \+ c\[2\] \* yt\) \* exp", "c[1] * yt + c[2] * yt) * exp"),
    ("eq6: 1 + h -> h", r"return 1\.0 \+ exp_form\(cs->gelu_right", "return exp_form(cs->gelu_right"),
    ("y~ = y + f(T)", r"double yt = clamp0\(y - fT\);", "double yt = clamp0(y + fT);"),
    ("eq6 y~ = y + f(T)", r"gelu_right, clamp0\(y - fT\)", "gelu_right, clamp0(y + fT)"),
    ("eq5: 2y -> y", r"\(2\.0 \* y \+ c\[2\]", "(y + c[2]"),
    ("eq5: sqrt(-y) -> sqrt(y)", r"sqrt\(clamp0\(-y\)\)\) \* outer", "sqrt(clamp0(y))) * outer"),
    ("eq5: sqrt(y + c1) -> sqrt(y - c1)", r"sqrt\(clamp0\(y \+ c\[1\]\)\)", "sqrt(clamp0(y - c[1]))"),
    ("eq5: y^2 -> y", r"c\[3\] \* y \* y \+ inner", "c[3] * y + inner"),
    ("eq5: inner abs dropped", r"double inner = fabs\(c\[4\] \* y \+ c\[5\]\);", "double inner = c[4] * y + c[5];"),
    ("eq5: outer abs dropped", r"double outer = fabs\(c\[3\] \* y \* y \+ inner \+ c\[6\]\) \+ c\[7\];",
     "double outer = (c[3] * y * y + inner + c[6]) + c[7];"),
    ("eq5: + c7 -> - c7", r"\+ c\[6\]\) \+ c\[7\];", "+ c[6]) - c[7];"),
    ("eq7: y~^2 -> y~", r"c\[3\] \* yt \* yt;", "c[3] * yt;"),
    ("eq7: sqrt dropped", r"c\[0\] \+ c\[1\] \* sqrt\(yt\) \+ c\[2\] \* yt \+ c\[3\]", "c[0] + c[1] * yt + c[2] * yt + c[3]"),
    ("silu tables exchanged", r"const double \*c = cs->silu_left;", "const double *c = cs->silu_right;"),
    ("gelu branches exchanged", r"if \(s\) \{ +/\* Eq\. \(5\) \*/", "if (!s) {"),
    ("silu branches exchanged", r"if \(s\) \{ +/\* Eq\. \(7\) \*/", "if (!s) {"),
]


@pytest.mark.parametrize("name,pattern,repl", SOURCE_MUTANTS, ids=[m[0] for m in SOURCE_MUTANTS])
def test_planted_source_mistake_is_caught(name, pattern, repl, rows, tmp_path):
    src = open(os.path.join(os.path.dirname(O.__file__), "invact_oracle.c")).read()
    mutated, count = re.subn(pattern, repl, src, count=1)
    assert count == 1, f"pattern of mutant '{name}' no longer matches the oracle source"
    c_file = tmp_path / "mutant.c"
    c_file.write_text(mutated)
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-shared", "-fPIC", "-o", str(so), str(c_file), "-lm"], check=True)
    L = Lib(O.load(str(so)))
    assert q_pin_failures(L, rows), f"pins did not notice: {name}"


# ---------------------------------------------------------------- readings

def test_eq8_as_printed_equals_the_evaluated_form():
    # (1 + h)(1 - y) + y = 1 + h (1 - y); checked in 60-digit arithmetic with the
    # oracle's own (binary32-rounded) constants, also for y beyond 2^53.
    mp.mp.dps = 60
    c = [mp.mpf(v) for v in O.default_coeffs()[17:22]]
    fT = mp.mpf(O.fT("silu", f32=True))
    for y in (-0.27, -0.1, 0.0, 0.3, 1.0, 2.5, 7.0, 20.0, 1e3, 1e17, 1e30):
        ym = mp.mpf(y)
        yt = max(ym - fT, 0)
        h = (c[0] + c[1] * mp.sqrt(yt) + c[2] * yt) * mp.exp(c[3] * (c[4] - yt) ** 3)
        printed = (1 + h) * (1 - ym) + ym
        got = O.q("silu", [y], [0])[0]
        assert abs(mp.mpf(got) - printed) < mp.mpf("1e-13"), (y, got, printed)


@pytest.mark.parametrize("kind", KINDS)
def test_clamp_and_specials(kind):
    fT32 = O.fT(kind, f32=True)
    # below the stored minimum the right branch stays at its value at y~ = 0
    a = O.q(kind, [fT32 - 1e-3, fT32 - 2.0 ** -9, fT32], [0, 0, 0])
    if kind == "silu":
        h0 = O.q(kind, [fT32], [0])[0]           # 1 + h(0)(1 - y): h(0) from the value at fT
        h0 = (h0 - 1.0) / (1.0 - fT32)
        assert np.allclose(a[:2], 1.0 + h0 * (1.0 - np.array([fT32 - 1e-3, fT32 - 2.0 ** -9])), rtol=0, atol=1e-15)
    else:
        assert a[0] == a[1] == a[2]
    # left branch never produces NaN from a negative sqrt argument
    ys = np.array([fT32 - 1e-3, fT32, -0.0, 0.0, 1e-3])
    assert np.all(np.isfinite(O.q(kind, ys, np.ones(5, np.uint8))))
    # NaN goes through; +inf on the right branch is 1
    assert np.isnan(O.q(kind, [np.nan], [0])[0]) and np.isnan(O.q(kind, [np.nan], [1])[0])
    assert O.q(kind, [np.inf], [0])[0] == 1.0


def test_known_sign_defects_of_the_printed_approximation_are_reproduced():
    # With the printed coefficients the approximate derivative has the wrong sign
    # on a short interval right of T (GELU) and does not vanish at y -> 0- (SiLU).
    # That is the paper's method; the oracle reproduces it rather than repairing it.
    k = "gelu_erf"
    assert -0.02 < O.q(k, [O.fT(k, f32=True)], [0])[0] < -0.017
    x = np.linspace(O.T(k) + 1e-4, -0.70, 2001)
    q = O.q(k, O.f(k, x), np.zeros(x.size, np.uint8))
    root = x[np.argmax(q > 0)]
    assert -0.72 < root < -0.71
    assert -9e-4 < O.q("silu", [-1e-30], [1])[0] < -8e-4
    assert 1.6e-3 < O.q("silu", [O.fT("silu", f32=True)], [0])[0] < 1.9e-3


# ---------------------------------------------------------------- layer forward / backward

@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("n", [0, 1, 63, 64, 65, 1000])
def test_layer_forward_backward_compose_the_parts(kind, dtype, n):
    rng = np.random.default_rng(n + 7)
    x = synth.storage_to_f64(synth.to_storage(rng.standard_normal(n).astype(np.float32) * 2, dtype), dtype)
    g = synth.storage_to_f64(synth.to_storage(rng.standard_normal(n).astype(np.float32), dtype), dtype)
    ye, ys, m = O.invact_fwd(kind, dtype, x)
    assert np.array_equal(ye, O.f(kind, x))
    assert np.array_equal(ys, O.round_to(dtype, ye))
    assert np.array_equal(m, O.pack(O.indicator(kind, x)))
    assert m.size == O.mask_bytes(n)
    # what is stored lies on the storage grid and within half an ulp of f(x)
    assert np.array_equal(synth.storage_to_f64(synth.f64_to_storage_exact(ys, dtype), dtype), ys)
    p = 24 if dtype == "fp32" else 8
    with np.errstate(divide="ignore"):
        ulp = 2.0 ** (np.floor(np.log2(np.abs(ye))) - p + 1)
    assert np.all(np.abs(ys - ye) <= 0.5 * ulp)
    gx = O.invact_bwd(kind, ys, m, g)
    assert np.array_equal(gx, g * O.q(kind, ys, O.unpack(m, n)))


@pytest.mark.parametrize("kind", KINDS)
def test_gated_block_reduces_to_products(kind):
    n = 777
    rng = np.random.default_rng(3)
    gate = synth.storage_to_f64(synth.to_storage(rng.standard_normal(n).astype(np.float32), "bf16"), "bf16")
    up = synth.storage_to_f64(synth.to_storage(rng.standard_normal(n).astype(np.float32), "bf16"), "bf16")
    gh = synth.storage_to_f64(synth.to_storage(rng.standard_normal(n).astype(np.float32) * 0.01, "bf16"), "bf16")
    ae, as_, he, m = O.glu_fwd(kind, "bf16", gate, up)
    ye, ys, m2 = O.invact_fwd(kind, "bf16", gate)
    assert np.array_equal(ae, ye) and np.array_equal(as_, ys) and np.array_equal(m, m2)
    assert np.array_equal(he, ye * up)
    gg, gu = O.glu_bwd(kind, as_, up, m, gh)
    assert np.array_equal(gu, gh * as_)
    assert np.array_equal(gg, gh * up * O.q(kind, as_, O.unpack(m, n)))
    # chain rule against the exact derivative: d h / d gate = up f'(gate), up to the
    # approximation error of q and the rounding of the stored activation
    exact = gh * up * O.df(kind, gate)
    assert np.max(np.abs(gg - exact)) <= 4e-2 * np.max(np.abs(gh * up))


def test_point_values_can_be_regenerated_from_the_printed_formulas():
    """tests/golden/gen_q_point_values.py (mpmath, no oracle code) reproduces every stored digit of the fixture."""
    import importlib.util
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "gen_q_point_values.py")
    spec = importlib.util.spec_from_file_location("gen_q_point_values", path)
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    stored = {}
    with open(os.path.join(os.path.dirname(path), "q_point_values.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                kind, branch, xs, value = line.split()
                stored[(kind, branch, xs)] = value
    assert set(stored) == set(gen.POINTS)
    for kind, branch, xs in gen.POINTS:
        T = gen.minimiser(kind)
        x = T if xs == "T" else gen.M(xs)
        value = gen.q(kind, branch, gen.F[kind](x), gen.F[kind](T))
        text = stored[(kind, branch, xs)]
        digits = len(text.split(".")[1])
        assert abs(value - gen.M(text)) <= gen.M(10) ** -digits * gen.M("0.5001"), (kind, branch, xs, value, text)
