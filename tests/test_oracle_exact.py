"""Pins of the oracle's exact parts: forward f (O1), indicator and bit pack (O2),
derivative and branch-wise inverse (O3), T and f(T), and the storage rounding.

Each check compares the oracle with something that does not come from the
oracle: an identity, a closed form, a library routine (torch / scipy / numpy /
mpmath evaluating the textbook definition), or brute force.
"""
import math

import mpmath as mp
import numpy as np
import pytest
import scipy.optimize
import scipy.special
import scipy.stats
import torch

import oracle as O
import synth

KINDS = ["gelu_tanh", "gelu_erf", "silu"]
mp.mp.dps = 40


# textbook definitions at 40 digits (GELU: Hendrycks & Gimpel; SiLU: Elfwing et al.)
def mp_f(kind, x):
    with mp.workdps(700):      # 1 + tanh u and 1 + erf cancel hundreds of digits in the left tail
        return +_mp_f(kind, x)


def _mp_f(kind, x):
    x = mp.mpf(x)
    if kind == "gelu_erf":
        return x * (1 + mp.erf(x / mp.sqrt(2))) / 2
    if kind == "gelu_tanh":
        return x * (1 + mp.tanh(mp.sqrt(2 / mp.pi) * (x + mp.mpf("0.044715") * x ** 3))) / 2
    return x / (1 + mp.exp(-x))


def torch_f(kind, x):
    t = torch.tensor(x, dtype=torch.float64)
    if kind == "gelu_erf":
        return torch.nn.functional.gelu(t)
    if kind == "gelu_tanh":
        return torch.nn.functional.gelu(t, approximate="tanh")
    return torch.nn.functional.silu(t)


def all_bf16_values():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    with np.errstate(invalid="ignore"):                  # signalling NaN patterns
        v = synth.bf16_bits_to_f32(bits).astype(np.float64)
    return bits, v


# ---------------------------------------------------------------- O1

@pytest.mark.parametrize("kind", KINDS)
def test_forward_matches_mpmath_definition(kind):
    xs = np.concatenate([np.linspace(-14, 14, 337), [-37.5, -20.25, -1e-3, 1e-3, 1e-20, -1e-20, 50.0, 88.0]])
    ys = O.f(kind, xs)
    for x, y in zip(xs, ys):
        ref = mp_f(kind, x)
        if ref == 0:
            assert y == 0
        else:
            assert abs((mp.mpf(y) - ref) / ref) < mp.mpf("2e-13"), (kind, x, y, ref)


@pytest.mark.parametrize("kind", KINDS)
def test_forward_matches_torch_float64(kind):
    xs = np.linspace(-4.0, 12.0, 20001)
    ref = torch_f(kind, xs).numpy()
    got = O.f(kind, xs)
    # torch's tanh form cancels for x << 0, hence the absolute term
    assert np.all(np.abs(got - ref) <= 1e-14 * np.abs(ref) + 1e-15)


@pytest.mark.parametrize("kind", KINDS)
def test_forward_odd_part_identity(kind):
    # f(x) - f(-x) = x for x Phi(x), x sigma(x) and x sigma(2u(x)) (u odd)
    xs = np.concatenate([np.linspace(0, 30, 3001), np.logspace(-30, 2, 200)])
    d = O.f(kind, xs) - O.f(kind, -xs)
    assert np.all(np.abs(d - xs) <= 4e-16 * np.maximum(xs, 1e-300))


@pytest.mark.parametrize("kind", KINDS)
def test_forward_every_bf16_value(kind):
    bits, v = all_bf16_values()
    y = O.f(kind, v)
    finite = np.isfinite(v)
    assert np.all(np.isnan(y[np.isnan(v)]))
    # sign, bounds and limits that hold for every real x
    assert np.all(y[finite & (v > 0)] > 0)
    assert np.all(y[finite & (v < 0)] <= 0)
    assert np.all(y[finite] >= O.fT(kind))
    assert np.all(y[finite & (v > 0)] <= v[finite & (v > 0)])
    assert np.all(np.abs(y[finite]) <= np.abs(v[finite]))
    # infinities and zeros
    assert O.f(kind, [np.inf])[0] == np.inf
    ninf = O.f(kind, [-np.inf])[0]
    assert ninf == 0 and math.copysign(1, ninf) == -1
    assert O.f(kind, [0.0])[0] == 0
    # torch (float64) on every finite bf16 value where torch itself is well conditioned
    sel = finite & (v > -5) & (np.abs(v) < 1e30)
    ref = torch_f(kind, v[sel]).numpy()
    # (absolute term: torch's 1 + tanh u and 1 + erf cancel for x < 0)
    assert np.all(np.abs(y[sel] - ref) <= 1e-13 * np.abs(ref) + 3e-16 * (v[sel] < 0))
    # mpmath on a stride of the patterns, including the far left tail
    for i in range(0, 65536, 97):
        if finite[i] and abs(v[i]) < 1e4:
            ref = mp_f(kind, v[i])
            if abs(ref) > mp.mpf("1e-300"):
                assert abs((mp.mpf(y[i]) - ref) / ref) < mp.mpf("1e-12"), (kind, v[i])


# ---------------------------------------------------------------- T, f(T)

@pytest.mark.parametrize("kind", KINDS)
def test_T_is_the_minimiser(kind, golden):
    T, fT = O.T(kind), O.fT(kind)
    row = [r for r in golden("constants.txt") if r[0] == kind][0]
    assert abs(T - float(row[1])) < 4e-16
    assert abs(fT - float(row[2])) < 1e-16
    assert abs(O.df(kind, [T])[0]) < 1e-15
    for delta in (1e-6, 1e-3, 0.1, 1.0):
        lo, hi = O.f(kind, [T - delta, T + delta])
        assert lo > fT and hi > fT
    # f' changes sign exactly once on the negative axis
    xs = np.linspace(-30, 0, 30001)
    sgn = np.sign(O.df(kind, xs))
    assert np.count_nonzero(np.diff(sgn[sgn != 0])) == 1
    # binary32 roundings used by the indicator and by q
    assert O.T(kind, f32=True) == float(np.float32(T))
    assert O.fT(kind, f32=True) == float(np.float32(fT))


def test_T_silu_closed_form():
    w = scipy.special.lambertw(math.exp(-1.0)).real
    assert abs(O.T("silu") - (-1.0 - w)) < 4e-16
    assert abs(O.fT("silu") - (-w)) < 2e-16
    assert abs(O.fT("silu") - (1.0 + O.T("silu"))) < 2e-16


def test_T_gelu_erf_by_library_root_finder():
    g = lambda t: scipy.stats.norm.cdf(t) + t * scipy.stats.norm.pdf(t)
    root = scipy.optimize.brentq(g, -2.0, -0.5, xtol=1e-15, rtol=1e-15)
    assert abs(O.T("gelu_erf") - root) < 1e-14


# ---------------------------------------------------------------- O3: f'

@pytest.mark.parametrize("kind", KINDS)
def test_derivative_matches_mpmath_differentiation(kind):
    xs = np.concatenate([np.linspace(-9, 9, 145), [-20.0, -12.5, 15.0, 1e-8]])
    ds = O.df(kind, xs)
    for x, d in zip(xs, ds):
        ref = mp.diff(lambda t: mp_f(kind, t), mp.mpf(x))
        assert abs(mp.mpf(d) - ref) <= mp.mpf("1e-13") * abs(ref) + mp.mpf("1e-30"), (kind, x, d, ref)


@pytest.mark.parametrize("kind", KINDS)
def test_derivative_matches_torch_autograd(kind):
    xs = np.linspace(-4, 12, 4001)
    t = torch.tensor(xs, dtype=torch.float64, requires_grad=True)
    if kind == "gelu_erf":
        y = torch.nn.functional.gelu(t)
    elif kind == "gelu_tanh":
        y = torch.nn.functional.gelu(t, approximate="tanh")
    else:
        y = torch.nn.functional.silu(t)
    y.sum().backward()
    assert np.all(np.abs(O.df(kind, xs) - t.grad.numpy()) <= 1e-13)


@pytest.mark.parametrize("kind", KINDS)
def test_derivative_central_differences_and_symmetry(kind):
    xs = np.linspace(-12, 12, 2401)
    h = 1e-5
    fd = (O.f(kind, xs + h) - O.f(kind, xs - h)) / (2 * h)
    assert np.all(np.abs(fd - O.df(kind, xs)) <= 2e-9)
    # f(x) - f(-x) = x  =>  f'(x) + f'(-x) = 1
    assert np.all(np.abs(O.df(kind, xs) + O.df(kind, -xs) - 1.0) <= 4e-16)
    assert O.df(kind, [np.inf])[0] == 1.0 and O.df(kind, [-np.inf])[0] == 0.0


@pytest.mark.parametrize("kind", KINDS)
def test_derivative_maximum(kind, golden):
    row = [r for r in golden("derivative_maxima.txt") if r[0] == kind][0]
    xm, dm = float(row[1]), float(row[2])
    xs = np.linspace(0.5, 4, 350001)
    d = O.df(kind, xs)
    i = int(np.argmax(d))
    assert abs(xs[i] - xm) < 2e-5
    assert abs(d[i] - dm) < 2e-11                       # grid step 1e-5
    assert abs(O.df(kind, [xm])[0] - dm) < 1e-13
    if kind == "gelu_erf":
        r2 = math.sqrt(2.0)
        assert abs(dm - (scipy.stats.norm.cdf(r2) + r2 * scipy.stats.norm.pdf(r2))) < 1e-14


def test_silu_derivative_structure():
    # f' = sigma + y (1 - sigma): the structure behind Eqs. (7)-(8)
    xs = np.linspace(-30, 30, 6001)
    sig = scipy.special.expit(xs)
    sigc = scipy.special.expit(-xs)                      # 1 - sigma without cancellation
    assert np.all(np.abs(O.df("silu", xs) - (sig + O.f("silu", xs) * sigc)) <= 1e-15)


# ---------------------------------------------------------------- O3: inverse

@pytest.mark.parametrize("kind", KINDS)
def test_inverse_round_trip(kind):
    T = O.T(kind)
    xl = np.concatenate([np.linspace(-30 if kind == "silu" else -8, T, 4001)])
    xr = np.concatenate([np.linspace(T, 30, 4001), [100.0, 1e4, 1e10]])
    for x, s in ((xl, 1), (xr, 0)):
        y = O.f(kind, x)
        xi = O.finv(kind, y, np.full(x.size, s, np.uint8))
        # f(finv(y)) = y
        back = O.f(kind, xi)
        assert np.all(np.abs(back - y) <= 1e-14 * np.abs(y) + 1e-300)
        # finv(f(x)) = x away from the minimum, where the inverse is well conditioned
        far = np.abs(x - T) > 1e-2
        assert np.all(np.abs(xi[far] - x[far]) <= 1e-10 * np.maximum(1, np.abs(x[far])))
        assert np.all((xi <= T) if s else (xi >= T))


@pytest.mark.parametrize("kind", KINDS)
def test_inverse_every_bf16_value_and_edges(kind):
    _, v = all_bf16_values()
    T, fT = O.T(kind), O.fT(kind)
    fin = np.isfinite(v)
    for s in (0, 1):
        ok = fin & (v >= fT) & ((v < 0) if s else np.ones_like(fin))
        y = v[ok]
        xi = O.finv(kind, y, np.full(y.size, s, np.uint8))
        assert np.all(np.isfinite(xi))
        back = O.f(kind, xi)
        assert np.all(np.abs(back - y) <= 1e-13 * np.abs(y) + 1e-300)
    # the two branches meet at T
    assert O.finv(kind, [fT], [0])[0] == T and O.finv(kind, [fT], [1])[0] == T
    # values no branch reaches
    assert np.isnan(O.finv(kind, [fT - 1e-3], [0])[0])
    assert np.isnan(O.finv(kind, [0.5], [1])[0])
    assert O.finv(kind, [-0.0], [1])[0] == -np.inf
    assert O.finv(kind, [np.inf], [0])[0] == np.inf


# ---------------------------------------------------------------- O2

@pytest.mark.parametrize("kind,count", [("silu", 16348), ("gelu_erf", 16447), ("gelu_tanh", 16447)])
def test_indicator_over_all_bf16(kind, count):
    _, v = all_bf16_values()
    s = O.indicator(kind, v)
    T32 = np.float32(O.T(kind))
    with np.errstate(invalid="ignore"):
        expect = (v.astype(np.float32) < T32)
    assert np.array_equal(s.astype(bool), expect)
    # 16 256 finite negative bf16 patterns lie at or below -1 ... counted independently:
    # patterns 0x8000|m with value < T are the contiguous block from the first
    # pattern below T up to -inf (0xFF80)
    first = int(synth.f32_to_bf16_bits(np.array([T32], np.float32))[0])
    while synth.bf16_bits_to_f32(np.array([first], np.uint16))[0] >= T32:
        first += 1
    assert int(s.sum()) == 0xFF80 - first + 1            # includes -inf
    assert int(s[np.isfinite(v)].sum()) == count
    # ties and specials
    assert O.indicator(kind, [O.T(kind, f32=True)])[0] == 0
    assert O.indicator(kind, [np.nextafter(np.float32(T32), np.float32(-9))])[0] == 1
    assert list(O.indicator(kind, [np.nan, 0.0, -0.0, np.inf, -np.inf])) == [0, 0, 0, 0, 1]


@pytest.mark.parametrize("n", [0, 1, 7, 8, 63, 64, 65, 511, 513, 4099])
def test_pack_layout(n):
    rng = np.random.default_rng(n)
    s = (rng.random(n) < 0.3).astype(np.uint8)
    m = O.pack(s)
    assert m.size == 8 * ((n + 63) // 64) == O.mask_bytes(n)
    # numpy's little-endian bit packing is the paper's byte layout
    ref = np.packbits(s, bitorder="little")
    assert np.array_equal(m[:ref.size], ref)
    assert not m[ref.size:].any()
    # as 64-bit little-endian words: bit (i mod 64) of word (i div 64)
    words = m.view("<u8")
    for i in range(n):
        assert (int(words[i // 64]) >> (i % 64)) & 1 == s[i]
        assert (int(m[i // 8]) >> (i % 8)) & 1 == s[i]
    assert sum(bin(int(w)).count("1") for w in words) == int(s.sum())
    assert np.array_equal(O.unpack(m, n), s)


# ---------------------------------------------------------------- storage rounding

def test_round_to_fp32_matches_numpy_cast():
    rng = np.random.default_rng(5)
    v = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-45, 39, 20000),
                        [0.0, -0.0, 1e-46, -1e-46, 3.4028235677973366e38, 3.5e38, -1e39, np.inf, np.nan,
                         1.0 + 2.0 ** -24, 1.0 + 3 * 2.0 ** -24, 2.0 ** -149, 2.0 ** -150, 1.5 * 2.0 ** -149]])
    with np.errstate(over="ignore"):
        ref = v.astype(np.float32).astype(np.float64)
    got = O.round_to("fp32", v)
    assert np.array_equal(got, ref, equal_nan=True)
    assert np.array_equal(np.signbit(got), np.signbit(ref))


def test_round_to_bf16_matches_torch_cast_and_ties():
    rng = np.random.default_rng(6)
    # binary32 inputs: torch rounds those to bfloat16 once, to nearest even
    v32 = (rng.standard_normal(40000) * 10.0 ** rng.integers(-44, 38, 40000)).astype(np.float32)
    ref = torch.from_numpy(v32).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_to("bf16", v32.astype(np.float64))
    assert np.array_equal(got, ref)
    assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(v32)).astype(np.float64), ref)
    # doubles that are not binary32 values: ties, and a value a double->float->bf16
    # cast would round twice (1 + 2^-8 + 2^-30 must go up, not to even)
    cases = {1.0 + 2.0 ** -8: 1.0, 1.0 + 3 * 2.0 ** -8: 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -8 + 2.0 ** -30: 1.0 + 2.0 ** -7,
             -(1.0 + 2.0 ** -8): -1.0, 2.0 ** -133: 2.0 ** -133, 2.0 ** -134: 0.0, 1.5 * 2.0 ** -133: 2.0 ** -132,
             3.3895313892515355e38: 3.3895313892515355e38, 3.4e38: np.inf, 0.0: 0.0}
    for v, r in cases.items():
        assert O.round_to("bf16", [v])[0] == r, (v, r)
    # every bf16 value is a fixed point
    _, allv = all_bf16_values()
    assert np.array_equal(O.round_to("bf16", allv), allv, equal_nan=True)


# ---------------------------------------------------------------- sanitizer build of the oracle

def test_oracle_runs_clean_under_ubsan_and_bounds_checks(tmp_path):
    """The oracle compiled with -fsanitize=undefined (traps on any finding) on ragged sizes."""
    import subprocess
    import sys
    import os
    so = tmp_path / "liboracle_ubsan.so"
    O.build(force=True, out=str(so), extra_flags=("-fsanitize=undefined", "-fno-sanitize-recover=all", "-g"))
    code = f"""
import sys, numpy as np
sys.path.insert(0, {os.path.dirname(os.path.dirname(O.__file__))!r})
import oracle as O
O._lib = O.load({str(so)!r})
rng = np.random.default_rng(0)
for n in (0, 1, 7, 63, 64, 65, 1000):
    x = rng.standard_normal(n) * 3
    x[:3] = [np.nan, np.inf, -np.inf][:min(3, n)]
    g = rng.standard_normal(n)
    for kind in ("gelu_tanh", "gelu_erf", "silu"):
        for dtype in ("fp32", "bf16"):
            ye, ys, m = O.invact_fwd(kind, dtype, x)
            O.invact_bwd(kind, ys, m, g)
            a, s, h, m2 = O.glu_fwd(kind, dtype, x, g)
            O.glu_bwd(kind, s, g, m2, g)
            _, yt = O.pbit_fwd(kind, dtype, x)
            O.pbit_bwd(kind, dtype, yt, g)
        O.finv(kind, O.f(kind, x), O.indicator(kind, x))
    assert O.unpack(O.pack((x < 0).astype(np.uint8)), n).sum() == (x < 0).sum()
print("clean")
"""
    res = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0 and "clean" in res.stdout, res.stderr[-2000:]
