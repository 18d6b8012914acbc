"""Pins of the oracle's precision-bit variant (Method, "Precision Bit Inverted
Activation"): the forward stores f(x) with its lowest significand bit replaced by
the indicator, Y = (Y & ~1) | S; the backward reads S = Y & 1 and evaluates q at
the stored Y.  The rule is a bit operation, so it is pinned by redoing it with
numpy's integer views of the storage patterns."""
import numpy as np
import pytest

import oracle as O
import synth

KINDS = ["gelu_tanh", "gelu_erf", "silu"]


def patterns(values, dtype):
    """Storage bit patterns (as uint32) of float64 values lying on the dtype's grid."""
    st = synth.f64_to_storage_exact(values, dtype)
    return st.view(np.uint32).copy() if dtype == "fp32" else st.astype(np.uint32)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_forward_replaces_the_lowest_bit(kind, dtype):
    rng = np.random.default_rng(3)
    x = synth.storage_to_f64(synth.to_storage((rng.standard_normal(50000) * 2.5).astype(np.float32), dtype), dtype)
    x = np.concatenate([x, [0.0, -0.0, O.T(kind, f32=True), -30.0, 30.0, np.inf, -np.inf]])
    ye, ys = O.pbit_fwd(kind, dtype, x)
    plain = O.round_to(dtype, ye)
    s = O.indicator(kind, x).astype(np.uint32)
    p_tag, p_plain = patterns(ys, dtype), patterns(plain, dtype)
    assert np.array_equal(p_tag & 1, s)                               # the bit carries the indicator
    assert np.array_equal(p_tag >> 1, p_plain >> 1)                   # nothing else changed
    same = (p_plain & 1) == s
    assert np.array_equal(ys[same], plain[same])
    assert np.array_equal(ye, O.f(kind, x))
    # at most one unit in the last place away from the correctly rounded value
    p = 24 if dtype == "fp32" else 8
    fin = np.isfinite(ye) & (np.abs(plain) >= 2.0 ** -126)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(plain[fin]))) - p + 1)
    assert np.all(np.abs(ys[fin] - plain[fin]) <= ulp)
    # -inf maps to -0, whose pattern becomes the smallest negative subnormal once tagged
    assert ys[-1] < 0 and abs(ys[-1]) == 2.0 ** (-126 - (p - 1))
    assert ys[-2] == np.inf


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_tag_and_read_round_trip(dtype):
    if dtype == "bf16":
        bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
        with np.errstate(invalid="ignore"):
            v = synth.storage_to_f64(bits, dtype)
        pat = bits.astype(np.uint32)
    else:
        rng = np.random.default_rng(9)
        pat = rng.integers(0, 2 ** 32, 200000, dtype=np.uint64).astype(np.uint32)
        with np.errstate(invalid="ignore"):
            v = pat.view(np.float32).astype(np.float64)
    L = O.lib()
    d = O.DTYPES[dtype]
    fin = np.isfinite(v)            # the forward never tags an infinity with 1, and a tagged infinity is a NaN
    for s in (0, 1):
        tagged = np.array([L.oracle_tag_lsb(d, float(x), s) for x in v[fin][::17]])
        assert np.array_equal(patterns(tagged, dtype), (pat[fin][::17] & ~np.uint32(1)) | s)
        assert all(L.oracle_read_lsb(d, float(t)) == s for t in tagged[::5])


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_backward_reads_the_bit_and_uses_the_stored_value(kind, dtype):
    rng = np.random.default_rng(5)
    x = synth.storage_to_f64(synth.to_storage((rng.standard_normal(20000) * 2).astype(np.float32), dtype), dtype)
    g = rng.standard_normal(x.size)
    _, ys = O.pbit_fwd(kind, dtype, x)
    gx = O.pbit_bwd(kind, dtype, ys, g)
    s = (patterns(ys, dtype) & 1).astype(np.uint8)
    assert np.array_equal(s, O.indicator(kind, x))
    assert np.array_equal(gx, g * O.q(kind, ys, s))
    # the price of the variant: the stored activation moves by up to one ulp, the gradient hardly at all
    _, plain, m = O.invact_fwd(kind, dtype, x)
    ref = O.invact_bwd(kind, plain, m, g)
    assert np.max(np.abs(gx - ref)) <= (4e-2 if dtype == "bf16" else 1e-3) * np.max(np.abs(g))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_a_nan_stays_a_nan_through_the_tag(kind, dtype):
    """The indicator of a NaN is 0 and clearing the lowest bit must not turn it into an infinity."""
    ye, ys = O.pbit_fwd(kind, dtype, np.array([np.nan, -np.nan]))
    assert np.all(np.isnan(ye)) and np.all(np.isnan(ys))
    assert np.all(np.isnan(O.pbit_bwd(kind, dtype, ys, np.ones(2))))
