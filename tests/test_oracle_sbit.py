"""Pins of the oracle's sign-bit variant (Section 3.3, "Sign-bit Inverted Activation", and its
listing): the forward stores f(x) - C (C = min f, so the value is non-negative) with its sign bit
replaced by the indicator; the consumer rebuilds |Y| + C; the backward reads the sign and evaluates
q at |Y| + C.  Pinned by redoing the bit operations with numpy's integer views, by the round trip
back to f(x), and by the ordinary variant (whose result it must reproduce up to the rounding of
the stored value)."""
import numpy as np
import pytest

import oracle as O
import synth

KINDS = ["gelu_tanh", "gelu_erf", "silu"]
P = {"fp32": 24, "bf16": 8}


def patterns(values, dtype):
    st = synth.f64_to_storage_exact(values, dtype)
    return st.view(np.uint32).copy() if dtype == "fp32" else st.astype(np.uint32)


def sign_bit(dtype):
    return np.uint32(0x80000000 if dtype == "fp32" else 0x8000)


def inputs(dtype, n=50000, seed=3):
    rng = np.random.default_rng(seed)
    x = synth.storage_to_f64(synth.to_storage((rng.standard_normal(n) * 2.5).astype(np.float32), dtype), dtype)
    return x


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_forward_stores_f_minus_its_minimum_with_the_indicator_as_sign(kind, dtype):
    x = np.concatenate([inputs(dtype), [0.0, -0.0, O.T(kind, f32=True), -30.0, 30.0, np.inf, -np.inf]])
    C = O.fT(kind, f32=True)
    ve, yt = O.sbit_fwd(kind, dtype, x)
    s = O.indicator(kind, x).astype(np.uint32)
    pat = patterns(yt, dtype)
    assert np.array_equal((pat & sign_bit(dtype)) != 0, s.astype(bool))            # the sign carries the indicator
    assert np.array_equal(pat & ~sign_bit(dtype), patterns(O.round_to(dtype, ve), dtype))   # the rest is RNE(f - C)
    f = O.f(kind, x)
    assert np.all(ve >= 0)
    fin = np.isfinite(f)
    assert np.array_equal(ve[fin], np.maximum(f[fin] - C, 0.0))
    # f(T) is the minimum: the difference is negative only by the rounding of C to binary32
    assert np.min(f[fin] - C) > -2.0 ** -25 * abs(C)
    # -inf -> f = -0 -> stored magnitude -C, sign 1; +inf stays +inf with sign 0
    assert yt[-1] == O.round_to(dtype, np.array([C]))[0] and yt[-2] == np.inf


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_decode_gives_back_the_activation(kind, dtype):
    x = inputs(dtype, seed=4)
    C = O.fT(kind, f32=True)
    _, yt = O.sbit_fwd(kind, dtype, x)
    ye, ys = O.sbit_decode(kind, dtype, yt)
    assert np.array_equal(ye, np.abs(yt) + C)
    assert np.array_equal(ys, O.round_to(dtype, ye))
    # |Y| + C differs from f(x) by the rounding of the stored difference: half an ulp of f - C
    f = O.f(kind, x)
    ulp_v = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(yt), 2.0 ** -126))) - P[dtype] + 1)
    assert np.all(np.abs(ye - f) <= 0.5 * ulp_v + 2.0 ** -25 * abs(C))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_backward_reads_the_sign_and_evaluates_q_at_the_rebuilt_value(kind, dtype):
    x = inputs(dtype, n=20000, seed=5)
    g = np.random.default_rng(6).standard_normal(x.size)
    C = O.fT(kind, f32=True)
    _, yt = O.sbit_fwd(kind, dtype, x)
    gx = O.sbit_bwd(kind, yt, g)
    s = np.signbit(yt).astype(np.uint8)
    assert np.array_equal(s, O.indicator(kind, x))
    y32 = (np.abs(yt) + C).astype(np.float32).astype(np.float64)      # Y + C in binary32 registers
    assert np.array_equal(gx, g * O.q(kind, y32, s))
    # same gradient as the ordinary variant up to what the two stored values differ by
    _, plain, m = O.invact_fwd(kind, dtype, x)
    ref = O.invact_bwd(kind, plain, m, g)
    assert np.max(np.abs(gx - ref)) <= (4e-2 if dtype == "bf16" else 1e-3) * np.max(np.abs(g))
    # and closer to the exact derivative than the ordinary variant in bfloat16: the stored f - C keeps its
    # relative precision next to the minimum, where f' goes like its square root
    if dtype == "bf16":
        exact = g * O.df(kind, x)
        assert np.sqrt(np.mean((gx - exact) ** 2)) < np.sqrt(np.mean((ref - exact) ** 2))


# ---------------------------------------------------------------- the consumer: (|Y| + C) W^T and dW = dOut^T (|Y| + C)

def linear_case(kind, dtype, M=37, N=19, K=24, seed=5):
    rng = np.random.default_rng(seed)
    x = synth.storage_to_f64(synth.to_storage((rng.standard_normal(M * K) * 2.0).astype(np.float32), dtype), dtype)
    _, yt = O.sbit_fwd(kind, dtype, x)
    w = synth.storage_to_f64(synth.to_storage(rng.standard_normal(N * K).astype(np.float32), dtype), dtype)
    g = synth.storage_to_f64(synth.to_storage(rng.standard_normal(M * N).astype(np.float32), dtype), dtype)
    b = synth.storage_to_f64(synth.to_storage(rng.standard_normal(N).astype(np.float32), dtype), dtype)
    return yt.reshape(M, K), w.reshape(N, K), g.reshape(M, N), b


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_linear_consumer_reduces_to_the_decode(kind, dtype):
    """With the identity as weight the product IS the decoded activation; a one-hot dOut picks one of its rows."""
    yt, _, _, _ = linear_case(kind, dtype, K=24)
    M, K = yt.shape
    dec = O.sbit_decode(kind, dtype, yt.reshape(-1))[1].reshape(M, K)
    assert np.array_equal(O.sbit_linear(kind, dtype, yt, np.eye(K)), dec)
    assert np.array_equal(O.sbit_linear(kind, dtype, -yt, np.eye(K)), dec)          # only |Y| enters
    for m, n in ((0, 0), (5, 3), (M - 1, 7)):
        g = np.zeros((M, 8)); g[m, n] = 1.0
        gw = O.sbit_linear_wgrad(kind, dtype, yt, g)
        assert np.array_equal(gw[n], dec[m]) and np.count_nonzero(gw) == np.count_nonzero(dec[m])


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_linear_consumer_against_a_library_product_and_its_own_adjoint(kind, dtype):
    yt, w, g, b = linear_case(kind, dtype)
    M, K = yt.shape
    dec = O.sbit_decode(kind, dtype, yt.reshape(-1))[1].reshape(M, K)
    out = O.sbit_linear(kind, dtype, yt, w, b)
    assert np.allclose(out, dec @ w.T + b, rtol=1e-13, atol=1e-13)                  # numpy's matmul on the decoded values
    assert np.allclose(out - O.sbit_linear(kind, dtype, yt, w), np.broadcast_to(b, out.shape), rtol=0, atol=1e-13)
    gw = O.sbit_linear_wgrad(kind, dtype, yt, g)
    assert np.allclose(gw, g.T @ dec, rtol=1e-13, atol=1e-13)
    # <dOut, (Y + C) W^T> = <dOut^T (Y + C), W>: a transposed operand or a wrong index on either side breaks this
    lhs = np.sum(g * O.sbit_linear(kind, dtype, yt, w))
    rhs = np.sum(gw * w)
    assert abs(lhs - rhs) <= 1e-11 * max(1.0, abs(lhs))
    # closed form: a constant saved tensor and a weight of ones give K (c + C) rounded as the decode rounds it
    c = float(O.round_to(dtype, np.array([0.75]))[0])
    one = O.sbit_decode(kind, dtype, np.array([c]))[1][0]
    assert np.allclose(O.sbit_linear(kind, dtype, np.full((3, K), -c), np.ones((2, K))), K * one, rtol=1e-14)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", KINDS)
def test_linear_consumer_input_gradient(kind, dtype):
    """dX = (dOut W) * q(|Y| + C, S): reduces to the activation's own backward, agrees with a library product,
    is the adjoint of the forward product once q is divided out, and is the derivative of the layer."""
    yt, w, g, _ = linear_case(kind, dtype)
    (M, K), N = yt.shape, w.shape[0]
    gx = O.sbit_linear_dgrad(kind, yt, g, w)
    # the identity as weight leaves the backward of the activation alone
    gy = (np.arange(M * K) % 7 - 3.0).reshape(M, K)
    assert np.array_equal(O.sbit_linear_dgrad(kind, yt, gy, np.eye(K)), O.sbit_bwd(kind, yt.reshape(-1), gy.reshape(-1)).reshape(M, K))
    # numpy's matmul for the product, the pinned element-wise backward for the rest (N != K: a transposed
    # operand does not even have the shape)
    assert np.allclose(gx, O.sbit_bwd(kind, yt.reshape(-1), (g @ w).reshape(-1)).reshape(M, K), rtol=1e-13, atol=1e-13)
    # adjoint of the forward product: <dX / q, Z> = <dOut, Z W^T> for any Z
    q = O.sbit_bwd(kind, yt.reshape(-1), np.ones(M * K)).reshape(M, K)
    z = np.random.default_rng(8).standard_normal((M, K))
    ok = np.abs(q) > 1e-3
    lhs = np.sum(np.where(ok, gx / np.where(ok, q, 1.0), (g @ w)) * z)
    rhs = np.sum(g * (z @ w.T))
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(rhs))
    # a one-hot dOut picks a row of the weight
    one = np.zeros((M, N)); one[3, 5] = 2.0
    picked = O.sbit_linear_dgrad(kind, yt, one, w)
    assert np.array_equal(picked[3], 2.0 * w[5] * q[3]) and np.count_nonzero(np.delete(picked, 3, 0)) == 0


@pytest.mark.parametrize("kind", KINDS)
def test_linear_consumer_input_gradient_is_the_derivative_of_the_layer(kind):
    """Central differences of L(x) = <R, f(x) W^T> with the exact f: dL/dx = f'(x) * (R W), which the oracle's
    dX reproduces up to the approximation error of q and the rounding of the saved tensor."""
    rng = np.random.default_rng(12)
    M, N, K = 9, 7, 11
    x = synth.storage_to_f64(synth.to_storage((rng.standard_normal(M * K) * 2.0).astype(np.float32), "fp32"), "fp32")
    w, r = rng.standard_normal((N, K)), rng.standard_normal((M, N))
    loss = lambda xs: np.sum(r * (O.f(kind, xs).reshape(M, K) @ w.T))
    h = 1e-6
    numeric = np.empty(M * K)
    for i in range(M * K):
        e = np.zeros(M * K); e[i] = h
        numeric[i] = (loss(x + e) - loss(x - e)) / (2 * h)
    _, yt = O.sbit_fwd(kind, "fp32", x)
    gx = O.sbit_linear_dgrad(kind, yt.reshape(M, K), r, w).reshape(-1)
    assert np.max(np.abs(gx - numeric)) <= 2e-2 * np.max(np.abs(r @ w))
    assert np.max(np.abs(gx - numeric)) > 0            # q is an approximation: an exact match would mean f' was used
