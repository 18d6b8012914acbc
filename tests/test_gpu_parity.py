"""GPU parity: libinvact (through its C ABI, via the ctypes binding) against the
CPU oracle, element by element, on the same seeded inputs.

Sizes here are ones the oracle finishes in seconds; they span many 8-element
chunks, several workgroups and ragged tails.  Full-size workloads are in
test_gpu_workloads.py.
"""
import numpy as np
import pytest
import torch

import oracle as O
import parity as PT
from paper_2407_15545_amd import binding as B
import synth

pytestmark = pytest.mark.gpu

KINDS = ["gelu_tanh", "gelu_erf", "silu"]
DTYPES = ["fp32", "bf16"]
SIZES = [1, 7, 8, 63, 64, 65, 511, 513, 4096 + 8, (1 << 20) + 3]


def draw(n, seed, dtype, std=2.0):
    return synth.to_storage(synth.normal(n, seed, std), dtype)


def mask_of(t):
    return t.cpu().numpy()


# ---------------------------------------------------------------- invact_fwd

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("kind", KINDS)
def test_fwd_matches_oracle(kind, dtype):
    for n in SIZES:
        PT.say(f"invact_fwd {kind} {dtype} n={n}")
        xs = draw(n, n, dtype)
        x64 = synth.storage_to_f64(xs, dtype)
        ye, _, m_ref = O.invact_fwd(kind, dtype, x64)
        y, m = B.invact_fwd(kind, PT.to_device(xs, dtype))
        torch.cuda.synchronize()
        assert m.numel() == O.mask_bytes(n)
        assert np.array_equal(mask_of(m), m_ref), f"mask differs, n={n}"
        err = PT.forward_errors(PT.to_f64(y), ye, dtype)
        assert err.max() <= 1.0, (n, PT.worst(err, x64, ye, PT.to_f64(y)))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("kind", KINDS)
def test_fwd_every_bf16_input(kind, dtype):
    """All 65 536 bfloat16 patterns as inputs (as binary32 values for the fp32 path)."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    xs = bits if dtype == "bf16" else synth.bf16_bits_to_f32(bits)
    with np.errstate(invalid="ignore"):
        x64 = synth.storage_to_f64(xs, dtype)
    ye, _, m_ref = O.invact_fwd(kind, dtype, x64)
    PT.say(f"invact_fwd {kind} {dtype} all bf16 patterns")
    y, m = B.invact_fwd(kind, PT.to_device(xs, dtype))
    torch.cuda.synchronize()
    assert np.array_equal(mask_of(m), m_ref)
    err = PT.forward_errors(PT.to_f64(y), ye, dtype)
    assert err.max() <= 1.0, PT.worst(err, x64, ye, PT.to_f64(y))
    # signed zero of the far left tail and of -inf
    got = PT.to_f64(y)
    ninf = int(np.where(bits == 0xFF80)[0][0])
    assert got[ninf] == 0 and np.signbit(got[ninf])
    assert got[int(np.where(bits == 0x7F80)[0][0])] == np.inf


@pytest.mark.parametrize("kind", KINDS)
def test_fwd_fp32_dense_ranges(kind):
    """binary32 forward on dense sweeps of every binade that matters, incl. the left tail."""
    rng = np.random.default_rng(11)
    parts = [rng.uniform(-110, 0, 1 << 18), rng.uniform(0, 110, 1 << 16), rng.uniform(-14, -4, 1 << 18),
             rng.uniform(-2, 2, 1 << 18), -np.exp2(rng.uniform(-140, 7, 1 << 16)), np.exp2(rng.uniform(-140, 127, 1 << 16))]
    xs = np.concatenate(parts).astype(np.float32)
    x64 = xs.astype(np.float64)
    ye, _, m_ref = O.invact_fwd(kind, "fp32", x64)
    PT.say(f"invact_fwd {kind} fp32 dense ranges n={xs.size}")
    y, m = B.invact_fwd(kind, PT.to_device(xs, "fp32"))
    torch.cuda.synchronize()
    assert np.array_equal(mask_of(m), m_ref)
    err = PT.forward_errors(PT.to_f64(y), ye, "fp32")
    assert err.max() <= 1.0, PT.worst(err, x64, ye, PT.to_f64(y))


# ---------------------------------------------------------------- invact_bwd

def bwd_case(kind, dtype, n, seed):
    xs = draw(n, seed, dtype)
    gs = draw(n, seed + 1, dtype, 1.0)
    x64 = synth.storage_to_f64(xs, dtype)
    g64 = synth.storage_to_f64(gs, dtype)
    _, ys64, m_ref = O.invact_fwd(kind, dtype, x64)
    return ys64, m_ref, gs, g64


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("kind", KINDS)
def test_bwd_matches_oracle(kind, dtype):
    for n in SIZES:
        PT.say(f"invact_bwd {kind} {dtype} n={n}")
        ys64, m_ref, gs, g64 = bwd_case(kind, dtype, n, 100 + n)
        ref = O.invact_bwd(kind, ys64, m_ref, g64)
        y_dev = PT.to_device(synth.f64_to_storage_exact(ys64, dtype), dtype)
        gx = B.invact_bwd(kind, y_dev, torch.from_numpy(m_ref).cuda(), PT.to_device(gs, dtype))
        torch.cuda.synchronize()
        err = PT.backward_errors(PT.to_f64(gx), ref, g64, dtype)
        assert err.max() <= 1.0, (n, PT.worst(err, ys64, g64, ref, PT.to_f64(gx)))


@pytest.mark.parametrize("kind", KINDS)
def test_bwd_every_bf16_y_and_both_mask_bits(kind):
    """All 131 072 (y, s) pairs with y a bfloat16 pattern, grad_y = 1.

    Pairs the forward can produce, and their neighbourhood (y within [-1, 1] on
    the left branch, any y on the right branch), must match the oracle.  For
    left-branch pairs far outside the range of f the binary32 evaluation
    overflows where the double one does not; there only NaN-ness and the
    absence of a fault are checked."""
    bits = np.tile(np.arange(65536, dtype=np.uint32).astype(np.uint16), 2)
    s = np.repeat(np.array([0, 1], np.uint8), 65536)
    with np.errstate(invalid="ignore"):
        y64 = synth.storage_to_f64(bits, "bf16")
    m = O.pack(s)
    g = np.ones(bits.size)
    ref = O.invact_bwd(kind, y64, m, g)
    PT.say(f"invact_bwd {kind} bf16 all (y, s) pairs")
    gx = B.invact_bwd(kind, PT.to_device(bits, "bf16"), torch.from_numpy(m).cuda(),
                      PT.to_device(synth.to_storage(g.astype(np.float32), "bf16"), "bf16"))
    torch.cuda.synchronize()
    got = PT.to_f64(gx)
    with np.errstate(invalid="ignore"):
        strict = (s == 0) | (np.abs(y64) <= 1.0) | np.isnan(y64)
    err = PT.backward_errors(got[strict], ref[strict], g[strict], "bf16")
    assert err.max() <= 1.0, PT.worst(err, y64[strict], s[strict].astype(float), ref[strict], got[strict])
    assert np.all(np.isnan(got[np.isnan(y64)]))


@pytest.mark.parametrize("kind", KINDS)
def test_bwd_fp32_dense_in_y(kind):
    """binary32 backward on y dense over the range of f on both branches (valid pairs only)."""
    rng = np.random.default_rng(17)
    fT = O.fT(kind, f32=True)
    yl = np.concatenate([rng.uniform(fT, 0, 1 << 18), fT + np.exp2(rng.uniform(-30, -3, 1 << 16)),
                         -np.exp2(rng.uniform(-60, -3, 1 << 16))])
    yr = np.concatenate([rng.uniform(fT, 1, 1 << 18), rng.uniform(1, 40, 1 << 17),
                         fT + np.exp2(rng.uniform(-30, -3, 1 << 16)), np.exp2(rng.uniform(-40, 100, 1 << 14)),
                         [fT, fT - 1e-4, np.inf, 64.0, 65.0, 1e30]])
    y = np.concatenate([yl, yr]).astype(np.float32)
    y = np.maximum(y, np.float32(fT) - np.float32(2e-4))
    s = np.concatenate([np.ones(yl.size, np.uint8), np.zeros(yr.size, np.uint8)])
    g = rng.standard_normal(y.size).astype(np.float32)
    m = O.pack(s)
    ref = O.invact_bwd(kind, y.astype(np.float64), m, g.astype(np.float64))
    PT.say(f"invact_bwd {kind} fp32 dense y n={y.size}")
    gx = B.invact_bwd(kind, PT.to_device(y, "fp32"), torch.from_numpy(m).cuda(), PT.to_device(g, "fp32"))
    torch.cuda.synchronize()
    got = PT.to_f64(gx)
    err = PT.backward_errors(got, ref, g.astype(np.float64), "fp32")
    assert err.max() <= 1.0, PT.worst(err, y.astype(np.float64), s.astype(float), ref, got)
    # reported: the plain result-relative figure the tolerance rule replaces
    lit = PT.literal_ulps(got, ref, "fp32")
    fin = np.isfinite(lit)
    absq = np.abs(got - ref)[fin] / np.abs(g)[fin]
    small = np.abs(ref[fin] / g[fin]) < 0.5
    PT.say(f"  {kind}: max |gpu-ref|/|g| = {absq.max():.3g} (where |q| < 0.5: {absq[small].max():.3g}), "
        f"literal max ulp = {lit[fin].max():.3g}, share over 2 ulp = {(lit[fin] > 2).mean():.3g}")


# ---------------------------------------------------------------- gated block

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("kind", KINDS)
def test_gated_fwd_bwd_match_oracle(kind, dtype):
    for n in SIZES:
        PT.say(f"geglu fwd/bwd {kind} {dtype} n={n}")
        gate_s, up_s, gh_s = draw(n, 200 + n, dtype, 1.5), draw(n, 201 + n, dtype, 1.0), draw(n, 202 + n, dtype, 0.01)
        gate, up, gh = (synth.storage_to_f64(a, dtype) for a in (gate_s, up_s, gh_s))
        ae, as_, he, m_ref = O.glu_fwd(kind, dtype, gate, up)
        act, h, m = B.geglu_invact_fwd(kind, PT.to_device(gate_s, dtype), PT.to_device(up_s, dtype))
        torch.cuda.synchronize()
        assert np.array_equal(mask_of(m), m_ref)
        e1 = PT.forward_errors(PT.to_f64(act), ae, dtype)
        e2 = PT.forward_errors(PT.to_f64(h), he, dtype)
        assert e1.max() <= 1.0, (n, PT.worst(e1, gate, ae, PT.to_f64(act)))
        assert e2.max() <= 1.0, (n, PT.worst(e2, gate, up, he, PT.to_f64(h)))
        # backward from what the ORACLE's forward saved
        gg_ref, gu_ref = O.glu_bwd(kind, as_, up, m_ref, gh)
        act_dev = PT.to_device(synth.f64_to_storage_exact(as_, dtype), dtype)
        gg, gu = B.geglu_invact_bwd(kind, act_dev, PT.to_device(up_s, dtype), torch.from_numpy(m_ref).cuda(),
                                    PT.to_device(gh_s, dtype))
        torch.cuda.synchronize()
        e3 = PT.forward_errors(PT.to_f64(gu), gu_ref, dtype)          # plain product: 2 ulp literally
        e4 = PT.backward_errors(PT.to_f64(gg), gg_ref, gh * up, dtype)
        assert e3.max() <= 1.0, (n, PT.worst(e3, gh, as_, gu_ref, PT.to_f64(gu)))
        assert e4.max() <= 1.0, (n, PT.worst(e4, as_, gh * up, gg_ref, PT.to_f64(gg)))


@pytest.mark.parametrize("kind", KINDS)
def test_gated_fwd_every_bf16_gate_with_ordinary_and_extreme_up(kind):
    """Every bfloat16 pattern as the gate against sixteen values of `up`, from tiny to 10^38, infinite and NaN.
    With bfloat16 storage the product is formed from the activation as binary32 holds it, and where |f(gate)| is
    below 2^-126 that value may be flushed or gradually underflowed (an absolute error of up to 2^-126, allowed for
    the stored activation too); h inherits it times |up|.  So: 2 ulp of h, or 2^-126 |up| where |f(gate)| < 2^-126;
    there, an infinite `up` may give NaN (flushed to zero first) or the signed infinity."""
    ups = synth.to_storage(np.array([1.5, -0.75, 3.0e30, -2.0e-30, 0.0, 1.0, np.inf, 7.0e-40, -1.0e38, np.nan, 0.3333,
                                     -4096.0, 2.0 ** -126, 1e7, 1e15, -1e22], dtype=np.float32), "bf16")
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    gate_s, up_s = np.repeat(bits, ups.size), np.tile(ups, bits.size)
    with np.errstate(invalid="ignore"):
        gate, up = synth.storage_to_f64(gate_s, "bf16"), synth.storage_to_f64(up_s, "bf16")
    ae, _, he, m_ref = O.glu_fwd(kind, "bf16", gate, up)
    PT.say(f"geglu fwd {kind} bf16: all gate patterns x {ups.size} values of up")
    act, h, m = B.geglu_invact_fwd(kind, PT.to_device(gate_s, "bf16"), PT.to_device(up_s, "bf16"))
    torch.cuda.synchronize()
    assert np.array_equal(mask_of(m), m_ref)
    e1 = PT.forward_errors(PT.to_f64(act), ae, "bf16")
    assert e1.max() <= 1.0, PT.worst(e1, gate, ae, PT.to_f64(act))
    got = PT.to_f64(h)
    with np.errstate(invalid="ignore"):
        tiny = np.abs(ae) < 2.0 ** -126
        e2 = PT.forward_errors(got, he, "bf16")
        inherited = tiny & np.isfinite(up) & (np.abs(got - he) <= 2.0 ** -126 * np.abs(up))
        at_infinity = tiny & np.isinf(up) & (np.isnan(got) | (got == np.sign(gate) * up))
    e2[inherited | at_infinity] = 0.0
    assert e2.max() <= 1.0, PT.worst(e2, gate, up, he, got)
    assert (inherited & (PT.forward_errors(got, he, "bf16") > 1.0)).sum() < 2000          # a narrow band, not a loophole


@pytest.mark.parametrize("kind", KINDS)
def test_gated_bwd_every_bf16_activation_both_mask_bits_and_extreme_factors(kind):
    """All (act, s) pairs with act a bfloat16 pattern, against eight (grad_h, up) pairs from ordinary to infinite
    and NaN, including one whose product overflows.  grad_up = grad_h * act to 2 ulp; grad_gate = grad_h * up * q
    with the backward's tolerance (left-branch activations far outside f's range as in the plain backward's test).
    grad_h * up is formed first: where it overflows the result is the infinity even if q would make it finite."""
    pairs = synth.to_storage(np.array([[1.0, 1.0], [-0.75, 1.5], [1e-20, 1e20], [3e19, 3e19], [np.inf, -2.0],
                                       [1.0, np.nan], [0.0, 5.0], [1e-30, 1e-30]], dtype=np.float32).reshape(-1), "bf16").reshape(-1, 2)
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    act_s = np.tile(np.repeat(bits, len(pairs)), 2)
    gh_s, up_s = np.tile(np.tile(pairs[:, 0], bits.size), 2), np.tile(np.tile(pairs[:, 1], bits.size), 2)
    s = np.repeat(np.array([0, 1], np.uint8), bits.size * len(pairs))
    with np.errstate(invalid="ignore"):
        a64, g64, u64 = (synth.storage_to_f64(v, "bf16") for v in (act_s, gh_s, up_s))
    m = O.pack(s)
    gg_ref, gu_ref = O.glu_bwd(kind, a64, u64, m, g64)
    PT.say(f"geglu_invact_bwd {kind} bf16: all (act, s) pairs x {len(pairs)} (grad_h, up) pairs")
    gg, gu = B.geglu_invact_bwd(kind, PT.to_device(act_s, "bf16"), PT.to_device(up_s, "bf16"), torch.from_numpy(m).cuda(),
                                PT.to_device(gh_s, "bf16"))
    torch.cuda.synchronize()
    gg_got, gu_got = PT.to_f64(gg), PT.to_f64(gu)
    e_up = PT.forward_errors(gu_got, gu_ref, "bf16")
    assert e_up.max() <= 1.0, PT.worst(e_up, g64, a64, gu_ref, gu_got)
    with np.errstate(invalid="ignore", over="ignore"):
        # activations f cannot produce: far left-branch ones as in the plain test; below -1 on either branch q is
        # astronomically large, and times a product that underflowed in binary32 the comparison means nothing
        strict = ((s == 0) & (a64 >= -1.0)) | (np.abs(a64) <= 1.0) | np.isnan(a64)
        product = (g64 * u64).astype(np.float32).astype(np.float64)           # as binary32 forms it
        e_gate = PT.backward_errors(gg_got, gg_ref, g64 * u64, "bf16")
        overflowed = np.isinf(product) & np.isfinite(g64) & np.isfinite(u64)
        e_gate[overflowed & np.where(np.isnan(gg_ref) | (gg_ref == 0), np.isnan(gg_got),          # inf * 0 where q is 0
                                     gg_got == np.sign(gg_ref) * np.inf)] = 0.0
    assert e_gate[strict].max() <= 1.0, PT.worst(e_gate[strict], a64[strict], g64[strict], u64[strict], gg_ref[strict], gg_got[strict])


def test_swiglu_entry_points_equal_geglu_with_silu():
    n = 70001
    gate_s, up_s, gh_s = draw(n, 5, "bf16"), draw(n, 6, "bf16", 1.0), draw(n, 7, "bf16", 0.01)
    gate, up, gh = (PT.to_device(a, "bf16") for a in (gate_s, up_s, gh_s))
    PT.say("swiglu_invact_fwd/bwd vs geglu(silu)")
    a1, h1, m1 = B.swiglu_invact_fwd(gate, up)
    a2, h2, m2 = B.geglu_invact_fwd("silu", gate, up)
    g1 = B.swiglu_invact_bwd(a1, up, m1, gh)
    g2 = B.geglu_invact_bwd("silu", a2, up, m2, gh)
    torch.cuda.synchronize()
    for p, q in ((a1, a2), (h1, h2), (m1, m2), (g1[0], g2[0]), (g1[1], g2[1])):
        assert torch.equal(p.view(torch.uint8) if p.dtype != torch.uint8 else p,
                           q.view(torch.uint8) if q.dtype != torch.uint8 else q)


# ---------------------------------------------------------------- contract details

@pytest.mark.parametrize("dtype", DTYPES)
def test_in_place_and_canaries(dtype):
    """Element-wise aliasing is allowed, and nothing is written past the outputs."""
    kind, n = "silu", 100003
    pad = 64
    xs = draw(n, 31, dtype)
    gs = draw(n, 32, dtype, 1.0)
    x = PT.to_device(xs, dtype)
    td = PT.TORCH_DTYPE[dtype]
    PT.say(f"in-place / canaries {dtype}")
    # reference results out of place
    y_ref, m_ref = B.invact_fwd(kind, x)
    gx_ref = B.invact_bwd(kind, y_ref, m_ref, PT.to_device(gs, dtype))
    # outputs carved out of larger buffers whose surroundings hold a canary
    nb = B.mask_bytes(n)
    ybuf = torch.full((n + 2 * pad,), 7.0, dtype=td, device="cuda")
    mbuf = torch.full((nb + 2 * pad,), 0xAB, dtype=torch.uint8, device="cuda")
    yv, mv = ybuf[pad:pad + n], mbuf[pad:pad + nb]
    yv.copy_(x)
    B.invact_fwd(kind, yv, y=yv, mask=mv)                         # y == x
    torch.cuda.synchronize()
    assert torch.equal(yv.view(torch.uint8), y_ref.view(torch.uint8)) and torch.equal(mv, m_ref)
    assert bool((ybuf[:pad] == 7.0).all()) and bool((ybuf[pad + n:] == 7.0).all())
    assert bool((mbuf[:pad] == 0xAB).all()) and bool((mbuf[pad + nb:] == 0xAB).all())
    gbuf = torch.full((n + 2 * pad,), 7.0, dtype=td, device="cuda")
    gv = gbuf[pad:pad + n]
    gv.copy_(PT.to_device(gs, dtype))
    B.invact_bwd(kind, y_ref, m_ref, gv, grad_x=gv)               # grad_x == grad_y
    torch.cuda.synchronize()
    assert torch.equal(gv.view(torch.uint8), gx_ref.view(torch.uint8))
    assert bool((gbuf[:pad] == 7.0).all()) and bool((gbuf[pad + n:] == 7.0).all())
    # gated: grad_up == grad_h
    up = PT.to_device(draw(n, 33, dtype, 1.0), dtype)
    gg_ref, gu_ref = B.geglu_invact_bwd(kind, y_ref, up, m_ref, PT.to_device(gs, dtype))
    gv.copy_(PT.to_device(gs, dtype))
    gg, gu = B.geglu_invact_bwd(kind, y_ref, up, m_ref, gv, grad_up=gv)
    torch.cuda.synchronize()
    assert torch.equal(gg.view(torch.uint8), gg_ref.view(torch.uint8))
    assert torch.equal(gu.view(torch.uint8), gu_ref.view(torch.uint8))


def test_mask_padding_is_rewritten_as_zero():
    for n in (1, 9, 65, 127, 129, 1000):
        m = torch.full((B.mask_bytes(n),), 0xFF, dtype=torch.uint8, device="cuda")
        x = torch.full((n,), -5.0, dtype=torch.bfloat16, device="cuda")      # every bit set
        PT.say(f"mask padding n={n}")
        B.invact_fwd("silu", x, mask=m)
        torch.cuda.synchronize()
        assert np.array_equal(m.cpu().numpy(), O.pack(np.ones(n, np.uint8)))


def same_bits(a, b):
    return torch.equal(a.view(torch.uint8), b.view(torch.uint8))


@pytest.mark.parametrize("dtype", DTYPES)
def test_other_stream_and_grid_shapes_give_identical_bits(dtype):
    """Every entry point on a side stream, with other caps on resident workgroups and as a persistent grid of
    several sizes: same bits as the default."""
    n = (1 << 22) + 13 * 512 + 77
    kind = "gelu_erf"
    x, up, g = (PT.to_device(draw(n, 41 + i, dtype), dtype) for i in range(3))

    def run_all():
        y, m = B.invact_fwd(kind, x)
        gx = B.invact_bwd(kind, y, m, g)
        act, h, m2 = B.geglu_invact_fwd(kind, x, up)
        gg, gu = B.geglu_invact_bwd(kind, act, up, m2, g)
        yp = B.invact_pbit_fwd(kind, x)
        gp = B.invact_pbit_bwd(kind, yp, g)
        yt = B.invact_sbit_fwd(kind, x)
        yd = B.invact_sbit_decode(kind, yt)
        gs = B.invact_sbit_bwd(kind, yt, g)
        torch.cuda.synchronize()
        return [y, m, gx, act, h, m2, gg, gu, yp, gp, yt, yd, gs]

    PT.say(f"streams / grid shapes {dtype}")
    ref = run_all()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        got = run_all()
    assert all(same_bits(a, b) for a, b in zip(ref, got))
    try:
        for cap in (1, 5, 16, 32):
            PT.say(f"  at most {cap} resident workgroups per compute unit")
            assert B.set_resident_blocks(cap) == cap
            got = run_all()
            assert all(same_bits(a, b) for a, b in zip(ref, got)), cap
        assert B.set_resident_blocks(33) < 0 and B.set_resident_blocks(-1) < 0
    finally:
        B.set_resident_blocks(0)
    try:
        for bpc in (1, 3, 16, 64):
            PT.say(f"  persistent grid, {bpc} workgroups per compute unit")
            assert B.set_blocks_per_cu(bpc) == bpc
            got = run_all()
            assert all(same_bits(a, b) for a, b in zip(ref, got)), bpc
    finally:
        B.set_blocks_per_cu(0)


def test_nan_and_infinities_flow_through():
    special = [float("nan"), float("inf"), float("-inf"), 0.0, -0.0, 1.0, -1.0, -3.0] * 3
    for dtype in DTYPES:
        td = PT.TORCH_DTYPE[dtype]
        x = torch.tensor(special, dtype=td, device="cuda")
        x64 = np.array(special, dtype=np.float64)
        g = torch.ones_like(x)
        for kind in KINDS:
            PT.say(f"specials {kind} {dtype}")
            ye, ys, mr = O.invact_fwd(kind, dtype, x64)
            y, m = B.invact_fwd(kind, x)
            # backward from what the oracle's forward saved
            y_saved = PT.to_device(synth.f64_to_storage_exact(ys, dtype), dtype)
            gx = B.invact_bwd(kind, y_saved, torch.from_numpy(mr).cuda(), g)
            torch.cuda.synchronize()
            yv, gv = PT.to_f64(y), PT.to_f64(gx)
            assert np.array_equal(m.cpu().numpy(), mr)
            assert PT.forward_errors(yv, ye, dtype).max() <= 1.0
            assert np.isnan(yv[0]) and yv[1] == np.inf and yv[2] == 0 and np.signbit(yv[2])
            assert np.isnan(gv[0]) and gv[1] == 1.0
            ref = O.invact_bwd(kind, ys, mr, np.ones(x.numel()))
            assert PT.backward_errors(gv, ref, np.ones(x.numel()), dtype).max() <= 1.0


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("kind", KINDS)
def test_infinite_and_nan_gradients_through_every_backward(kind, dtype):
    """An infinite incoming gradient times q is the signed infinity (the oracle's inf * q), a NaN one a NaN, in all
    four backward entry points, on saved values from both branches and both sides of q's way of being summed."""
    xs = synth.to_storage(np.array([-6.0, -2.0, -0.9, -0.7, -0.2, 0.0, 0.3, 1.0, 2.5, 7.0, 30.0], dtype=np.float32), dtype)
    grads = np.array([np.inf, -np.inf, np.nan], dtype=np.float32)
    x_s, g_s = np.repeat(xs, grads.size), synth.to_storage(np.tile(grads, xs.size), dtype)
    x64, g64 = synth.storage_to_f64(x_s, dtype), synth.storage_to_f64(g_s, dtype)
    n = x64.size
    dev = lambda v: PT.to_device(synth.f64_to_storage_exact(v, dtype), dtype)
    g = PT.to_device(g_s, dtype)
    PT.say(f"infinite gradients {kind} {dtype}")

    def same(got, ref):
        got = PT.to_f64(got)
        return np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(got[~np.isnan(ref)], ref[~np.isnan(ref)])

    _, ys, m = O.invact_fwd(kind, dtype, x64)
    assert same(B.invact_bwd(kind, dev(ys), torch.from_numpy(m).cuda(), g), O.invact_bwd(kind, ys, m, g64))
    _, yp = O.pbit_fwd(kind, dtype, x64)
    assert same(B.invact_pbit_bwd(kind, dev(yp), g), O.pbit_bwd(kind, dtype, yp, g64))
    _, yt = O.sbit_fwd(kind, dtype, x64)
    assert same(B.invact_sbit_bwd(kind, dev(yt), g), O.sbit_bwd(kind, yt, g64))
    up = np.full(n, -1.5)
    gg_ref, gu_ref = O.glu_bwd(kind, ys, up, m, g64)
    gg, gu = B.geglu_invact_bwd(kind, dev(ys), dev(up), torch.from_numpy(m).cuda(), g)
    torch.cuda.synchronize()
    assert same(gg, gg_ref) and same(gu, gu_ref)
