"""Binary32 kernels against the oracle over the whole input space.

Every STRIDE-th binary32 bit pattern goes through
  * invact_fwd, invact_pbit_fwd, invact_sbit_fwd, invact_sbit_decode (all patterns) and geglu_invact_fwd (all
    patterns as the gate, `up` cycling through ordinary and extreme values);
  * invact_bwd, invact_pbit_bwd, invact_sbit_bwd with grad_y = 1 and geglu_invact_bwd with ordinary and extreme
    (grad_h, up) pairs, over every stored y the backward can meet: y >= f(T) - 2^-12 with s = 0, and y in
    [f(T) - 2^-12, +0] with s = 1;
with the tolerances of tests/parity.py; masks, tag bits and sign bits must be exact.  STRIDE is 61 by default
(7 * 10^7 patterns per case, a few seconds); with INVACT_EXHAUSTIVE=1 in the environment it is 1, i.e. all 2^32
patterns (2-4 minutes per case):

    INVACT_EXHAUSTIVE=1 python -m pytest tests/test_gpu_exhaustive.py -m gpu -s

Each case prints one RESULT line (worst error in units of the tolerance, worst literal error in ulps, where).
"""
import os
import time

import numpy as np
import pytest
import torch

import oracle as O
import parity as PT
from paper_2407_15545_amd import binding as B

pytestmark = pytest.mark.gpu
KINDS = ["gelu_tanh", "gelu_erf", "silu"]
STRIDE = 1 if os.environ.get("INVACT_EXHAUSTIVE") == "1" else 61
BLOCK = 1 << 26          # patterns per launch


def pattern_blocks(first, last):
    """Strided pattern ranges covering first..last inclusive, as (start, count) with stride STRIDE."""
    a = first
    while a <= last:
        count = min(BLOCK, (last - a) // STRIDE + 1)
        yield a, count
        a += count * STRIDE


def patterns_to_device(start, count):
    bits = start + STRIDE * torch.arange(count, dtype=torch.int64, device="cuda")
    return bits.to(torch.int32).view(torch.float32)       # the conversion wraps patterns >= 2^31 as intended


class Worst:
    def __init__(self):
        self.tol, self.ulp, self.where_tol, self.where_ulp, self.total = 0.0, 0.0, None, None, 0

    def update(self, start, got, ref, err):
        i = int(np.nanargmax(err))
        if err[i] > self.tol:
            self.tol, self.where_tol = float(err[i]), (hex(start + STRIDE * i), float(got[i]), float(ref[i]))
        with np.errstate(invalid="ignore", over="ignore"):
            lit = np.where(np.isfinite(ref) & np.isfinite(got) & (np.abs(ref) >= 2.0 ** -126),
                           np.abs(got - ref) / PT.ulp(ref, "fp32"), 0.0)
        j = int(np.argmax(lit))
        if lit[j] > self.ulp:
            self.ulp, self.where_ulp = float(lit[j]), (hex(start + STRIDE * j), float(got[j]), float(ref[j]))
        self.total += err.size


@pytest.mark.parametrize("kind", KINDS)
def test_forward_over_all_binary32_inputs(kind):
    w, mask_ok, t0 = Worst(), True, time.time()
    for start, count in pattern_blocks(0x00000000, 0xFFFFFFFF):
        PT.say(f"exhaustive fwd {kind}: patterns from {start:#010x}, {count} of them, stride {STRIDE}")
        x = patterns_to_device(start, count)
        y, m = B.invact_fwd(kind, x)
        torch.cuda.synchronize()
        x64 = x.cpu().numpy().astype(np.float64)
        ye, _, m_ref = O.invact_fwd(kind, "fp32", x64)
        mask_ok &= bool(np.array_equal(m.cpu().numpy(), m_ref))
        got = y.cpu().numpy().astype(np.float64)
        w.update(start, got, ye, PT.forward_errors(got, ye, "fp32"))
    print(f"\nRESULT fwd {kind} stride {STRIDE}: {w.total} inputs, worst {w.tol:.4f} of the tolerance at {w.where_tol}, "
          f"worst literal {w.ulp:.4g} ulp at {w.where_ulp}, masks {'bit-exact' if mask_ok else 'DIFFER'} "
          f"[{time.time() - t0:.0f} s]", flush=True)
    assert mask_ok
    assert w.tol <= 1.0, w.where_tol


@pytest.mark.parametrize("kind", KINDS)
def test_backward_over_all_binary32_saved_outputs(kind):
    fT = np.float32(O.fT(kind, f32=True))
    lo = np.float32(fT - np.float32(2.0 ** -12))
    lo_bits = int(np.array([lo]).view(np.uint32)[0])          # negative: larger pattern = more negative
    ranges = [(0x00000000, 0x7F800000, 0),                     # s = 0: +0 .. +inf
              (0x80000000, lo_bits, 0),                        # s = 0: -0 .. f(T) - 2^-12
              (0x80000000, lo_bits, 1),                        # s = 1: -0 .. f(T) - 2^-12
              (0x00000000, 0x00000000, 1)]                     # s = 1: +0
    w, t0 = Worst(), time.time()
    for first, last, s in ranges:
        for start, count in pattern_blocks(first, last):
            PT.say(f"exhaustive bwd {kind} s={s}: patterns from {start:#010x}, {count} of them, stride {STRIDE}")
            y = patterns_to_device(start, count)
            mask = torch.full((B.mask_bytes(count),), 0xFF if s else 0, dtype=torch.uint8, device="cuda")
            gx = B.invact_bwd(kind, y, mask, torch.ones(count, dtype=torch.float32, device="cuda"))
            torch.cuda.synchronize()
            y64 = y.cpu().numpy().astype(np.float64)
            ref = O.q(kind, y64, np.full(count, s, np.uint8))
            got = gx.cpu().numpy().astype(np.float64)
            w.update(start, got, ref, PT.backward_errors(got, ref, np.ones(count), "fp32"))
    print(f"\nRESULT bwd {kind} stride {STRIDE}: {w.total} cases, worst {w.tol:.4f} of the tolerance at {w.where_tol}, "
          f"worst literal {w.ulp:.4g} ulp at {w.where_ulp} [{time.time() - t0:.0f} s]", flush=True)
    assert w.tol <= 1.0, w.where_tol


@pytest.mark.parametrize("kind", KINDS)
def test_precision_bit_forward_over_all_binary32_inputs(kind):
    """invact_pbit_fwd: bit 0 of the stored pattern is the indicator for every input (0 for a NaN), the value
    within 2 ulp of the oracle's rounded-then-tagged one and within 3 ulp of f(x) itself."""
    w, bits_ok, t0 = Worst(), True, time.time()
    for start, count in pattern_blocks(0x00000000, 0xFFFFFFFF):
        PT.say(f"exhaustive pbit fwd {kind}: patterns from {start:#010x}, {count} of them, stride {STRIDE}")
        x = patterns_to_device(start, count)
        y = B.invact_pbit_fwd(kind, x)
        torch.cuda.synchronize()
        x64 = x.cpu().numpy().astype(np.float64)
        ye, ys = O.pbit_fwd(kind, "fp32", x64)
        tag = y.view(torch.int32).cpu().numpy().view(np.uint32) & 1
        bits_ok &= bool(np.array_equal(tag, O.indicator(kind, x64).astype(np.uint32)))
        got = y.cpu().numpy().astype(np.float64)
        w.update(start, got, ys, PT.forward_errors(got, ys, "fp32"))
        assert (PT.forward_errors(got, ye, "fp32") * 2).max() <= 3.0
    print(f"\nRESULT pbit fwd {kind} stride {STRIDE}: {w.total} inputs, worst {w.tol:.4f} of the tolerance at {w.where_tol}, "
          f"worst literal {w.ulp:.4g} ulp at {w.where_ulp}, tag bits {'exact' if bits_ok else 'DIFFER'} "
          f"[{time.time() - t0:.0f} s]", flush=True)
    assert bits_ok
    assert w.tol <= 1.0, w.where_tol


@pytest.mark.parametrize("kind", KINDS)
def test_sign_bit_forward_over_all_binary32_inputs(kind):
    """invact_sbit_fwd: the sign bit of the stored pattern is the indicator for every input, NaNs included (their
    indicator is 0); the magnitude against the exact f(x) - C with the tolerance of tests/test_gpu_sbit.py."""
    from test_gpu_sbit import magnitude_errors, sign_bits
    C = O.fT(kind, f32=True)
    worst, where, signs_ok, total, t0 = 0.0, None, True, 0, time.time()
    for start, count in pattern_blocks(0x00000000, 0xFFFFFFFF):
        PT.say(f"exhaustive sbit fwd {kind}: patterns from {start:#010x}, {count} of them, stride {STRIDE}")
        x = patterns_to_device(start, count)
        yt = B.invact_sbit_fwd(kind, x)
        torch.cuda.synchronize()
        x64 = x.cpu().numpy().astype(np.float64)
        ve, _ = O.sbit_fwd(kind, "fp32", x64)
        signs_ok &= bool(np.array_equal(sign_bits(yt), O.indicator(kind, x64)))
        got = yt.cpu().numpy().astype(np.float64)
        err = magnitude_errors(got, ve, O.f(kind, x64), C, "fp32")
        i = int(np.argmax(err))
        if err[i] > worst:
            worst, where = float(err[i]), (hex(start + STRIDE * i), float(got[i]), float(ve[i]))
        total += count
    print(f"\nRESULT sbit fwd {kind} stride {STRIDE}: {total} inputs, worst {worst:.4f} of the tolerance at {where}, "
          f"sign bits {'exact' if signs_ok else 'DIFFER'} [{time.time() - t0:.0f} s]", flush=True)
    assert signs_ok
    assert worst <= 1.0, where


@pytest.mark.parametrize("kind", KINDS)
def test_gated_forward_over_all_binary32_gates(kind):
    """geglu_invact_fwd with every binary32 pattern as the gate; `up` cycles through ordinary, huge, tiny, zero,
    infinite and NaN values, so that h = f(gate) * up also overflows and underflows.  The stored activation and h
    against the oracle (2 ulp; h is formed from the unrounded activation), the mask bit for bit."""
    ups = torch.tensor([1.5, -0.75, 3.0e30, -2.0e-30, 0.0, 1.0, float("inf"), 7.0e-42, -1.0e38, float("nan"),
                        0.333333343267, -4096.0, 2.0 ** -126], dtype=torch.float32, device="cuda")     # 13: prime to 61 and 64
    wa, wh, mask_ok, t0 = Worst(), Worst(), True, time.time()
    for start, count in pattern_blocks(0x00000000, 0xFFFFFFFF):
        PT.say(f"exhaustive gated fwd {kind}: patterns from {start:#010x}, {count} of them, stride {STRIDE}")
        gate = patterns_to_device(start, count)
        up = ups[torch.arange(count, device="cuda") % ups.numel()]
        act, h, m = B.geglu_invact_fwd(kind, gate, up)
        torch.cuda.synchronize()
        g64, u64 = gate.cpu().numpy().astype(np.float64), up.cpu().numpy().astype(np.float64)
        ae, _, he, m_ref = O.glu_fwd(kind, "fp32", g64, u64)
        mask_ok &= bool(np.array_equal(m.cpu().numpy(), m_ref))
        a_got, h_got = act.cpu().numpy().astype(np.float64), h.cpu().numpy().astype(np.float64)
        wa.update(start, a_got, ae, PT.forward_errors(a_got, ae, "fp32"))
        # f(gate) is never 0 for a finite gate, but far out it underflows, in the oracle's binary64 at another gate
        # than in the kernel's arithmetic; times an infinite `up` that is the difference between NaN and an
        # infinity.  There either answer passes.
        either = np.isinf(u64) & (np.abs(ae) < 1e-290) & ~np.isnan(g64)
        with np.errstate(invalid="ignore"):
            assert np.all(np.isnan(h_got[either]) | (h_got[either] == np.sign(g64[either]) * u64[either]))    # f has its gate's sign
        err_h = PT.forward_errors(h_got, he, "fp32")
        err_h[either] = 0.0
        wh.update(start, np.where(either, he, h_got), he, err_h)
    print(f"\nRESULT gated fwd {kind} stride {STRIDE}: {wa.total} inputs, activation worst {wa.tol:.4f} of the tolerance at "
          f"{wa.where_tol}, h worst {wh.tol:.4f} at {wh.where_tol} (literal {wh.ulp:.4g} ulp at {wh.where_ulp}), masks "
          f"{'bit-exact' if mask_ok else 'DIFFER'} [{time.time() - t0:.0f} s]", flush=True)
    assert mask_ok
    assert wa.tol <= 1.0, wa.where_tol
    assert wh.tol <= 1.0, wh.where_tol


@pytest.mark.parametrize("kind", KINDS)
def test_sign_bit_decode_over_all_binary32_patterns(kind):
    """invact_sbit_decode: |y_tagged| + C is one correctly rounded binary32 addition, so every pattern must come back
    bit for bit as the oracle's rounded sum (NaN for NaN)."""
    same, total, t0 = True, 0, time.time()
    for start, count in pattern_blocks(0x00000000, 0xFFFFFFFF):
        PT.say(f"exhaustive sbit decode {kind}: patterns from {start:#010x}, {count} of them, stride {STRIDE}")
        yt = patterns_to_device(start, count)
        y = B.invact_sbit_decode(kind, yt)
        torch.cuda.synchronize()
        _, ys = O.sbit_decode(kind, "fp32", yt.cpu().numpy().astype(np.float64))
        got = y.cpu().numpy()
        want = ys.astype(np.float32)
        nan = np.isnan(want)
        same &= bool(np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32)))
        total += count
    print(f"\nRESULT sbit decode {kind} stride {STRIDE}: {total} patterns, {'bit-exact' if same else 'DIFFER'} "
          f"[{time.time() - t0:.0f} s]", flush=True)
    assert same


@pytest.mark.parametrize("kind", KINDS)
def test_gated_backward_over_all_binary32_saved_activations(kind):
    """geglu_invact_bwd with every stored activation the backward can meet (as in the plain backward's test) and
    (grad_h, up) cycling through ordinary, tiny, huge, zero, infinite and NaN pairs, some with a product beyond
    binary32 (the result is then the infinity the oracle's double arithmetic rounds to, unless q makes it finite
    again, which the kernel cannot see: those few cases are left out): grad_up = grad_h * act to 2 ulp, grad_gate = grad_h * up * q with the backward's tolerance at the
    scale of grad_h * up."""
    pairs = torch.tensor([[1.0, 1.0], [-0.75, 1.5], [1e-20, 1e20], [1e19, -1e-19], [3e-20, 3e-20], [1e-30, 1e-30],
                          [float("inf"), 1.0], [1.0, float("nan")], [0.0, 5.0], [-2.5e-3, 0.0], [7.0e-42, 1e3],
                          [1e15, 1e15], [-3.0, 2.0 ** -126], [3e19, 3e19], [float("-inf"), -2.0], [1e30, -1e30]],
                         dtype=torch.float32, device="cuda")      # 16 pairs; the last three: an infinite product
    fT = np.float32(O.fT(kind, f32=True))
    lo_bits = int(np.array([np.float32(fT - np.float32(2.0 ** -12))]).view(np.uint32)[0])
    ranges = [(0x00000000, 0x7F800000, 0), (0x80000000, lo_bits, 0), (0x80000000, lo_bits, 1), (0x00000000, 0x00000000, 1)]
    wg, wu, t0 = Worst(), Worst(), time.time()
    for first, last, s in ranges:
        for start, count in pattern_blocks(first, last):
            PT.say(f"exhaustive gated bwd {kind} s={s}: patterns from {start:#010x}, {count} of them, stride {STRIDE}")
            act = patterns_to_device(start, count)
            pick = pairs[torch.arange(count, device="cuda") % pairs.shape[0]]
            gh, up = pick[:, 0].clone(), pick[:, 1].clone()          # clones: a one-element view is not realigned by contiguous()
            mask = torch.full((B.mask_bytes(count),), 0xFF if s else 0, dtype=torch.uint8, device="cuda")
            gg, gu = B.geglu_invact_bwd(kind, act, up, mask, gh)
            torch.cuda.synchronize()
            a64, g64, u64 = (t.cpu().numpy().astype(np.float64) for t in (act, gh, up))
            gg_ref, gu_ref = O.glu_bwd(kind, a64, u64, mask.cpu().numpy(), g64)
            gg_got, gu_got = gg.cpu().numpy().astype(np.float64), gu.cpu().numpy().astype(np.float64)
            wu.update(start, gu_got, gu_ref, PT.forward_errors(gu_got, gu_ref, "fp32"))
            with np.errstate(invalid="ignore", over="ignore"):
                err = PT.backward_errors(gg_got, gg_ref, g64 * u64, "fp32")
                # grad_h * up overflows binary32 but the product with a small q would not: the kernel gives the infinity
                err[np.isinf((g64 * u64).astype(np.float32)) & np.isfinite(g64) & np.isfinite(gg_ref.astype(np.float32))] = 0.0
                wg.update(start, gg_got, gg_ref, err)
    print(f"\nRESULT gated bwd {kind} stride {STRIDE}: {wg.total} cases, grad_gate worst {wg.tol:.4f} of the tolerance at "
          f"{wg.where_tol}, grad_up worst {wu.tol:.4f} at {wu.where_tol} [{time.time() - t0:.0f} s]", flush=True)
    assert wu.tol <= 1.0, wu.where_tol
    assert wg.tol <= 1.0, wg.where_tol


@pytest.mark.parametrize("kind", KINDS)
def test_mask_free_backwards_over_all_binary32_saved_values(kind):
    """invact_pbit_bwd and invact_sbit_bwd over every saved value they can meet, grad_y = 1, against the oracle with
    the backward's tolerance.  Precision bit: the patterns of the plain backward's test with bit 0 forced to s.
    Sign bit: magnitude m = y - C with the sign bit as s; s = 0: every m from 0 to +inf, s = 1: m up to -C + 2^-12
    (saved outputs up to +0 and a little beyond)."""
    fT = np.float32(O.fT(kind, f32=True))
    lo_bits = int(np.array([np.float32(fT - np.float32(2.0 ** -12))]).view(np.uint32)[0])
    top_bits = int(np.array([np.float32(-fT + np.float32(2.0 ** -12))]).view(np.uint32)[0])
    wp, ws, t0 = Worst(), Worst(), time.time()
    ones = lambda count: torch.ones(count, dtype=torch.float32, device="cuda")
    for first, last, s in [(0x00000000, 0x7F800000, 0), (0x80000000, lo_bits, 0), (0x80000000, lo_bits, 1), (0x00000000, 0x00000000, 1)]:
        for start, count in pattern_blocks(first, last):
            PT.say(f"exhaustive pbit bwd {kind} s={s}: patterns from {start:#010x}, {count} of them, stride {STRIDE}")
            y = ((patterns_to_device(start, count).view(torch.int32) & -2) | s).view(torch.float32)
            gx = B.invact_pbit_bwd(kind, y, ones(count))
            torch.cuda.synchronize()
            ref = O.pbit_bwd(kind, "fp32", y.cpu().numpy().astype(np.float64), np.ones(count))
            got = gx.cpu().numpy().astype(np.float64)
            wp.update(start, got, ref, PT.backward_errors(got, ref, np.ones(count), "fp32"))
    for first, last, s in [(0x00000000, 0x7F800000, 0), (0x00000000, top_bits, 1)]:
        for start, count in pattern_blocks(first, last):
            PT.say(f"exhaustive sbit bwd {kind} s={s}: magnitudes from {start:#010x}, {count} of them, stride {STRIDE}")
            yt = (patterns_to_device(start, count).view(torch.int32) | (-0x80000000 if s else 0)).view(torch.float32)
            gx = B.invact_sbit_bwd(kind, yt, ones(count))
            torch.cuda.synchronize()
            ref = O.sbit_bwd(kind, yt.cpu().numpy().astype(np.float64), np.ones(count))
            got = gx.cpu().numpy().astype(np.float64)
            ws.update(start, got, ref, PT.backward_errors(got, ref, np.ones(count), "fp32"))
    print(f"\nRESULT pbit bwd {kind} stride {STRIDE}: {wp.total} cases, worst {wp.tol:.4f} of the tolerance at {wp.where_tol}; "
          f"sbit bwd: {ws.total} cases, worst {ws.tol:.4f} at {ws.where_tol} [{time.time() - t0:.0f} s]", flush=True)
    assert wp.tol <= 1.0, wp.where_tol
    assert ws.tol <= 1.0, ws.where_tol
