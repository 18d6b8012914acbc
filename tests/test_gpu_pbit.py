"""GPU parity of the precision-bit variant (invact_pbit_fwd / invact_pbit_bwd)
against the oracle.

Forward: bit 0 of every stored pattern must equal the indicator exactly; the
stored value may differ from the oracle's (correctly rounded, then tagged) one
by at most 2 ulp, i.e. one step of the even-spaced grid the tagged values live
on.  Backward: fed with the ORACLE's stored y, same tolerance as invact_bwd."""
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
SIZES = [1, 7, 63, 64, 65, 511, 513, 4096 + 8, (1 << 20) + 3]


def patterns(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16).astype(np.uint32)
    return t.view(torch.int32).cpu().numpy().view(np.uint32)


def inputs(n, seed, dtype):
    x = synth.to_storage(synth.normal(n, seed, 2.0), dtype)
    g = synth.to_storage(synth.normal(n, seed + 1, 1.0), dtype)
    return x, g


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("kind", KINDS)
def test_pbit_forward_and_backward(kind, dtype):
    for n in SIZES:
        PT.say(f"invact_pbit fwd/bwd {kind} {dtype} n={n}")
        xs, gs = inputs(n, 300 + n, dtype)
        x64, g64 = synth.storage_to_f64(xs, dtype), synth.storage_to_f64(gs, dtype)
        ye, ys = O.pbit_fwd(kind, dtype, x64)
        y = B.invact_pbit_fwd(kind, PT.to_device(xs, dtype))
        torch.cuda.synchronize()
        assert np.array_equal(patterns(y) & 1, O.indicator(kind, x64).astype(np.uint32)), "indicator bit differs"
        err = PT.forward_errors(PT.to_f64(y), ys, dtype)
        assert err.max() <= 1.0, (n, PT.worst(err, x64, ys, PT.to_f64(y)))
        # and never further than 3 ulp from the exact value (2 of the evaluation + 1 of the tag)
        assert (PT.forward_errors(PT.to_f64(y), ye, dtype) * 2).max() <= 3.0
        # backward from the oracle's stored (tagged) output
        ref = O.pbit_bwd(kind, dtype, ys, g64)
        gx = B.invact_pbit_bwd(kind, PT.to_device(synth.f64_to_storage_exact(ys, dtype), dtype), PT.to_device(gs, dtype))
        torch.cuda.synchronize()
        err = PT.backward_errors(PT.to_f64(gx), ref, g64, dtype)
        assert err.max() <= 1.0, (n, PT.worst(err, ys, g64, ref, PT.to_f64(gx)))


@pytest.mark.parametrize("kind", KINDS)
def test_pbit_every_bf16_input(kind):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    with np.errstate(invalid="ignore"):
        x64 = synth.storage_to_f64(bits, "bf16")
    ye, ys = O.pbit_fwd(kind, "bf16", x64)
    PT.say(f"invact_pbit_fwd {kind} all bf16 patterns")
    y = B.invact_pbit_fwd(kind, PT.to_device(bits, "bf16"))
    torch.cuda.synchronize()
    assert np.array_equal(patterns(y) & 1, O.indicator(kind, x64).astype(np.uint32))       # NaNs included: their indicator is 0
    err = PT.forward_errors(PT.to_f64(y), ys, "bf16")
    assert err.max() <= 1.0, PT.worst(err, x64, ys, PT.to_f64(y))
    # every (tagged y) pattern through the backward, grad_y = 1
    with np.errstate(invalid="ignore"):
        y64 = x64                                                    # reuse the patterns as stored outputs
    strict = (np.abs(y64) <= 1.0) | ((bits & 1) == 0) | np.isnan(y64)     # left-branch y far outside f's range: see test_gpu_parity
    ref = O.pbit_bwd(kind, "bf16", y64, np.ones(y64.size))
    gx = B.invact_pbit_bwd(kind, PT.to_device(bits, "bf16"), torch.ones(y64.size, dtype=torch.bfloat16, device="cuda"))
    torch.cuda.synchronize()
    got = PT.to_f64(gx)
    err = PT.backward_errors(got[strict], ref[strict], np.ones(int(strict.sum())), "bf16")
    assert err.max() <= 1.0, PT.worst(err, y64[strict], ref[strict], got[strict])


@pytest.mark.parametrize("dtype", DTYPES)
def test_pbit_in_place(dtype):
    n = 70001
    xs, gs = inputs(n, 77, dtype)
    x, g = PT.to_device(xs, dtype), PT.to_device(gs, dtype)
    PT.say(f"invact_pbit in place {dtype}")
    y = B.invact_pbit_fwd("silu", x)
    gx = B.invact_pbit_bwd("silu", y, g)
    x2, g2 = x.clone(), g.clone()
    B.invact_pbit_fwd("silu", x2, y=x2)
    B.invact_pbit_bwd("silu", y, g2, grad_x=g2)
    torch.cuda.synchronize()
    assert torch.equal(x2.view(torch.uint8), y.view(torch.uint8))
    assert torch.equal(g2.view(torch.uint8), gx.view(torch.uint8))


@pytest.mark.parametrize("kind", KINDS)
def test_pbit_nan_inputs_stay_nan_in_binary32(kind):
    """Clearing bit 0 of the signalling NaNs 0x7F800001 / 0xFF800001 would leave an infinity: the forward
    must store a NaN for every NaN input, and the backward must give NaN for it (the oracle does both)."""
    pats = np.array([0x7F800001, 0xFF800001, 0x7FC00000, 0xFFC00001, 0x7FFFFFFF, 0x7F800002] * 100, dtype=np.uint32)
    x = torch.from_numpy(pats.view(np.int32)).cuda().view(torch.float32)
    ye, ys = O.pbit_fwd(kind, "fp32", np.full(pats.size, np.nan))
    assert np.all(np.isnan(ys))
    PT.say(f"invact_pbit_fwd {kind} fp32 NaN patterns")
    y = B.invact_pbit_fwd(kind, x)
    gx = B.invact_pbit_bwd(kind, y, torch.ones_like(y))
    torch.cuda.synchronize()
    assert torch.isnan(y).all(), patterns(y)[:6]
    assert torch.isnan(gx).all()
    assert np.all(np.isnan(O.pbit_bwd(kind, "fp32", ys, np.ones(pats.size))))
