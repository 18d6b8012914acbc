"""Tensors beyond 4 GiB: element and byte offsets that do not fit 32 bits.

An element-wise kernel must produce the same bits for an element wherever it sits, so windows of a very large
tensor -- its first elements, a stretch across the 2^32-byte mark, a stretch across the 2^32-element mark where
there is one, and the ragged end -- are compared bit for bit (masks included) with the same entry point run on a
copy of the window alone, and the window's results with the oracle.  Needs about 75 GB of device memory."""
import numpy as np
import pytest
import torch

import oracle as O
import parity as PT
from paper_2407_15545_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def give_the_memory_back():
    """The tests here hold tens of gigabytes; return torch's cached blocks to the device afterwards."""
    yield
    torch.cuda.empty_cache()


WINDOW = (1 << 20) + 64          # elements; window starts are multiples of 64, so a window owns whole mask words


def windows(n, itemsize):
    """Window starts: the first elements, across the 2^32-byte mark, across the 2^32-element mark if there is one,
    and the last window, which ends at n (ragged)."""
    half = (WINDOW // 2) // 64 * 64
    starts = [0, (1 << 32) // itemsize - half]
    if n > (1 << 32) + WINDOW:
        starts.append((1 << 32) - half)
    starts.append((n - WINDOW + 63) // 64 * 64)
    return starts


def window_of(t, start, n):
    return t[start:min(start + WINDOW, n)].clone()


def mask_window(mask, start, count):
    return mask[start // 8: start // 8 + B.mask_bytes(count)].clone()


@pytest.mark.parametrize("dtype, log2n", [("bf16", 32), ("fp32", 31)])
def test_forward_and_backward_beyond_4_gib(dtype, log2n):
    free, _ = torch.cuda.mem_get_info()
    if free < 90 << 30:
        pytest.skip("needs about 75 GB of free device memory")
    td = PT.TORCH_DTYPE[dtype]
    n = (1 << log2n) + (1 << 20) + 77
    kind = "gelu_erf"
    PT.say(f"large tensors {dtype}: n = {n} ({n * torch.empty(0, dtype=td).element_size() / 2 ** 30:.1f} GiB each)")
    gen = torch.Generator(device="cuda").manual_seed(5)
    x = torch.empty(n, dtype=td, device="cuda")
    for a in range(0, n, 1 << 28):                                     # filled piecewise: no 2^32-element temporaries
        b = min(a + (1 << 28), n)
        x[a:b] = torch.randn(b - a, generator=gen, device="cuda", dtype=torch.float32).mul_(2.0).to(td)
    g = torch.empty(n, dtype=td, device="cuda")
    for a in range(0, n, 1 << 28):
        b = min(a + (1 << 28), n)
        g[a:b] = torch.randn(b - a, generator=gen, device="cuda", dtype=torch.float32).to(td)

    PT.say("  invact_fwd / invact_bwd on the whole tensor")
    y, mask = B.invact_fwd(kind, x)
    gx = B.invact_bwd(kind, y, mask, g)
    PT.say("  swiglu_invact_fwd / swiglu_invact_bwd on the whole tensor")
    act, h, gmask = B.swiglu_invact_fwd(x, g)
    gg, gu = B.swiglu_invact_bwd(act, g, gmask, x)
    torch.cuda.synchronize()
    assert mask.numel() == B.mask_bytes(n)

    for start in windows(n, x.element_size()):
        count = min(WINDOW, n - start)
        PT.say(f"  window at element {start} ({count} elements)")
        xs, gs = window_of(x, start, n), window_of(g, start, n)
        ys, ms = B.invact_fwd(kind, xs)
        gxs = B.invact_bwd(kind, ys, ms, gs)
        acts, hs, gms = B.swiglu_invact_fwd(xs, gs)
        ggs, gus = B.swiglu_invact_bwd(acts, gs, gms, xs)
        torch.cuda.synchronize()
        same = lambda big, small: torch.equal(window_of(big, start, n).view(torch.uint8), small.view(torch.uint8))
        assert same(y, ys) and same(gx, gxs) and same(act, acts) and same(h, hs) and same(gg, ggs) and same(gu, gus), start
        # mask bits of the window (the last byte of a ragged window holds zero padding in both)
        assert torch.equal(mask_window(mask, start, count), ms) and torch.equal(mask_window(gmask, start, count), gms), start
        # and the window against the oracle
        x64 = PT.to_f64(xs)
        ye, _, m_ref = O.invact_fwd(kind, dtype, x64)
        assert np.array_equal(ms.cpu().numpy(), m_ref)
        assert PT.forward_errors(PT.to_f64(ys), ye, dtype).max() <= 1.0

    # the two mask-free variants share the kernels' skeleton; their windows bit for bit as well
    del y, gx, act, h, gg, gu, mask, gmask
    PT.say("  precision-bit and sign-bit entry points on the whole tensor")
    yp = B.invact_pbit_fwd(kind, x)
    gp = B.invact_pbit_bwd(kind, yp, g)
    yt = B.invact_sbit_fwd(kind, x)
    yd = B.invact_sbit_decode(kind, yt)
    gs_ = B.invact_sbit_bwd(kind, yt, g)
    torch.cuda.synchronize()
    for start in windows(n, x.element_size()):
        xs, gs = window_of(x, start, n), window_of(g, start, n)
        yps = B.invact_pbit_fwd(kind, xs)
        yts = B.invact_sbit_fwd(kind, xs)
        small = [yps, B.invact_pbit_bwd(kind, yps, gs), yts, B.invact_sbit_decode(kind, yts), B.invact_sbit_bwd(kind, yts, gs)]
        torch.cuda.synchronize()
        for big, sm in zip([yp, gp, yt, yd, gs_], small):
            assert torch.equal(window_of(big, start, n).view(torch.uint8), sm.view(torch.uint8)), start


def test_products_next_to_their_size_limit():
    """The matrix products address their operands with 32-bit byte offsets, which is why each matrix must hold fewer
    than 2^31 elements: a saved tensor of 2^31 - 2^20 elements (4 GiB) goes through all three.  Rows from both
    ends against the oracle for the forward and the input gradient; for the weight gradient, whose sum runs over
    all 33 million rows, the whole against the sum of the two halves computed separately."""
    free, _ = torch.cuda.mem_get_info()
    if free < 40 << 30:
        pytest.skip("needs about 20 GB of free device memory")
    import synth
    kind, K, N = "silu", 64, 64
    M = ((1 << 31) - (1 << 20)) // K
    assert M % 128 == 0 and M * K < 1 << 31
    PT.say(f"products at M = {M}, N = {N}, K = {K}: {M * K * 2 / 2 ** 30:.2f} GiB per M x K matrix")
    gen = torch.Generator(device="cuda").manual_seed(9)
    yt = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    g = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    for a in range(0, M, 1 << 22):
        b = min(a + (1 << 22), M)
        x = torch.randn((b - a) * K, generator=gen, device="cuda", dtype=torch.float32).mul_(2.0).to(torch.bfloat16)
        yt[a:b] = B.invact_sbit_fwd(kind, x).view(b - a, K)
        g[a:b] = torch.randn((b - a, N), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    w = (torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32) * K ** -0.5).to(torch.bfloat16)
    out = B.invact_sbit_linear_fwd(kind, yt, w)
    gx = B.invact_sbit_linear_dgrad(kind, yt, g, w)
    gw = B.invact_sbit_linear_wgrad_ws(kind, yt, g)
    half = M // 2
    gw_halves = B.invact_sbit_linear_wgrad_ws(kind, yt[:half], g[:half]).float() + B.invact_sbit_linear_wgrad_ws(kind, yt[half:], g[half:]).float()
    torch.cuda.synchronize()
    f64 = lambda t: PT.to_f64(t.reshape(-1)).reshape(t.shape)
    w64 = f64(w)
    for rows in (slice(0, 96), slice(M - 96, M), slice(M // 2 - 48, M // 2 + 48)):
        yt64, g64 = f64(yt[rows]), f64(g[rows])
        dec = O.sbit_decode(kind, "bf16", yt64.reshape(-1))[1].reshape(yt64.shape)
        ref = O.sbit_linear(kind, "bf16", yt64, w64)
        tol = 2.0 * PT.ulp(ref, "bf16") + (K + 2) * 2.0 ** -24 * (np.abs(dec) @ np.abs(w64).T)
        assert np.all(np.abs(f64(out[rows]) - ref) <= tol), rows
        ref = O.sbit_linear_dgrad(kind, yt64, g64, w64)
        q = np.abs(O.sbit_bwd(kind, yt64.reshape(-1), np.ones(yt64.size)).reshape(yt64.shape))
        tol = 2.0 * PT.ulp(ref, "bf16") + (N + 2) * 2.0 ** -24 * (np.abs(g64) @ np.abs(w64)) * q + 2.0 ** -22 * np.abs(g64 @ w64)
        assert np.all(np.abs(f64(gx[rows]) - ref) <= tol), rows
    # three bfloat16 roundings and two orders of a binary32 sum over 33 million terms of size ~1
    scale = float(gw_halves.abs().max())
    assert float((gw.float() - gw_halves).abs().max()) <= 2.0 ** -6 * scale + 1e-3 * scale
    assert scale > 100.0          # sums of 3e7 products of O(1) numbers: far from zero, so garbage would show
