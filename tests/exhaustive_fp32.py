#!/usr/bin/env python3
"""Exhaustive binary32 check of the GPU kernels against the oracle (run by hand; not collected by pytest).

    python tests/exhaustive_fp32.py fwd  KIND      every one of the 2^32 binary32 inputs through invact_fwd
    python tests/exhaustive_fp32.py bwd  KIND      every binary32 y >= f(T) - 2^-12 with s = 0, and every
                                                    y in [f(T) - 2^-12, +0] with s = 1, through invact_bwd (grad_y = 1)

Prints the worst error in units of the tolerance of tests/parity.py (<= 1 passes), the worst literal ulp
error, and for the forward whether every mask bit matched.  Takes a few minutes per kind; progress is printed
after every block of 2^26 patterns.
"""
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))
import oracle as O                                    # noqa: E402
import parity as PT                                   # noqa: E402
from paper_2407_15545_amd import binding as B         # noqa: E402

BLOCK = 1 << 26


def blocks_of(first, last):
    """Pattern ranges [a, b) covering first..last inclusive."""
    a = first
    while a <= last:
        b = min(a + BLOCK, last + 1)
        yield a, b
        a = b


def patterns_to_device(a, b):
    bits = torch.arange(a, b, dtype=torch.int64, device="cuda").to(torch.int32)   # wraps for patterns >= 2^31
    return bits.view(torch.float32)


def main():
    mode, kind = sys.argv[1], sys.argv[2]
    torch.cuda.set_device(0)
    worst_tol, worst_ulp, where_tol, where_ulp, mask_ok, total = 0.0, 0.0, None, None, True, 0
    t0 = time.time()
    if mode == "fwd":
        ranges = [(0x00000000, 0xFFFFFFFF, None)]
    else:
        fT = np.float32(O.fT(kind, f32=True))
        lo = np.float32(fT - np.float32(2.0 ** -12))
        lo_bits = int(np.array([lo]).view(np.uint32)[0])                # negative: larger pattern = more negative
        ranges = [(0x00000000, 0x7F800000, 0),                           # s = 0: +0 .. +inf
                  (0x80000000, lo_bits, 0),                              # s = 0: -0 .. f(T) - 2^-12
                  (0x80000000, lo_bits, 1),                              # s = 1: -0 .. f(T) - 2^-12
                  (0x00000000, 0x00000000, 1)]                           # s = 1: +0
    for first, last, s in ranges:
        for a, b in blocks_of(first, last):
            v = patterns_to_device(a, b)
            n = b - a
            if mode == "fwd":
                y, m = B.invact_fwd(kind, v)
                torch.cuda.synchronize()
                x64 = v.cpu().numpy().astype(np.float64)
                ye, _, m_ref = O.invact_fwd(kind, "fp32", x64)
                mask_ok &= bool(np.array_equal(m.cpu().numpy(), m_ref))
                got = y.cpu().numpy().astype(np.float64)
                err = PT.forward_errors(got, ye, "fp32")
                ref = ye
            else:
                mask = torch.full((B.mask_bytes(n),), 0xFF if s else 0, dtype=torch.uint8, device="cuda")
                g = torch.ones(n, dtype=torch.float32, device="cuda")
                gx = B.invact_bwd(kind, v, mask, g)
                torch.cuda.synchronize()
                y64 = v.cpu().numpy().astype(np.float64)
                ref = O.q(kind, y64, np.full(n, s, np.uint8))
                got = gx.cpu().numpy().astype(np.float64)
                err = PT.backward_errors(got, ref, np.ones(n), "fp32")
            i = int(np.nanargmax(err))
            if err[i] > worst_tol:
                worst_tol, where_tol = float(err[i]), (hex(a + i), float(got[i]), float(ref[i]))
            with np.errstate(invalid="ignore", over="ignore"):
                lit = np.where(np.isfinite(ref) & np.isfinite(got) & (np.abs(ref) >= 2.0 ** -126),
                               np.abs(got - ref) / PT.ulp(ref, "fp32"), 0.0)
            j = int(np.argmax(lit))
            if lit[j] > worst_ulp:
                worst_ulp, where_ulp = float(lit[j]), (hex(a + j), float(got[j]), float(ref[j]))
            total += n
            print(f"{mode} {kind} s={s} patterns {a:#010x}..{b - 1:#010x}: worst so far {worst_tol:.3f} of the tolerance, "
                  f"{worst_ulp:.3g} ulp literally, masks {'ok' if mask_ok else 'DIFFER'}  [{time.time() - t0:.0f} s]", flush=True)
    print(f"RESULT {mode} {kind}: {total} cases, worst {worst_tol:.4f} of the tolerance at {where_tol}, "
          f"worst literal {worst_ulp:.4g} ulp at {where_ulp}, masks {'bit-exact' if mask_ok else 'DIFFER'}", flush=True)
    sys.exit(0 if worst_tol <= 1.0 and mask_ok else 1)


if __name__ == "__main__":
    main()
