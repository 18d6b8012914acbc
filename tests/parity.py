"""Shared helpers of the GPU parity tests: tolerance rules and tensor plumbing.

Tolerances:
  forward  : |gpu - f(x)| <= 2 ulp_D(f(x)), D the storage dtype; where
             |f(x)| < 2^-126 an absolute 2^-126 (gradual underflow and flush
             to zero both pass).
  backward : |gpu - ref| <= 2 ulp_D(ref)  or  <= 2 * 2^-23 * |g|, with g the
             factor q is multiplied by (grad_y, or grad_h * up): two binary32
             ulps at q's natural scale of 1.  The second arm is needed because
             q = 1 + h passes through zero, where no binary32 evaluation can
             keep a result-relative bound.
  masks    : bit-exact, padding included.
"""
import os
import sys

import numpy as np
import torch

import synth

P_BITS = {"fp32": 24, "bf16": 8}
TORCH_DTYPE = {"fp32": torch.float32, "bf16": torch.bfloat16}
F32_MAX = float(np.finfo(np.float32).max)
BF16_MAX = float.fromhex("0x1.fep127")
MAX_FINITE = {"fp32": F32_MAX, "bf16": BF16_MAX}


# INVACT_REPORT_DIR: where a run may leave its reports (the names of the cases it ran, accuracy figures);
# nothing is written when it is not set.
REPORT_DIR = os.environ.get("INVACT_REPORT_DIR") or None


def say(*a):
    """Name the case before a GPU step (stderr, flushed); with INVACT_REPORT_DIR set, also keep a copy there."""
    print(*a, file=sys.stderr, flush=True)
    if REPORT_DIR and os.path.isdir(REPORT_DIR):
        with open(os.path.join(REPORT_DIR, "parity_report.txt"), "a") as fh:
            print(*a, file=fh)


def ulp(ref, dtype):
    """Spacing of the dtype's grid at |ref| (subnormal spacing below 2^-126)."""
    a = np.abs(np.asarray(ref, dtype=np.float64))
    with np.errstate(divide="ignore", invalid="ignore"):
        e = np.floor(np.log2(a))
    e = np.where(np.isfinite(e), e, -126.0)
    e = np.clip(e, -126.0, 127.0)
    return np.exp2(e - (P_BITS[dtype] - 1))


def to_device(storage, dtype):
    """Storage array from synth (float32 / uint16 bit patterns) -> CUDA tensor."""
    if dtype == "fp32":
        return torch.from_numpy(np.ascontiguousarray(storage, dtype=np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(storage, dtype=np.uint16).view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t):
    """CUDA tensor -> float64 numpy array of the exact stored values."""
    t = t.detach()
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return synth.bf16_bits_to_f32(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def expected_overflow(ref, dtype):
    """Where the rounded reference is infinite (|ref| beyond the largest finite value + half an ulp)."""
    lim = MAX_FINITE[dtype] + 0.5 * float(ulp(MAX_FINITE[dtype], dtype))
    return np.abs(ref) >= lim


def forward_errors(gpu, ref, dtype):
    """Error of gpu vs the exact double reference in units of the tolerance (<= 1 passes)."""
    gpu = np.asarray(gpu, np.float64); ref = np.asarray(ref, np.float64)
    out = np.zeros(ref.shape)
    nan = np.isnan(ref)
    out[nan] = np.where(np.isnan(gpu[nan]), 0.0, np.inf)
    ovf = expected_overflow(ref, dtype) & ~nan
    out[ovf] = np.where(gpu[ovf] == np.sign(ref[ovf]) * np.inf, 0.0, np.inf)
    rest = ~nan & ~ovf
    tol = 2.0 * ulp(ref[rest], dtype)
    tol = np.where(np.abs(ref[rest]) < 2.0 ** -126, 2.0 ** -126, tol)
    with np.errstate(invalid="ignore"):
        err = np.abs(gpu[rest] - ref[rest]) / tol
    out[rest] = np.where(np.isfinite(gpu[rest]), err, np.inf)
    return out


def backward_errors(gpu, ref, scale, dtype):
    """Error of a backward output in units of the tolerance; scale = |g| (see module docstring)."""
    gpu = np.asarray(gpu, np.float64); ref = np.asarray(ref, np.float64)
    scale = np.abs(np.asarray(scale, np.float64))
    out = np.zeros(ref.shape)
    nan = np.isnan(ref)
    out[nan] = np.where(np.isnan(gpu[nan]), 0.0, np.inf)
    ovf = expected_overflow(ref, dtype) & ~nan
    out[ovf] = np.where(gpu[ovf] == np.sign(ref[ovf]) * np.inf, 0.0, np.inf)
    rest = ~nan & ~ovf
    tol = np.maximum(2.0 * ulp(ref[rest], dtype), 2.0 * 2.0 ** -23 * scale[rest])
    with np.errstate(invalid="ignore"):
        err = np.abs(gpu[rest] - ref[rest]) / tol
    out[rest] = np.where(np.isfinite(gpu[rest]), err, np.inf)
    return out


def literal_ulps(gpu, ref, dtype):
    """Plain result-relative error in ulps of the reference (reported, not asserted)."""
    with np.errstate(invalid="ignore"):
        return np.abs(np.asarray(gpu, np.float64) - np.asarray(ref, np.float64)) / ulp(ref, dtype)


def worst(err, *cols, k=3):
    """Readable description of the k largest entries of err with the matching rows of cols."""
    idx = np.argsort(-np.nan_to_num(err, nan=np.inf))[:k]
    return [(int(i), float(err[i])) + tuple(float(c[i]) for c in cols) for i in idx]
