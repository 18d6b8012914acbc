"""ctypes front end of the CPU oracle (``invact_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library and its Python binding never
import this package, and this package imports nothing of theirs.

All arrays are float64 numpy arrays holding the exact values of the binary32 /
bfloat16 inputs; masks are uint8 arrays of ``mask_bytes(n)`` bytes.
"""
import ctypes
import os
import subprocess

import numpy as np

GELU_TANH, GELU_ERF, SILU = 0, 1, 2
FP32, BF16 = 0, 1
KINDS = {"gelu_tanh": GELU_TANH, "gelu_erf": GELU_ERF, "silu": SILU}
DTYPES = {"fp32": FP32, "bf16": BF16}

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "invact_oracle.c")
_LIB = os.path.join(_HERE, "libinvact_oracle.so")


def build(force=False, src=_SRC, out=_LIB, extra_flags=()):
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP)."""
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
           *extra_flags, "-o", out, src, "-lm"]
    subprocess.run(cmd, check=True)
    return out


_dbl_p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_u8_p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")


def load(path=None):
    """Load a compiled oracle and declare its prototypes."""
    lib = ctypes.CDLL(path or build())
    c_int, c_size, c_dbl = ctypes.c_int, ctypes.c_size_t, ctypes.c_double
    protos = {
        "oracle_f_scalar": (c_dbl, [c_int, c_dbl]),
        "oracle_df_scalar": (c_dbl, [c_int, c_dbl]),
        "oracle_finv_scalar": (c_dbl, [c_int, c_dbl, c_int]),
        "oracle_q_scalar": (c_dbl, [c_int, c_dbl, c_int]),
        "oracle_round_scalar": (c_dbl, [c_int, c_dbl]),
        "oracle_T": (c_dbl, [c_int]),
        "oracle_fT": (c_dbl, [c_int]),
        "oracle_T_f32": (c_dbl, [c_int]),
        "oracle_fT_f32": (c_dbl, [c_int]),
        "oracle_default_coeffs": (None, [_dbl_p]),
        "oracle_f": (None, [c_int, _dbl_p, _dbl_p, c_size]),
        "oracle_df": (None, [c_int, _dbl_p, _dbl_p, c_size]),
        "oracle_finv": (None, [c_int, _dbl_p, _u8_p, _dbl_p, c_size]),
        "oracle_q": (None, [c_int, _dbl_p, _u8_p, _dbl_p, c_size]),
        "oracle_q_coeffs": (None, [c_int, _dbl_p, c_dbl, _dbl_p, _u8_p, _dbl_p, c_size]),
        "oracle_printed_coeffs": (None, [_dbl_p]),
        "oracle_round": (None, [c_int, _dbl_p, _dbl_p, c_size]),
        "oracle_indicator": (None, [c_int, _dbl_p, _u8_p, c_size]),
        "oracle_mask_bytes": (c_size, [c_size]),
        "oracle_pack": (None, [_u8_p, _u8_p, c_size]),
        "oracle_unpack": (None, [_u8_p, _u8_p, c_size]),
        "oracle_invact_fwd": (None, [c_int, c_int, _dbl_p, _dbl_p, _dbl_p, _u8_p, c_size]),
        "oracle_invact_bwd": (None, [c_int, _dbl_p, _u8_p, _dbl_p, _dbl_p, c_size]),
        "oracle_glu_fwd": (None, [c_int, c_int, _dbl_p, _dbl_p, _dbl_p, _dbl_p, _dbl_p, _u8_p, c_size]),
        "oracle_glu_bwd": (None, [c_int, _dbl_p, _dbl_p, _u8_p, _dbl_p, _dbl_p, _dbl_p, c_size]),
        "oracle_tag_lsb": (c_dbl, [c_int, c_dbl, c_int]),
        "oracle_read_lsb": (c_int, [c_int, c_dbl]),
        "oracle_pbit_fwd": (None, [c_int, c_int, _dbl_p, _dbl_p, _dbl_p, c_size]),
        "oracle_pbit_bwd": (None, [c_int, c_int, _dbl_p, _dbl_p, _dbl_p, c_size]),
        "oracle_sbit_fwd": (None, [c_int, c_int, _dbl_p, _dbl_p, _dbl_p, c_size]),
        "oracle_sbit_decode": (None, [c_int, c_int, _dbl_p, _dbl_p, _dbl_p, c_size]),
        "oracle_sbit_bwd": (None, [c_int, _dbl_p, _dbl_p, _dbl_p, c_size]),
        "oracle_sbit_linear": (None, [c_int, c_int, _dbl_p, _dbl_p, ctypes.c_void_p, _dbl_p, c_size, c_size, c_size]),
        "oracle_sbit_linear_wgrad": (None, [c_int, c_int, _dbl_p, _dbl_p, _dbl_p, c_size, c_size, c_size]),
        "oracle_sbit_linear_dgrad": (None, [c_int, _dbl_p, _dbl_p, _dbl_p, _dbl_p, c_size, c_size, c_size]),
        "oracle_num_threads": (c_int, []),
    }
    for name, (res, args) in protos.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = load()
    return _lib


def _kind(kind):
    return KINDS[kind] if isinstance(kind, str) else int(kind)


def _dtype(dtype):
    return DTYPES[dtype] if isinstance(dtype, str) else int(dtype)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64).reshape(-1)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8).reshape(-1)


def mask_bytes(n):
    return int(lib().oracle_mask_bytes(n))


def T(kind, f32=False):
    return (lib().oracle_T_f32 if f32 else lib().oracle_T)(_kind(kind))


def fT(kind, f32=False):
    return (lib().oracle_fT_f32 if f32 else lib().oracle_fT)(_kind(kind))


def f(kind, x):
    x = _f64(x); y = np.empty_like(x)
    lib().oracle_f(_kind(kind), x, y, x.size)
    return y


def df(kind, x):
    x = _f64(x); d = np.empty_like(x)
    lib().oracle_df(_kind(kind), x, d, x.size)
    return d


def finv(kind, y, s):
    y = _f64(y); s = _u8(s); x = np.empty_like(y)
    lib().oracle_finv(_kind(kind), y, s, x, y.size)
    return x


def q(kind, y, s, coeffs=None, fT_value=None):
    """The paper's approximation.  coeffs / fT_value override the constants."""
    y = _f64(y); s = _u8(s); out = np.empty_like(y)
    if coeffs is None and fT_value is None:
        lib().oracle_q(_kind(kind), y, s, out, y.size)
    else:
        c = default_coeffs() if coeffs is None else _f64(coeffs)
        t = fT(kind, f32=True) if fT_value is None else float(fT_value)
        lib().oracle_q_coeffs(_kind(kind), c, t, y, s, out, y.size)
    return out


def default_coeffs():
    """gelu_left[8], gelu_right[5], silu_left[4], silu_right[5] (binary32-rounded)."""
    c = np.empty(22, dtype=np.float64)
    lib().oracle_default_coeffs(c)
    return c


def printed_coeffs():
    """Same layout, exactly as printed in the appendix (unrounded)."""
    c = np.empty(22, dtype=np.float64)
    lib().oracle_printed_coeffs(c)
    return c


def round_to(dtype, v):
    v = _f64(v); out = np.empty_like(v)
    lib().oracle_round(_dtype(dtype), v, out, v.size)
    return out


def indicator(kind, x):
    x = _f64(x); s = np.empty(x.size, dtype=np.uint8)
    lib().oracle_indicator(_kind(kind), x, s, x.size)
    return s


def pack(s):
    s = _u8(s); m = np.empty(mask_bytes(s.size), dtype=np.uint8)
    lib().oracle_pack(s, m, s.size)
    return m


def unpack(mask, n):
    mask = _u8(mask); s = np.empty(n, dtype=np.uint8)
    assert mask.size >= (n + 7) // 8
    lib().oracle_unpack(mask, s, n)
    return s


def invact_fwd(kind, dtype, x):
    """-> (y_exact, y_stored, mask)"""
    x = _f64(x)
    ye = np.empty_like(x); ys = np.empty_like(x)
    m = np.empty(mask_bytes(x.size), dtype=np.uint8)
    lib().oracle_invact_fwd(_kind(kind), _dtype(dtype), x, ye, ys, m, x.size)
    return ye, ys, m


def invact_bwd(kind, y, mask, grad_y):
    """-> grad_x (unrounded double)"""
    y = _f64(y); g = _f64(grad_y); mask = _u8(mask)
    assert g.size == y.size and mask.size >= (y.size + 7) // 8
    gx = np.empty_like(y)
    lib().oracle_invact_bwd(_kind(kind), y, mask, g, gx, y.size)
    return gx


def glu_fwd(kind, dtype, gate, up):
    """-> (a_exact, a_stored, h_exact, mask)"""
    gate = _f64(gate); up = _f64(up)
    assert gate.size == up.size
    ae = np.empty_like(gate); as_ = np.empty_like(gate); he = np.empty_like(gate)
    m = np.empty(mask_bytes(gate.size), dtype=np.uint8)
    lib().oracle_glu_fwd(_kind(kind), _dtype(dtype), gate, up, ae, as_, he, m, gate.size)
    return ae, as_, he, m


def glu_bwd(kind, a, up, mask, grad_h):
    """-> (grad_gate, grad_up) (unrounded double)"""
    a = _f64(a); up = _f64(up); g = _f64(grad_h); mask = _u8(mask)
    assert a.size == up.size == g.size and mask.size >= (a.size + 7) // 8
    gg = np.empty_like(a); gu = np.empty_like(a)
    lib().oracle_glu_bwd(_kind(kind), a, up, mask, g, gg, gu, a.size)
    return gg, gu


def pbit_fwd(kind, dtype, x):
    """Precision-bit forward -> (y_exact, y_stored with its lowest bit set to s)"""
    x = _f64(x)
    ye = np.empty_like(x); ys = np.empty_like(x)
    lib().oracle_pbit_fwd(_kind(kind), _dtype(dtype), x, ye, ys, x.size)
    return ye, ys


def pbit_bwd(kind, dtype, y, grad_y):
    """Precision-bit backward -> grad_x (unrounded double); s is read from y's lowest bit"""
    y = _f64(y); g = _f64(grad_y)
    assert y.size == g.size
    gx = np.empty_like(y)
    lib().oracle_pbit_bwd(_kind(kind), _dtype(dtype), y, g, gx, y.size)
    return gx


def sbit_fwd(kind, dtype, x):
    """Sign-bit forward -> (f(x) - C exact, the same rounded to dtype with its sign bit set to s)"""
    x = _f64(x)
    ve = np.empty_like(x); yt = np.empty_like(x)
    lib().oracle_sbit_fwd(_kind(kind), _dtype(dtype), x, ve, yt, x.size)
    return ve, yt


def sbit_decode(kind, dtype, y_tagged):
    """|Y| + C -> (exact, rounded to dtype)"""
    yt = _f64(y_tagged)
    ye = np.empty_like(yt); ys = np.empty_like(yt)
    lib().oracle_sbit_decode(_kind(kind), _dtype(dtype), yt, ye, ys, yt.size)
    return ye, ys


def sbit_bwd(kind, y_tagged, grad_y):
    """Sign-bit backward -> grad_x (unrounded double); s is the sign bit of the saved tensor"""
    yt = _f64(y_tagged); g = _f64(grad_y)
    assert yt.size == g.size
    gx = np.empty_like(yt)
    lib().oracle_sbit_bwd(_kind(kind), yt, g, gx, yt.size)
    return gx


def sbit_linear(kind, dtype, y_tagged, weight, bias=None):
    """The sign-bit layer's consumer: (|Y| + C) W^T (+ bias) -> out [M, N] (unrounded double);
    y_tagged is [M, K], weight [N, K], bias [N] or None"""
    yt = np.ascontiguousarray(y_tagged, dtype=np.float64); w = np.ascontiguousarray(weight, dtype=np.float64)
    (M, K), (N, K2) = yt.shape, w.shape
    assert K == K2
    out = np.empty((M, N))
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float64)
        assert bias.shape == (N,)
    lib().oracle_sbit_linear(_kind(kind), _dtype(dtype), yt.reshape(-1), w.reshape(-1),
                             None if bias is None else bias.ctypes.data, out.reshape(-1), M, N, K)
    return out


def sbit_linear_wgrad(kind, dtype, y_tagged, grad_out):
    """dW = dOut^T (|Y| + C) -> [N, K] (unrounded double); y_tagged is [M, K], grad_out [M, N]"""
    yt = np.ascontiguousarray(y_tagged, dtype=np.float64); g = np.ascontiguousarray(grad_out, dtype=np.float64)
    (M, K), (M2, N) = yt.shape, g.shape
    assert M == M2
    gw = np.empty((N, K))
    lib().oracle_sbit_linear_wgrad(_kind(kind), _dtype(dtype), yt.reshape(-1), g.reshape(-1), gw.reshape(-1), M, N, K)
    return gw


def sbit_linear_dgrad(kind, y_tagged, grad_out, weight):
    """dX = (dOut W) * q(|Y| + C, S) -> [M, K] (unrounded double); y_tagged is [M, K], grad_out [M, N], weight [N, K]"""
    yt = np.ascontiguousarray(y_tagged, dtype=np.float64); g = np.ascontiguousarray(grad_out, dtype=np.float64)
    w = np.ascontiguousarray(weight, dtype=np.float64)
    (M, K), (M2, N), (N2, K2) = yt.shape, g.shape, w.shape
    assert M == M2 and N == N2 and K == K2
    gx = np.empty((M, K))
    lib().oracle_sbit_linear_dgrad(_kind(kind), yt.reshape(-1), g.reshape(-1), w.reshape(-1), gx.reshape(-1), M, N, K)
    return gx


def num_threads():
    return int(lib().oracle_num_threads())
