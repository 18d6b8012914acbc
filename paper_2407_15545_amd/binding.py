"""ctypes binding of libinvact.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch supplies
device memory (tensors) and streams, nothing else; there is no fallback: if the
library is missing, loading it raises.
"""
import ctypes
import functools
import os

import torch

KINDS = {"gelu_tanh": 0, "gelu_erf": 1, "silu": 2}
DTYPES = {torch.float32: 0, torch.bfloat16: 1}
DTYPE_NAMES = {"fp32": torch.float32, "bf16": torch.bfloat16}

# INVACT_LIB selects another build of the same library (used to compare build variants)
_LIB_PATH = os.environ.get("INVACT_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libinvact.so")
_lib = None

_vp, _sz, _int = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
_PROTOTYPES = {
    "invact_mask_bytes": (_sz, [_sz]),
    "invact_strerror": (ctypes.c_char_p, [_int]),
    "invact_set_blocks_per_cu": (_int, [_int]),
    "invact_set_resident_blocks": (_int, [_int]),
    "invact_set_linear_tile": (_int, [_int]),
    "invact_fwd": (_int, [_int, _int, _vp, _vp, _vp, _sz, _vp]),
    "invact_bwd": (_int, [_int, _int, _vp, _vp, _vp, _vp, _sz, _vp]),
    "geglu_invact_fwd": (_int, [_int, _int, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "geglu_invact_bwd": (_int, [_int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "invact_pbit_fwd": (_int, [_int, _int, _vp, _vp, _sz, _vp]),
    "invact_pbit_bwd": (_int, [_int, _int, _vp, _vp, _vp, _sz, _vp]),
    "invact_sbit_fwd": (_int, [_int, _int, _vp, _vp, _sz, _vp]),
    "invact_sbit_decode": (_int, [_int, _int, _vp, _vp, _sz, _vp]),
    "invact_sbit_bwd": (_int, [_int, _int, _vp, _vp, _vp, _sz, _vp]),
    "invact_sbit_linear_fwd": (_int, [_int, _int, _vp, _vp, _vp, _vp, _sz, _sz, _sz, _vp]),
    "invact_sbit_linear_wgrad": (_int, [_int, _int, _vp, _vp, _vp, _sz, _sz, _sz, _vp]),
    "invact_sbit_linear_dgrad": (_int, [_int, _int, _vp, _vp, _vp, _vp, _sz, _sz, _sz, _vp]),
    "invact_sbit_linear_wgrad_workspace": (_sz, [_sz, _sz, _sz]),
    "invact_sbit_linear_wgrad_ws": (_int, [_int, _int, _vp, _vp, _vp, _sz, _sz, _sz, _vp, _sz, _vp]),
    "invact_sbit_linear_wgrad_static": (_int, [_int, _int, _vp, _vp, _vp, _sz, _sz, _sz, _vp]),
    "invact_set_linear_splits": (_int, [_int]),
    "swiglu_invact_fwd": (_int, [_int, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "swiglu_invact_bwd": (_int, [_int, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
}


class InvactError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"libinvact: {message} (status {status})")
        self.status = status


def lib():
    """The loaded library with prototypes declared (raises if it is not built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2407_15545_amd.build` "
                "(there is no fallback implementation)")
        handle = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _PROTOTYPES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def strerror(status):
    return lib().invact_strerror(status).decode()


def _check(status):
    if status != 0:
        raise InvactError(status, strerror(status))


def _kind(kind):
    return KINDS[kind] if isinstance(kind, str) else int(kind)


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


class _on_device:
    """Makes the tensors' device current for the call; free when it already is."""
    __slots__ = ("index", "prev")

    def __init__(self, device):
        self.index = device.index

    def __enter__(self):
        self.prev = torch.cuda.current_device()
        if self.prev != self.index:
            torch.cuda.set_device(self.index)

    def __exit__(self, *exc):
        if self.prev != self.index:
            torch.cuda.set_device(self.prev)
        return False


def _tensors(*ts):
    first = ts[0]
    for t in ts:
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("tensors must be contiguous CUDA tensors")
        if t.dtype != first.dtype or t.numel() != first.numel() or t.device != first.device:
            raise ValueError("tensors of one call must share dtype, element count and device")
    if first.dtype not in DTYPES:
        raise ValueError(f"unsupported dtype {first.dtype}")
    return DTYPES[first.dtype], first.numel()


def _mask_arg(mask, n, like):
    nbytes = mask_bytes(n)
    if mask is None:
        return torch.empty(nbytes, dtype=torch.uint8, device=like.device)
    if mask.dtype != torch.uint8 or mask.numel() < nbytes or not mask.is_contiguous() or mask.device != like.device:
        raise ValueError(f"mask must be a contiguous uint8 tensor of >= {nbytes} bytes on the same device")
    return mask


@functools.lru_cache(maxsize=256)
def mask_bytes(n):
    return int(lib().invact_mask_bytes(n))


def set_blocks_per_cu(v):
    return int(lib().invact_set_blocks_per_cu(int(v)))


def set_resident_blocks(v):
    return int(lib().invact_set_resident_blocks(int(v)))


def invact_fwd(kind, x, y=None, mask=None, stream=None):
    """y = f(x) and the packed branch mask.  Returns (y, mask)."""
    y = torch.empty_like(x) if y is None else y
    dt, n = _tensors(x, y)
    mask = _mask_arg(mask, n, x)
    with _on_device(x.device):
        _check(lib().invact_fwd(_kind(kind), dt, x.data_ptr(), y.data_ptr(), mask.data_ptr(), n, _stream(stream)))
    return y, mask


def invact_bwd(kind, y, mask, grad_y, grad_x=None, stream=None):
    """grad_x = grad_y * q(y, mask).  Returns grad_x."""
    grad_x = torch.empty_like(grad_y) if grad_x is None else grad_x
    dt, n = _tensors(y, grad_y, grad_x)
    mask = _mask_arg(mask, n, y)
    with _on_device(y.device):
        _check(lib().invact_bwd(_kind(kind), dt, y.data_ptr(), mask.data_ptr(), grad_y.data_ptr(),
                                grad_x.data_ptr(), n, _stream(stream)))
    return grad_x


def geglu_invact_fwd(kind, gate, up, act=None, h=None, mask=None, stream=None):
    """act = f(gate), h = f(gate) * up and the mask.  Returns (act, h, mask)."""
    act = torch.empty_like(gate) if act is None else act
    h = torch.empty_like(gate) if h is None else h
    dt, n = _tensors(gate, up, act, h)
    mask = _mask_arg(mask, n, gate)
    with _on_device(gate.device):
        _check(lib().geglu_invact_fwd(_kind(kind), dt, gate.data_ptr(), up.data_ptr(), act.data_ptr(),
                                      h.data_ptr(), mask.data_ptr(), n, _stream(stream)))
    return act, h, mask


def geglu_invact_bwd(kind, act, up, mask, grad_h, grad_gate=None, grad_up=None, stream=None):
    """grad_up = grad_h * act, grad_gate = grad_h * up * q(act, mask).  Returns (grad_gate, grad_up)."""
    grad_gate = torch.empty_like(act) if grad_gate is None else grad_gate
    grad_up = torch.empty_like(act) if grad_up is None else grad_up
    dt, n = _tensors(act, up, grad_h, grad_gate, grad_up)
    mask = _mask_arg(mask, n, act)
    with _on_device(act.device):
        _check(lib().geglu_invact_bwd(_kind(kind), dt, act.data_ptr(), up.data_ptr(), mask.data_ptr(),
                                      grad_h.data_ptr(), grad_gate.data_ptr(), grad_up.data_ptr(), n,
                                      _stream(stream)))
    return grad_gate, grad_up


def invact_pbit_fwd(kind, x, y=None, stream=None):
    """Precision-bit forward: y = f(x) with the indicator in y's lowest bit.  Returns y."""
    y = torch.empty_like(x) if y is None else y
    dt, n = _tensors(x, y)
    with _on_device(x.device):
        _check(lib().invact_pbit_fwd(_kind(kind), dt, x.data_ptr(), y.data_ptr(), n, _stream(stream)))
    return y


def invact_pbit_bwd(kind, y, grad_y, grad_x=None, stream=None):
    """Precision-bit backward: grad_x = grad_y * q(y, bit 0 of y).  Returns grad_x."""
    grad_x = torch.empty_like(grad_y) if grad_x is None else grad_x
    dt, n = _tensors(y, grad_y, grad_x)
    with _on_device(y.device):
        _check(lib().invact_pbit_bwd(_kind(kind), dt, y.data_ptr(), grad_y.data_ptr(), grad_x.data_ptr(), n,
                                     _stream(stream)))
    return grad_x


def invact_sbit_fwd(kind, x, y_tagged=None, stream=None):
    """Sign-bit forward: f(x) - min f with the indicator in the sign bit.  Returns the tensor to save."""
    y_tagged = torch.empty_like(x) if y_tagged is None else y_tagged
    dt, n = _tensors(x, y_tagged)
    with _on_device(x.device):
        _check(lib().invact_sbit_fwd(_kind(kind), dt, x.data_ptr(), y_tagged.data_ptr(), n, _stream(stream)))
    return y_tagged


def invact_sbit_decode(kind, y_tagged, y=None, stream=None):
    """|y_tagged| + min f: the activation, rebuilt from the saved tensor.  Returns y."""
    y = torch.empty_like(y_tagged) if y is None else y
    dt, n = _tensors(y_tagged, y)
    with _on_device(y.device):
        _check(lib().invact_sbit_decode(_kind(kind), dt, y_tagged.data_ptr(), y.data_ptr(), n, _stream(stream)))
    return y


def invact_sbit_bwd(kind, y_tagged, grad_y, grad_x=None, stream=None):
    """Sign-bit backward: grad_x = grad_y * q(|y_tagged| + min f, sign bit).  Returns grad_x."""
    grad_x = torch.empty_like(grad_y) if grad_x is None else grad_x
    dt, n = _tensors(y_tagged, grad_y, grad_x)
    with _on_device(y_tagged.device):
        _check(lib().invact_sbit_bwd(_kind(kind), dt, y_tagged.data_ptr(), grad_y.data_ptr(), grad_x.data_ptr(), n,
                                     _stream(stream)))
    return grad_x


def swiglu_invact_fwd(gate, up, act=None, h=None, mask=None, stream=None):
    act = torch.empty_like(gate) if act is None else act
    h = torch.empty_like(gate) if h is None else h
    dt, n = _tensors(gate, up, act, h)
    mask = _mask_arg(mask, n, gate)
    with _on_device(gate.device):
        _check(lib().swiglu_invact_fwd(dt, gate.data_ptr(), up.data_ptr(), act.data_ptr(), h.data_ptr(),
                                       mask.data_ptr(), n, _stream(stream)))
    return act, h, mask


def swiglu_invact_bwd(act, up, mask, grad_h, grad_gate=None, grad_up=None, stream=None):
    grad_gate = torch.empty_like(act) if grad_gate is None else grad_gate
    grad_up = torch.empty_like(act) if grad_up is None else grad_up
    dt, n = _tensors(act, up, grad_h, grad_gate, grad_up)
    mask = _mask_arg(mask, n, act)
    with _on_device(act.device):
        _check(lib().swiglu_invact_bwd(dt, act.data_ptr(), up.data_ptr(), mask.data_ptr(), grad_h.data_ptr(),
                                       grad_gate.data_ptr(), grad_up.data_ptr(), n, _stream(stream)))
    return grad_gate, grad_up


def set_linear_tile(t):
    """Tile of the fused sign-bit products: 4 (256 x 256), 3 or 2 (128 x 128 with 8 or 4 wavefronts), or 0 (chosen by the output's size)."""
    if lib().invact_set_linear_tile(int(t)) < 0:
        raise ValueError("tile must be 0, 2, 3 or 4")


def _matrices(*ts):
    """dtype code and device of 2-D dense tensors that one call multiplies."""
    first = ts[0]
    for t in ts:
        if not (t.is_cuda and t.is_contiguous() and t.dim() == 2):
            raise ValueError("matrices must be contiguous 2-D CUDA tensors")
        if t.dtype != first.dtype or t.device != first.device:
            raise ValueError("matrices of one call must share dtype and device")
    if first.dtype not in DTYPES:
        raise ValueError(f"unsupported dtype {first.dtype}")
    return DTYPES[first.dtype]


def invact_sbit_linear_fwd(kind, y_tagged, weight, bias=None, out=None, stream=None):
    """out = (|y_tagged| + C) weight^T (+ bias): y_tagged [M, K], weight [N, K], bias [N] or None.  Returns out [M, N]."""
    (M, K), (N, K2) = y_tagged.shape, weight.shape
    if K != K2 or (bias is not None and (bias.shape != (N,) or bias.dtype != weight.dtype or not bias.is_contiguous())):
        raise ValueError("weight must be [N, K] and bias a contiguous [N] of the same dtype")
    out = torch.empty((M, N), dtype=y_tagged.dtype, device=y_tagged.device) if out is None else out
    dt = _matrices(y_tagged, weight, out)
    if out.shape != (M, N):
        raise ValueError("out must be [M, N]")
    with _on_device(y_tagged.device):
        _check(lib().invact_sbit_linear_fwd(_kind(kind), dt, y_tagged.data_ptr(), weight.data_ptr(),
                                            None if bias is None else bias.data_ptr(), out.data_ptr(), M, N, K,
                                            _stream(stream)))
    return out


def set_linear_splits(splits):
    """Parts the contraction of invact_sbit_linear_wgrad_ws is split into: 1..64, or 0 (chosen by the shape)."""
    if lib().invact_set_linear_splits(int(splits)) < 0:
        raise ValueError("splits must be in 0..64")


def sbit_linear_wgrad_workspace(M, N, K):
    """Bytes of workspace invact_sbit_linear_wgrad_ws needs for this shape (0: it does not split the contraction)."""
    return lib().invact_sbit_linear_wgrad_workspace(M, N, K)


def _wgrad_args(y_tagged, grad_out, grad_weight):
    (M, K), (M2, N) = y_tagged.shape, grad_out.shape
    if M != M2:
        raise ValueError("y_tagged and grad_out must have the same number of rows")
    if grad_weight is None:
        grad_weight = torch.empty((N, K), dtype=y_tagged.dtype, device=y_tagged.device)
    dt = _matrices(y_tagged, grad_out, grad_weight)
    if grad_weight.shape != (N, K):
        raise ValueError("grad_weight must be [N, K]")
    return dt, M, N, K, grad_weight


def invact_sbit_linear_wgrad(kind, y_tagged, grad_out, grad_weight=None, stream=None):
    """grad_weight = grad_out^T (|y_tagged| + C): y_tagged [M, K], grad_out [M, N].  Returns grad_weight [N, K]."""
    dt, M, N, K, grad_weight = _wgrad_args(y_tagged, grad_out, grad_weight)
    with _on_device(y_tagged.device):
        _check(lib().invact_sbit_linear_wgrad(_kind(kind), dt, y_tagged.data_ptr(), grad_out.data_ptr(),
                                              grad_weight.data_ptr(), M, N, K, _stream(stream)))
    return grad_weight


def invact_sbit_linear_wgrad_ws(kind, y_tagged, grad_out, grad_weight=None, workspace=None, stream=None):
    """The same product, allowed to split its contraction through `workspace` (a contiguous uint8 tensor of at least
    sbit_linear_wgrad_workspace(M, N, K) bytes on the same device; None: one is taken from torch's allocator)."""
    dt, M, N, K, grad_weight = _wgrad_args(y_tagged, grad_out, grad_weight)
    if workspace is None:
        nbytes = sbit_linear_wgrad_workspace(M, N, K)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=y_tagged.device) if nbytes else None
    elif workspace.dtype != torch.uint8 or not workspace.is_contiguous() or workspace.device != y_tagged.device:
        raise ValueError("workspace must be a contiguous uint8 tensor on the same device")
    with _on_device(y_tagged.device):
        _check(lib().invact_sbit_linear_wgrad_ws(_kind(kind), dt, y_tagged.data_ptr(), grad_out.data_ptr(),
                                                 grad_weight.data_ptr(), M, N, K,
                                                 None if workspace is None else workspace.data_ptr(),
                                                 0 if workspace is None else workspace.numel(), _stream(stream)))
    return grad_weight


def invact_sbit_linear_wgrad_static(kind, y_tagged, grad_out, grad_weight=None, stream=None):
    """The same product with its partial sums in the library's own per-GPU array: the call allocates nothing
    (pass grad_weight), and calls that overlap on one GPU race."""
    dt, M, N, K, grad_weight = _wgrad_args(y_tagged, grad_out, grad_weight)
    with _on_device(y_tagged.device):
        _check(lib().invact_sbit_linear_wgrad_static(_kind(kind), dt, y_tagged.data_ptr(), grad_out.data_ptr(),
                                                     grad_weight.data_ptr(), M, N, K, _stream(stream)))
    return grad_weight


def invact_sbit_linear_dgrad(kind, y_tagged, grad_out, weight, grad_x=None, stream=None):
    """grad_x = (grad_out weight) * q(|y_tagged| + C, sign): y_tagged [M, K], grad_out [M, N], weight [N, K].
    Returns grad_x [M, K]."""
    (M, K), (M2, N), (N2, K2) = y_tagged.shape, grad_out.shape, weight.shape
    if M != M2 or N != N2 or K != K2:
        raise ValueError("shapes must be y_tagged [M, K], grad_out [M, N], weight [N, K]")
    grad_x = torch.empty_like(y_tagged) if grad_x is None else grad_x
    dt = _matrices(y_tagged, grad_out, weight, grad_x)
    if grad_x.shape != (M, K):
        raise ValueError("grad_x must be [M, K]")
    with _on_device(y_tagged.device):
        _check(lib().invact_sbit_linear_dgrad(_kind(kind), dt, y_tagged.data_ptr(), grad_out.data_ptr(), weight.data_ptr(),
                                              grad_x.data_ptr(), M, N, K, _stream(stream)))
    return grad_x
