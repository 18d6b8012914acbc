"""Drop-in PyTorch layers over libinvact (Introduction, Listing 1; Algorithm 1).

    for layer in model.layers:
        layer.act_fn = InvActGELU()

Each layer's autograd function calls the C ABI for both passes and saves the
layer's OUTPUT plus the packed 1-bit mask instead of its input.  The output is
the tensor the next layer saves anyway, so between the two layers one tensor is
kept instead of two.  There is no CPU or eager fallback: tensors must live on
the GPU and be float32 or bfloat16.

Two wirings of the same kernels: the autograd functions below (Python), and the
same functions written in C++ (csrc/invact_torch.cpp -> libinvact_torch.so, torch
operators invact::act / act_pbit / glu), which are used when that library is
built: two Python autograd hops cost more than the two kernels of a 2^25-element
layer take on an MI355X.  INVACT_NN=python selects the Python wiring.
"""
import os

import torch

from . import binding as B

_TORCH_EXT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libinvact_torch.so")
_ops = None
if os.environ.get("INVACT_NN", "") != "python" and os.path.exists(_TORCH_EXT):
    B.lib()                                   # the kernels' library first: the extension links against it
    try:
        torch.ops.load_library(_TORCH_EXT)
        _ops = torch.ops.invact
    except OSError as e:                      # built against another torch: same kernels through the Python wiring
        import warnings
        warnings.warn(f"{_TORCH_EXT} does not load ({e}); using the Python autograd wiring")


def wiring():
    """'c++' if the layers go through libinvact_torch.so, 'python' if through the autograd functions here."""
    return "python" if _ops is None else "c++"


def set_wiring(name):
    """Switch between the two wirings ('c++' needs libinvact_torch.so).  Returns the previous one."""
    global _ops
    previous = wiring()
    if name == "python":
        _ops = None
    elif name == "c++":
        if not os.path.exists(_TORCH_EXT):
            raise RuntimeError(f"{_TORCH_EXT} is missing: build it with `python -m paper_2407_15545_amd.build`")
        B.lib()
        torch.ops.load_library(_TORCH_EXT)
        _ops = torch.ops.invact
    else:
        raise ValueError("wiring must be 'c++' or 'python'")
    return previous


def _dense(t):
    """t as the library wants it: contiguous, and starting on a 16-byte boundary.  A contiguous view into the
    middle of another tensor (t.view(-1)[3:]) is contiguous but need not be aligned: it is copied."""
    t = t.contiguous()
    return t if t.data_ptr() % 16 == 0 else t.clone()


class _InvAct(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, kind):
        y, mask = B.invact_fwd(kind, _dense(x))
        ctx.kind = kind
        ctx.save_for_backward(y, mask)
        return y.view_as(x)

    @staticmethod
    def backward(ctx, grad_y):
        y, mask = ctx.saved_tensors
        return B.invact_bwd(ctx.kind, y, mask, _dense(grad_y)).view_as(grad_y), None


class _InvActPrecisionBit(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, kind):
        y = B.invact_pbit_fwd(kind, _dense(x))
        ctx.kind = kind
        ctx.save_for_backward(y)
        return y.view_as(x)

    @staticmethod
    def backward(ctx, grad_y):
        (y,) = ctx.saved_tensors
        return B.invact_pbit_bwd(ctx.kind, y, _dense(grad_y)).view_as(grad_y), None


class _InvActGLU(torch.autograd.Function):
    @staticmethod
    def forward(ctx, gate, up, kind):
        up = _dense(up)
        act, h, mask = B.geglu_invact_fwd(kind, _dense(gate), up)
        ctx.kind = kind
        ctx.save_for_backward(act, up, mask)
        return h.view_as(gate)

    @staticmethod
    def backward(ctx, grad_h):
        act, up, mask = ctx.saved_tensors
        grad_gate, grad_up = B.geglu_invact_bwd(ctx.kind, act, up, mask, _dense(grad_h))
        return grad_gate.view_as(grad_h), grad_up.view_as(grad_h), None


class _SignBitActLinear(torch.autograd.Function):
    """Activation followed by a linear layer, sign-bit variant (Section 3.3 and its listing): the only
    saved activation is f(x) - min f with the indicator in its sign bit.  In bfloat16, with shapes the fused
    products take (in_features a multiple of 64; for the weight gradient a token count that is a multiple of
    64 and out_features a multiple of 8; for the input gradient out_features a multiple of 64), f(x) is rebuilt
    inside the matrix products and never exists in memory, and the input gradient is multiplied by q inside its
    product; otherwise invact_sbit_decode rebuilds f(x) for a library GEMM and it is dropped again.  The rebuilt
    |Y| + C equals f(x) only to an absolute error of about one ulp at |C| (the stored f - C and the sum live on
    the grid of max(|f|, |C|)): near x = 0 it keeps few of f(x)'s own digits, which in bfloat16 is visible."""

    @staticmethod
    def forward(ctx, x, weight, bias, kind, fused_dgrad=None):
        y_tagged = B.invact_sbit_fwd(kind, _dense(x)).view(-1, weight.shape[1])
        M, K = y_tagged.shape
        w = _dense(weight)
        if x.dtype == torch.bfloat16 and weight.dtype == torch.bfloat16 and K % 64 == 0 and M > 0:
            b = None if bias is None else bias.to(torch.bfloat16).contiguous()
            out = B.invact_sbit_linear_fwd(kind, y_tagged, w, b).view(*x.shape[:-1], weight.shape[0])
        else:
            out = torch.nn.functional.linear(B.invact_sbit_decode(kind, y_tagged.view(-1)).view_as(x), weight, bias)
        ctx.kind, ctx.has_bias, ctx.fused_dgrad = kind, bias is not None, fused_dgrad
        ctx.save_for_backward(y_tagged, weight)
        return out

    @staticmethod
    def backward(ctx, grad_out):
        y_tagged, weight = ctx.saved_tensors
        M, K = y_tagged.shape
        N = weight.shape[0]
        g2 = _dense(grad_out.reshape(-1, N))
        if y_tagged.dtype == torch.bfloat16 and g2.dtype == torch.bfloat16 and M % 64 == 0 and N % 8 == 0 and K % 8 == 0 and M > 0:
            # a narrow layer's weight gradient splits its long sum over the tokens; the workspace for the partial
            # sums comes from torch's allocator and goes back to it
            grad_w = B.invact_sbit_linear_wgrad_ws(ctx.kind, y_tagged, g2).to(weight.dtype)
        else:
            grad_w = g2.t().mm(B.invact_sbit_decode(ctx.kind, y_tagged.view(-1)).view(M, K))
        grad_b = g2.sum(0) if ctx.has_bias else None
        # (dOut W) * q in one kernel: no M x K temporary and one rounding fewer.  Its q is evaluated after the
        # product rather than beside it, so on large inputs it takes 2-11 % longer than the library's GEMM followed
        # by invact_sbit_bwd: by default it is used up to 2^24 elements, where it is the faster route.
        fused = ctx.fused_dgrad if ctx.fused_dgrad is not None else M * K <= 1 << 24
        if fused and y_tagged.dtype == torch.bfloat16 and g2.dtype == torch.bfloat16 and weight.dtype == torch.bfloat16 \
                and N % 64 == 0 and K % 8 == 0 and M > 0:
            grad_x = B.invact_sbit_linear_dgrad(ctx.kind, y_tagged, g2, _dense(weight))
        else:
            grad_x = B.invact_sbit_bwd(ctx.kind, y_tagged.view(-1), _dense(g2.mm(weight)).view(-1))
        grad_x = grad_x.view(*grad_out.shape[:-1], K)
        return grad_x, grad_w, grad_b, None, None


def invact(x, kind="gelu_erf", precision_bit=False):
    """y = f(x) with the inverted-activation backward."""
    if _ops is not None:
        return (_ops.act_pbit if precision_bit else _ops.act)(x, B.KINDS[kind])
    return (_InvActPrecisionBit if precision_bit else _InvAct).apply(x, kind)


def invact_glu(gate, up, kind="silu"):
    """h = f(gate) * up with the inverted-activation backward (SwiGLU for kind='silu', GeGLU for the GELUs)."""
    if _ops is not None:
        return _ops.glu(gate, up, B.KINDS[kind])
    return _InvActGLU.apply(gate, up, kind)


class InvAct(torch.nn.Module):
    def __init__(self, kind, precision_bit=False):
        super().__init__()
        if kind not in B.KINDS:
            raise ValueError(f"kind must be one of {sorted(B.KINDS)}")
        self.kind, self.precision_bit = kind, precision_bit

    def forward(self, x):
        return invact(x, self.kind, self.precision_bit)

    def extra_repr(self):
        return f"kind={self.kind!r}, precision_bit={self.precision_bit}"


class InvActGELU(InvAct):
    """Replacement for torch.nn.GELU (approximate='none' or 'tanh')."""

    def __init__(self, approximate="none", precision_bit=False):
        if approximate not in ("none", "tanh"):
            raise ValueError("approximate must be 'none' or 'tanh'")
        super().__init__("gelu_tanh" if approximate == "tanh" else "gelu_erf", precision_bit)


class InvActSiLU(InvAct):
    """Replacement for torch.nn.SiLU."""

    def __init__(self, precision_bit=False):
        super().__init__("silu", precision_bit)


class InvActGLU(torch.nn.Module):
    """h = f(gate) * up as one fused layer (SwiGLU: kind='silu'; GeGLU: 'gelu_erf' / 'gelu_tanh')."""

    def __init__(self, kind="silu"):
        super().__init__()
        if kind not in B.KINDS:
            raise ValueError(f"kind must be one of {sorted(B.KINDS)}")
        self.kind = kind

    def forward(self, gate, up):
        return invact_glu(gate, up, self.kind)


class SignBitActLinear(torch.nn.Linear):
    """linear(f(x)): an activation and the linear layer after it as ONE layer, the form the sign-bit variant
    needs (the saved tensor is not the activation, so the consumer has to be part of the layer)."""

    def __init__(self, in_features, out_features, bias=True, kind="gelu_erf", device=None, dtype=None,
                 fused_input_gradient=None):
        """fused_input_gradient: True / False forces or forbids the one-kernel input gradient
        (invact_sbit_linear_dgrad); None uses it where it is the faster route."""
        super().__init__(in_features, out_features, bias=bias, device=device, dtype=dtype)
        if kind not in B.KINDS:
            raise ValueError(f"kind must be one of {sorted(B.KINDS)}")
        self.kind, self.fused_input_gradient = kind, fused_input_gradient

    def forward(self, x):
        return _SignBitActLinear.apply(x, self.weight, self.bias, self.kind, self.fused_input_gradient)


def saved_activation_bytes(fn):
    """Bytes of distinct tensors autograd saves while running fn() (the paper's memory metric:
    stored activations only, parameters excluded by the caller passing them as leaves that
    require grad -- they are saved too but are the same in both variants)."""
    seen = {}

    def pack(t):
        if t.device.type == "cuda":
            seen[(t.untyped_storage().data_ptr(), t.storage_offset(), tuple(t.shape))] = t.numel() * t.element_size()
        return t

    with torch.autograd.graph.saved_tensors_hooks(pack, lambda t: t):
        out = fn()
    return sum(seen.values()), out
