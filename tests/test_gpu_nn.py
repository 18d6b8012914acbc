"""The PyTorch layers over the C ABI: gradients against torch's own autograd (up to the
approximation error of q, which the paper only plots), and the saved-activation memory
the method exists for (Introduction; Appendix "Memory Table")."""
import pytest
import torch
import torch.nn.functional as F

import parity as PT
from paper_2407_15545_amd import binding as B
from paper_2407_15545_amd import nn as inv

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["c++", "python"])
def wiring(request):
    """Every test runs through both wirings of the layers (C++ operators and Python autograd functions)."""
    previous = inv.set_wiring(request.param)
    yield request.param
    inv.set_wiring(previous)


REFS = {"gelu_erf": lambda x: F.gelu(x), "gelu_tanh": lambda x: F.gelu(x, approximate="tanh"), "silu": F.silu}


@pytest.mark.parametrize("precision_bit", [False, True])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("kind", ["gelu_erf", "gelu_tanh", "silu"])
def test_layer_matches_torch_autograd(kind, dtype, precision_bit):
    torch.manual_seed(0)
    x = (torch.randn(64, 1000, device="cuda") * 2).to(dtype).requires_grad_()
    g = torch.randn(64, 1000, device="cuda").to(dtype)
    PT.say(f"nn layer {kind} {dtype} precision_bit={precision_bit}")
    y = inv.invact(x, kind, precision_bit)
    (gx,) = torch.autograd.grad(y, x, g)
    xr = x.detach().double().requires_grad_()
    yr = REFS[kind](xr)
    (gr,) = torch.autograd.grad(yr, xr, g.double())
    # wiring check only (ulp-level parity with the oracle is in test_gpu_parity.py / test_gpu_pbit.py)
    eps = 2.0 ** -6 if dtype == torch.bfloat16 else 1e-5
    assert torch.all((y.double() - yr).abs() <= eps * yr.abs() + 1e-9)
    # q approximates f'(x) to a few 1e-2 at worst (GELU just right of the minimum)
    assert torch.all((gx.double() - gr).abs() <= (4e-2 + 4 * eps) * g.double().abs() + 1e-9)


@pytest.mark.parametrize("precision_bit", [False, True])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("kind", ["gelu_erf", "gelu_tanh", "silu"])
def test_layer_is_the_c_abi_bit_for_bit(kind, dtype, precision_bit):
    """The layer adds nothing to the kernels: its output, what it saves and its gradient are bit-identical to
    direct calls of the binding on the same tensors (a wrong kind, or y and x exchanged, cannot hide here)."""
    torch.manual_seed(4)
    x = (torch.randn(37, 1001, device="cuda") * 2).to(dtype).requires_grad_()
    g = torch.randn(37, 1001, device="cuda").to(dtype)
    PT.say(f"nn layer vs binding {kind} {dtype} precision_bit={precision_bit}")
    saved = []
    with torch.autograd.graph.saved_tensors_hooks(lambda t: saved.append(t) or t, lambda t: t):
        y = inv.invact(x, kind, precision_bit)
    (gx,) = torch.autograd.grad(y, x, g)
    same = lambda a, b: a.shape == b.shape and torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))
    flat = x.detach().reshape(-1)
    if precision_bit:
        y_ref = B.invact_pbit_fwd(kind, flat)
        gx_ref = B.invact_pbit_bwd(kind, y_ref, g.reshape(-1))
        assert len(saved) == 1 and same(saved[0].reshape(-1), y_ref)
    else:
        y_ref, m_ref = B.invact_fwd(kind, flat)
        gx_ref = B.invact_bwd(kind, y_ref, m_ref, g.reshape(-1))
        assert len(saved) == 2 and same(saved[0].reshape(-1), y_ref) and same(saved[1], m_ref)
    assert same(y.detach(), y_ref.view_as(x)) and same(gx, gx_ref.view_as(x))


@pytest.mark.parametrize("kind", ["silu", "gelu_erf", "gelu_tanh"])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_glu_layer_is_the_c_abi_bit_for_bit(kind, dtype):
    torch.manual_seed(5)
    gate = torch.randn(33, 515, device="cuda").to(dtype).requires_grad_()
    up = torch.randn(33, 515, device="cuda").to(dtype).requires_grad_()
    gh = torch.randn(33, 515, device="cuda").to(dtype)
    PT.say(f"nn glu vs binding {kind} {dtype}")
    saved = []
    with torch.autograd.graph.saved_tensors_hooks(lambda t: saved.append(t) or t, lambda t: t):
        h = inv.invact_glu(gate, up, kind)
    gg, gu = torch.autograd.grad(h, (gate, up), gh)
    same = lambda a, b: torch.equal(a.contiguous().view(torch.uint8).reshape(-1), b.contiguous().view(torch.uint8).reshape(-1))
    act_ref, h_ref, m_ref = B.geglu_invact_fwd(kind, gate.detach().reshape(-1), up.detach().reshape(-1))
    gg_ref, gu_ref = B.geglu_invact_bwd(kind, act_ref, up.detach().reshape(-1), m_ref, gh.reshape(-1))
    assert len(saved) == 3 and same(saved[0], act_ref) and same(saved[1], up.detach()) and same(saved[2], m_ref)
    assert same(h.detach(), h_ref) and same(gg, gg_ref) and same(gu, gu_ref)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_layers_take_misaligned_contiguous_views(dtype):
    """t.view(-1)[3:] is contiguous but starts 6 or 12 bytes into an allocation: the library wants 16-byte
    alignment, so the layers copy such an input (and such an incoming gradient) instead of raising."""
    torch.manual_seed(6)
    n = 5000
    base = (torch.randn(n + 3, device="cuda") * 2).to(dtype)
    gbase = torch.randn(n + 3, device="cuda").to(dtype)
    x = base[3:].detach().requires_grad_()
    g = gbase[3:]
    assert x.is_contiguous() and x.data_ptr() % 16 != 0 and g.data_ptr() % 16 != 0
    PT.say(f"nn layers on misaligned views {dtype}")
    aligned_x = base[3:].clone().requires_grad_()
    for fn in (lambda t: inv.invact(t, "gelu_erf"), lambda t: inv.invact(t, "silu", True),
               lambda t: inv.invact_glu(t, t.detach() * 0.5, "silu")):
        y = fn(x)
        (gx,) = torch.autograd.grad(y, x, g)
        y2 = fn(aligned_x)
        (gx2,) = torch.autograd.grad(y2, aligned_x, g.clone())
        assert torch.equal(y.detach().view(torch.uint8), y2.detach().view(torch.uint8))
        assert torch.equal(gx.view(torch.uint8), gx2.view(torch.uint8))
    with pytest.raises(B.InvactError):                      # the C ABI itself still refuses the pointer
        B.invact_fwd("silu", x.detach())


@pytest.mark.parametrize("kind", ["silu", "gelu_erf"])
def test_glu_layer_matches_torch_autograd(kind):
    torch.manual_seed(1)
    gate = torch.randn(32, 512, device="cuda", dtype=torch.bfloat16).requires_grad_()
    up = torch.randn(32, 512, device="cuda", dtype=torch.bfloat16).requires_grad_()
    gh = torch.randn(32, 512, device="cuda", dtype=torch.bfloat16)
    PT.say(f"nn glu {kind}")
    h = inv.InvActGLU(kind)(gate, up)
    gg, gu = torch.autograd.grad(h, (gate, up), gh)
    g64, u64 = gate.detach().double().requires_grad_(), up.detach().double().requires_grad_()
    hr = REFS[kind](g64) * u64
    ggr, gur = torch.autograd.grad(hr, (g64, u64), gh.double())
    assert torch.all((h.double() - hr).abs() <= 2.0 ** -6 * hr.abs() + 1e-9)
    assert torch.all((gu.double() - gur).abs() <= 2.0 ** -5 * gur.abs() + 1e-9)
    assert torch.all((gg.double() - ggr).abs() <= 5e-2 * (gh.double() * u64).abs() + 1e-9)


def test_saved_activation_memory_of_a_transformer_mlp_stack():
    """Linear -> act -> Linear blocks (BERT-base MLP shape), bf16: the standard layer keeps the
    activation's input AND output, the inverted one keeps the output and 1/16 of a tensor."""
    torch.manual_seed(2)
    layers, d, tokens = 4, 768, 2048
    w1 = [torch.randn(4 * d, d, device="cuda", dtype=torch.bfloat16, requires_grad=True) for _ in range(layers)]
    w2 = [torch.randn(d, 4 * d, device="cuda", dtype=torch.bfloat16, requires_grad=True) for _ in range(layers)]
    x0 = torch.randn(tokens, d, device="cuda", dtype=torch.bfloat16, requires_grad=True)

    def run(act):
        def fn():
            x = x0
            for a, b in zip(w1, w2):
                x = x + F.linear(act(F.linear(x, a)), b) * 0.01
            return x
        return inv.saved_activation_bytes(fn)[0]

    PT.say("saved-activation memory")
    weights = sum(w.numel() * 2 for w in w1 + w2)
    base = run(F.gelu) - weights
    ours = run(inv.InvActGELU()) - weights
    pbit = run(inv.InvActGELU(precision_bit=True)) - weights
    # per block: x (d) + pre-activation (4d) + activation (4d) -> x + activation + mask (4d/16)
    per_token = tokens * 2
    assert base == layers * per_token * (d + 4 * d + 4 * d)
    assert ours == layers * (per_token * (d + 4 * d) + tokens * 4 * d // 8)
    assert pbit == layers * per_token * (d + 4 * d)
    saving = 1 - ours / base
    PT.say(f"  saved activations: torch {base / 1e6:.1f} MB, InvAct {ours / 1e6:.1f} MB ({-100 * saving:.1f} %), "
        f"precision-bit {pbit / 1e6:.1f} MB ({-100 * (1 - pbit / base):.1f} %)")
    assert 0.40 < saving < 0.45


def test_layers_refuse_cpu_tensors():
    with pytest.raises((ValueError, RuntimeError)):
        inv.InvActSiLU()(torch.randn(8))


def test_block_bench_blocks_match_torch_and_time():
    """The blocks of the block-level timing script: same outputs as with torch's GELU up to the storage
    rounding, gradients up to the approximation error of q, and the timer (eager and graph replay) runs."""
    from paper_2407_15545_amd import block_bench as BB
    torch.manual_seed(0)
    x = torch.randn(256, BB.DIM, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    for cls in (BB.LinearAct, BB.Mlp, BB.GeGlu):
        torch.manual_seed(1)
        ref = cls(torch.nn.GELU()).to(device="cuda", dtype=torch.bfloat16)
        torch.manual_seed(1)
        got = cls(inv.InvActGELU()).to(device="cuda", dtype=torch.bfloat16)
        yr, yg = ref(x), got(x)
        assert torch.allclose(yr.float(), yg.float(), rtol=2e-2, atol=2e-2)
        g = torch.randn_like(yr)
        (gr,) = torch.autograd.grad(yr, x, g)
        (gg,) = torch.autograd.grad(yg, x, g)
        rel = (gr.float() - gg.float()).norm() / gr.float().norm()
        assert rel < 3e-2, (cls.__name__, float(rel))
    torch.manual_seed(1)
    fused = BB.GeGlu(glu=inv.InvActGLU("gelu_erf")).to(device="cuda", dtype=torch.bfloat16)
    assert torch.allclose(fused(x).float(), yg.float(), rtol=2e-2, atol=2e-2)
    xs = torch.randn(1 << 16, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    for graph in (False, True):
        assert BB.time_block(BB.Plain(inv.InvActGELU()), xs, iters=3, groups=2, graph=graph) > 0


@pytest.mark.parametrize("shape, dtype", [((512, 1024), torch.bfloat16),        # both products fused
                                          ((4, 96, 512), torch.bfloat16),        # 3-D input, fused
                                          ((100, 1000), torch.bfloat16),         # shapes the fused products refuse
                                          ((512, 1024), torch.float32)])         # binary32: decode + library GEMM
@pytest.mark.parametrize("kind", ["gelu_erf", "silu"])
def test_sign_bit_act_linear_matches_torch_and_saves_one_tensor(kind, shape, dtype, wiring):
    if wiring != "python":
        pytest.skip("the sign-bit layer has one wiring")
    torch.manual_seed(3)
    d_in, d_out = shape[-1], 256
    x = torch.randn(*shape, device="cuda", dtype=dtype, requires_grad=True)
    layer = inv.SignBitActLinear(d_in, d_out, kind=kind, device="cuda", dtype=dtype)
    PT.say(f"nn sign-bit act + linear {kind} {shape} {dtype}")
    out = layer(x)
    ref = F.linear(REFS[kind](x), layer.weight, layer.bias)
    assert torch.allclose(out.float(), ref.float(), rtol=3e-2, atol=3e-2)
    g = torch.randn_like(out)
    gx, gw, gb = torch.autograd.grad(out, (x, layer.weight, layer.bias), g)
    rx, rw, rb = torch.autograd.grad(ref, (x, layer.weight, layer.bias), g)
    for a, b in ((gx, rx), (gw, rw), (gb, rb)):
        assert (a.float() - b.float()).norm() / b.float().norm() < 3e-2
    for fused in (True, False):                 # the input gradient in one kernel, and as library GEMM + invact_sbit_bwd
        layer.fused_input_gradient = fused
        gx2, = torch.autograd.grad(layer(x), (x,), g)
        assert (gx2.float() - rx.float()).norm() / rx.float().norm() < 3e-2
    layer.fused_input_gradient = None
    # saved: the tagged tensor (same size as x) and the weight; torch keeps x, f(x) and the weight
    ours = inv.saved_activation_bytes(lambda: layer(x))[0]
    base = inv.saved_activation_bytes(lambda: F.linear(REFS[kind](x), layer.weight, layer.bias))[0]
    weight_bytes = layer.weight.numel() * x.element_size()
    assert ours - weight_bytes == x.numel() * x.element_size()
    assert base - weight_bytes == 2 * x.numel() * x.element_size()


def test_whole_model_memory_saving_matches_the_papers_table(wiring):
    """ViT-base built from its architecture parameters (random weights): swapping the 12 GELU modules for InvAct
    layers cuts the stored activations by the 23.8 % the paper's memory table prints, to within a point."""
    if wiring != "c++":
        pytest.skip("one wiring is enough for a count of saved bytes")
    pytest.importorskip("transformers")
    from paper_2407_15545_amd import memory_table as M
    make, inputs = M.build("vit", "sdpa")
    torch.manual_seed(0)
    model = make().to(device="cuda", dtype=torch.float32).train()
    batch = inputs("cuda", torch.float32)
    PT.say("memory table: ViT-base fp32")
    base = M.saved_bytes(model, batch)
    assert M.swap_activations(model) == 12
    ours = M.saved_bytes(model, batch)
    saving = 100 * (ours / base - 1)
    assert -24.8 <= saving <= -22.8, saving
    # the swapped model still runs backward
    out = model(**batch).last_hidden_state
    out.float().square().mean().backward()
    assert all(p.grad is None or torch.isfinite(p.grad).all() for p in model.parameters())
