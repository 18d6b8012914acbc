"""Saved-activation memory of whole transformer models with and without the InvAct layers
(Introduction, the table next to Listing 1; Appendix "Memory Table").

    python -m paper_2407_15545_amd.memory_table [--models bert ast vit clip] [--dtypes fp32 bf16] [--attn sdpa eager]

The paper's figure is "how much less memory is used for stored activations" for one forward pass of
four public models.  Stored activations depend on the architecture and the input shape only, not on
the weights, so the models are built here from their published architecture parameters with random
weights (nothing is downloaded) and fed random inputs of the shapes the appendix names:

  bert   BERT-base (12 x 768, MLP 3072, GELU), 1024 tokens
  ast    Audio Spectrogram Transformer (12 x 768, MLP 3072, GELU), 1024 x 128 spectrogram
  vit    ViT-base, patch 16, 224 x 224 image (12 x 768, MLP 3072, GELU)
  clip   CLIP ViT-L/14: text tower 12 x 768 / 77 tokens, vision tower 24 x 1024 / 224 x 224 image; its
         activation x * sigmoid(1.702 x) is SiLU with a rescaled argument and goes through the SiLU kernels
  llama  (not in the paper's table, not run by default) Llama-3.1-8B shape, 512 tokens, bf16: a gated MLP

Every tensor autograd saves during the forward (training mode) is counted once by its storage; parameters
are left out, as in the paper.  The activation modules of the models are then swapped for the InvAct
layers (the usage the paper's Listing 1 shows) and the count is repeated.
"""
import argparse

import torch

from . import binding as B
from . import nn as invact_nn


class _QuickGELU(torch.autograd.Function):
    """x * sigmoid(a x) = silu(a x) / a with a = 1.702.  The layer must save the very tensor it returns (the next
    layer saves that one anyway), so the rescaling is done in place on the forward's output and undone on a
    temporary in the backward: d/dx [silu(a x) / a] = silu'(a x) = q(silu(a x), s)."""
    A = 1.702

    @staticmethod
    def forward(ctx, x):
        y, mask = B.invact_fwd("silu", (x * _QuickGELU.A).contiguous())
        y.mul_(1.0 / _QuickGELU.A)
        ctx.save_for_backward(y, mask)
        return y.view_as(x)

    @staticmethod
    def backward(ctx, grad_y):
        y, mask = ctx.saved_tensors
        return B.invact_bwd("silu", y * _QuickGELU.A, mask, grad_y.contiguous()).view_as(grad_y)


class _FusedQuickGELU(torch.autograd.Function):
    """x * sigmoid(1.702 x) as ONE layer that saves its input, the way torch's GELU and SiLU modules do.
    (The model's own module composes it from a multiplication and a sigmoid, each of which saves a
    tensor.)  Used as a second baseline for CLIP."""

    @staticmethod
    def forward(ctx, x):
        ctx.save_for_backward(x)
        return x * torch.sigmoid(1.702 * x)

    @staticmethod
    def backward(ctx, g):
        (x,) = ctx.saved_tensors
        s = torch.sigmoid(1.702 * x)
        return g * (s + 1.702 * x * s * (1 - s))


class FusedQuickGELU(torch.nn.Module):
    def forward(self, x):
        return _FusedQuickGELU.apply(x)


class InvActQuickGELU(torch.nn.Module):
    def forward(self, x):
        return _QuickGELU.apply(x)


def build(name, attn):
    import transformers as T
    if name == "bert":
        cfg = T.BertConfig(max_position_embeddings=1024)
        make = lambda: T.BertModel(cfg, add_pooling_layer=False)
        inputs = lambda dev, dt: {"input_ids": torch.randint(0, cfg.vocab_size, (1, 1024), device=dev)}
    elif name == "ast":
        cfg = T.ASTConfig()
        make = lambda: T.ASTModel(cfg)
        inputs = lambda dev, dt: {"input_values": torch.randn(1, 1024, 128, device=dev, dtype=dt)}
    elif name == "vit":
        cfg = T.ViTConfig()
        make = lambda: T.ViTModel(cfg, add_pooling_layer=False)
        inputs = lambda dev, dt: {"pixel_values": torch.randn(1, 3, 224, 224, device=dev, dtype=dt)}
    elif name == "clip":
        cfg = T.CLIPConfig(
            text_config=dict(hidden_size=768, intermediate_size=3072, num_hidden_layers=12, num_attention_heads=12,
                             max_position_embeddings=77, vocab_size=49408, projection_dim=768),
            vision_config=dict(hidden_size=1024, intermediate_size=4096, num_hidden_layers=24, num_attention_heads=16,
                               image_size=224, patch_size=14, projection_dim=768),
            projection_dim=768)
        make = lambda: T.CLIPModel(cfg)
        inputs = lambda dev, dt: {"input_ids": torch.randint(0, 49407, (1, 77), device=dev),
                                  "pixel_values": torch.randn(1, 3, 224, 224, device=dev, dtype=dt)}
    elif name == "llama":               # not in the paper's table: a gated (SwiGLU) model, 512 tokens
        cfg = T.LlamaConfig(vocab_size=128256, hidden_size=4096, intermediate_size=14336, num_hidden_layers=32,
                            num_attention_heads=32, num_key_value_heads=8, max_position_embeddings=8192,
                            rope_theta=500000.0)

        def make():
            with torch.device("cuda"):
                return T.LlamaModel(cfg)
        inputs = lambda dev, dt: {"input_ids": torch.randint(0, cfg.vocab_size, (1, 512), device=dev)}
    else:
        raise ValueError(name)
    for c in (cfg, getattr(cfg, "text_config", None), getattr(cfg, "vision_config", None)):
        if c is not None:
            c._attn_implementation = attn
    return make, inputs


def fuse_quick_gelu(model):
    """Replace the composite x * sigmoid(1.702 x) modules by the single-layer baseline.  Returns how many."""
    from transformers import activations as A
    n = 0
    for module in model.modules():
        for attr in ("intermediate_act_fn", "activation_fn", "act_fn"):
            if isinstance(getattr(module, attr, None), A.QuickGELUActivation):
                setattr(module, attr, FusedQuickGELU())
                n += 1
    return n


def swap_activations(model, precision_bit=False):
    """Replace the models' activation modules by InvAct layers.  Returns how many were replaced."""
    from transformers import activations as A
    tanh_forms = tuple(c for c in (getattr(A, k, None) for k in ("NewGELUActivation", "GELUTanh", "PytorchGELUTanh")) if c)
    silu_forms = tuple(c for c in (getattr(A, "SiLUActivation", None), torch.nn.SiLU) if c)
    n = 0
    for module in model.modules():
        for attr in ("intermediate_act_fn", "activation_fn", "act_fn"):
            fn = getattr(module, attr, None)
            if isinstance(fn, A.GELUActivation):
                setattr(module, attr, invact_nn.InvActGELU(precision_bit=precision_bit))
            elif isinstance(fn, (A.QuickGELUActivation, FusedQuickGELU)):
                setattr(module, attr, InvActQuickGELU())
            elif isinstance(fn, silu_forms):
                setattr(module, attr, invact_nn.InvActSiLU(precision_bit=precision_bit))
            elif isinstance(fn, tanh_forms):
                setattr(module, attr, invact_nn.InvActGELU(approximate="tanh", precision_bit=precision_bit))
            else:
                continue
            n += 1
    return n


def saved_bytes(model, batch):
    """Bytes of the distinct storages autograd saves for one forward pass, parameters excluded."""
    params = {p.untyped_storage().data_ptr() for p in model.parameters()}
    seen = {}

    def pack(t):
        ptr = t.untyped_storage().data_ptr()
        if t.device.type == "cuda" and ptr not in params:
            seen[ptr] = max(seen.get(ptr, 0), t.untyped_storage().nbytes())
        return t

    with torch.autograd.graph.saved_tensors_hooks(pack, lambda t: t):
        out = model(**batch)
    del out
    return sum(seen.values())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--models", nargs="+", default=["bert", "ast", "vit", "clip"])
    ap.add_argument("--dtypes", nargs="+", default=["fp32", "bf16"])
    ap.add_argument("--attn", nargs="+", default=["sdpa", "eager"])
    args = ap.parse_args()
    torch.cuda.set_device(0)
    print(f"{'model':6s} {'dtype':5s} {'attention':9s} {'torch MB':>10s} {'InvAct MB':>10s} {'saving':>8s}  activations replaced", flush=True)
    for name in args.models:
        for dt in args.dtypes:
            td = {"fp32": torch.float32, "bf16": torch.bfloat16}[dt]
            for attn in args.attn:
                make, inputs = build(name, attn)
                torch.manual_seed(0)
                if name == "llama":     # 8 B parameters: created on the GPU, directly in the storage dtype
                    if dt == "fp32":
                        continue
                    torch.set_default_dtype(td)
                try:
                    model = make().to(device="cuda", dtype=td).train()
                finally:
                    torch.set_default_dtype(torch.float32)
                batch = inputs("cuda", td)
                base = saved_bytes(model, batch)
                fused = saved_bytes(model, batch) if fuse_quick_gelu(model) else None
                replaced = swap_activations(model)
                ours = saved_bytes(model, batch)
                print(f"{name:6s} {dt:5s} {attn:9s} {base / 1e6:10.1f} {ours / 1e6:10.1f} {100 * (ours / base - 1):+7.1f}%  {replaced}", flush=True)
                if name == "llama":     # the gated MLP as one fused layer: down(glu(gate(x), up(x)))
                    glu = invact_nn.InvActGLU("silu")
                    for layer in model.layers:
                        mlp = layer.mlp
                        mlp.forward = (lambda x, m=mlp: m.down_proj(glu(m.gate_proj(x), m.up_proj(x))))
                    both = saved_bytes(model, batch)
                    print(f"{'':6s} {'':5s} {'':9s} {base / 1e6:10.1f} {both / 1e6:10.1f} {100 * (both / base - 1):+7.1f}%  "
                          f"with the fused SwiGLU layer", flush=True)
                if fused is not None:
                    print(f"{'':6s} {'':5s} {'':9s} {fused / 1e6:10.1f} {ours / 1e6:10.1f} {100 * (ours / fused - 1):+7.1f}%  "
                          f"against the activation as one layer that saves its input", flush=True)
                del model, batch
                torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
