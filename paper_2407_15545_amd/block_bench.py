"""Block-level timing of the drop-in layers (Section 4.1, Table 1, rows 1-4; set-ups of the appendix).

    python -m paper_2407_15545_amd.block_bench [--dtypes bf16 fp32] [--iters 20]

For each architecture block the forward + backward time of one training step
is measured with torch's activation, with the InvAct layer and with the
precision-bit InvAct layer in its place (the variants take turns, group by group):

  plain        the nonlinearity alone on 2^25 elements (the paper's size), eagerly and replayed from a
               HIP graph (an MI355X needs ~60 us for this size, about what the Python call path of
               one step costs, so the eager figure measures the host), and on 2^28 elements
  linear+act   Linear(2^10 -> 2^10) + nonlinearity, batch 2^15
  mlp          Linear(2^10 -> 4*2^10) + nonlinearity + Linear(4*2^10 -> 2^10), batch 2^15; in bfloat16 also
               with the sign-bit variant, whose activation and second linear layer are one layer with its own
               products (Section 3.3)
  geglu        act(Linear(2^10 -> 4*2^10)) * Linear(2^10 -> 4*2^10), batch 2^15; for InvAct
               also with the fused gated kernel (one launch for activation and product)

  bert         BERT-base with its masked-LM head, batch 64 x 1024 tokens (Table 1, row 5)
  llama        Llama-3.1-8B-shaped causal LM, batch 1 x 512 tokens (row 6)

The GEMMs are torch's (hipBLASLt / rocBLAS); only the activation differs between
the columns.  Inputs and weights are seeded random numbers: the table is about
time, and the time of these kernels does not depend on the values.  The two
whole models are built from their architecture parameters (nothing is
downloaded); a step is forward + loss + backward, without an optimizer.
"""
import argparse
import statistics

import torch

from . import nn as invact_nn

BATCH, DIM = 1 << 15, 1 << 10


class Plain(torch.nn.Module):
    def __init__(self, act):
        super().__init__()
        self.act = act

    def forward(self, x):
        return self.act(x)


class LinearAct(torch.nn.Module):
    def __init__(self, act):
        super().__init__()
        self.fc = torch.nn.Linear(DIM, DIM)
        self.act = act

    def forward(self, x):
        return self.act(self.fc(x))


class Mlp(torch.nn.Module):
    def __init__(self, act):
        super().__init__()
        self.fc1 = torch.nn.Linear(DIM, 4 * DIM)
        self.act = act
        self.fc2 = torch.nn.Linear(4 * DIM, DIM)

    def forward(self, x):
        return self.fc2(self.act(self.fc1(x)))


class MlpSignBit(torch.nn.Module):
    """The same block with the sign-bit variant (Section 3.3): activation and second linear layer are one layer,
    whose two products rebuild the activation from the saved f(x) - min f while they load it."""

    def __init__(self, kind):
        super().__init__()
        self.fc1 = torch.nn.Linear(DIM, 4 * DIM)
        self.fc2 = invact_nn.SignBitActLinear(4 * DIM, DIM, kind=kind)

    def forward(self, x):
        return self.fc2(self.fc1(x))


class GeGlu(torch.nn.Module):
    """act(x W_gate) * (x W_up); `glu`, if given, computes activation and product in one call."""

    def __init__(self, act=None, glu=None):
        super().__init__()
        self.gate = torch.nn.Linear(DIM, 4 * DIM)
        self.up = torch.nn.Linear(DIM, 4 * DIM)
        self.act, self.glu = act, glu

    def forward(self, x):
        if self.glu is not None:
            return self.glu(self.gate(x), self.up(x))
        return self.act(self.gate(x)) * self.up(x)


def prepare(module, x, graph=False):
    """A callable that runs one forward + backward step of `module` (graph=True: replays a HIP graph of it)."""
    def step():
        y = module(x)
        y.backward(grad)
        x.grad = None
        for p in module.parameters():
            p.grad = None
    with torch.no_grad():
        grad = torch.randn_like(module(x))
    if graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        captured = torch.cuda.CUDAGraph()
        with torch.cuda.graph(captured):
            y = module(x)
            y.backward(grad)
        step = captured.replay
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    return step


def time_steps(steps, iters, groups=5):
    """Median over groups of the mean time (ms) of `iters` consecutive calls, for every entry of the dict
    `steps`; the entries take turns within each group, so that clock drift hits all of them alike."""
    times = {k: [] for k in steps}
    for _ in range(groups):
        for k, step in steps.items():
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                step()
            e1.record()
            torch.cuda.synchronize()
            times[k].append(e0.elapsed_time(e1) / iters)
    return {k: statistics.median(v) for k, v in times.items()}


def time_block(module, x, iters, groups=5, graph=False):
    """Forward + backward time (ms) of one module alone."""
    return time_steps({"m": prepare(module, x, graph)}, iters, groups)["m"]


def model_rows(which, iters):
    """Training-step time of whole models with torch's activation, InvAct and precision-bit InvAct."""
    import transformers as T
    from . import memory_table
    if which == "bert":
        name, td = "BERT-base (64 x 1024)", torch.float32
        cfg = T.BertConfig(max_position_embeddings=1024)
        make = lambda: T.BertForMaskedLM(cfg)
        ids = torch.randint(0, cfg.vocab_size, (64, 1024), device="cuda")
    else:
        name, td = "Llama-3.1-8B (1 x 512)", torch.bfloat16
        cfg = T.LlamaConfig(vocab_size=128256, hidden_size=4096, intermediate_size=14336, num_hidden_layers=32,
                            num_attention_heads=32, num_key_value_heads=8, max_position_embeddings=8192,
                            rope_theta=500000.0)
        make = lambda: T.LlamaForCausalLM(cfg)
        ids = torch.randint(0, cfg.vocab_size, (1, 512), device="cuda")
    cfg._attn_implementation = "sdpa"
    models = {}
    previous = torch.get_default_dtype()
    torch.set_default_dtype(td)
    try:
        for col in ("torch", "invact", "pbit") + (("fused",) if which == "llama" else ()):
            torch.manual_seed(0)
            with torch.device("cuda"):
                models[col] = make().train()
            if col == "fused":          # the gated MLP through the fused SwiGLU kernel: down(silu(gate(x)) * up(x))
                glu = invact_nn.InvActGLU("silu")
                for layer in models[col].model.layers:
                    mlp = layer.mlp
                    mlp.forward = (lambda x, m=mlp: m.down_proj(glu(m.gate_proj(x), m.up_proj(x))))
            elif col != "torch":
                memory_table.swap_activations(models[col], precision_bit=(col == "pbit"))
    finally:
        torch.set_default_dtype(previous)

    def stepper(model):
        def step():
            model(input_ids=ids, labels=ids).loss.backward()
            for p in model.parameters():
                p.grad = None
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        return step

    res = time_steps({col: stepper(m) for col, m in models.items()}, iters, groups=3)
    return name, {"bert": "fp32", "llama": "bf16"}[which], res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtypes", nargs="+", default=["bf16", "fp32"])
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--approximate", default="none", choices=["none", "tanh"])
    ap.add_argument("--blocks", nargs="+", default=["plain", "linear", "mlp", "geglu", "bert", "llama"])
    args = ap.parse_args()
    torch.cuda.set_device(0)
    torch.backends.cuda.matmul.allow_tf32 = False
    kind = "gelu_erf" if args.approximate == "none" else "gelu_tanh"

    acts = {
        "torch": lambda: torch.nn.GELU(approximate=args.approximate),
        "invact": lambda: invact_nn.InvActGELU(approximate=args.approximate),
        "pbit": lambda: invact_nn.InvActGELU(approximate=args.approximate, precision_bit=True),
    }
    blocks = {
        "plain GELU (2^25)": (Plain, (1 << 25,)),
        "plain GELU (2^25), graph": (Plain, (1 << 25,)),
        "plain GELU (2^28)": (Plain, (1 << 28,)),
        "Linear + GELU": (LinearAct, (BATCH, DIM)),
        "Transformer MLP block": (Mlp, (BATCH, DIM)),
        "GeGLU": (GeGlu, (BATCH, DIM)),
    }
    print(f"layers wired through {invact_nn.wiring()}", flush=True)
    print(f"{'block':26s} {'dtype':5s} {'torch ms':>9s} {'InvAct ms':>18s} {'precision-bit ms':>18s} {'InvAct fused ms':>18s}", flush=True)
    for dt in args.dtypes:
        td = {"bf16": torch.bfloat16, "fp32": torch.float32}[dt]
        for name, (cls, shape) in blocks.items():
            if not any(name.lower().replace(" ", "").startswith(b) or b in name.lower() for b in args.blocks):
                continue
            torch.manual_seed(0)
            x = torch.randn(*shape, device="cuda", dtype=torch.float32).to(td).requires_grad_(True)
            modules = {}
            for col, make in acts.items():
                torch.manual_seed(1)
                modules[col] = cls(make()).to(device="cuda", dtype=td)
            if cls is GeGlu:
                torch.manual_seed(1)
                modules["fused"] = GeGlu(glu=invact_nn.InvActGLU(kind)).to(device="cuda", dtype=td)
            if cls is Mlp and dt == "bf16":                      # the fused products are bfloat16 only
                torch.manual_seed(1)
                modules["sbit"] = MlpSignBit(kind).to(device="cuda", dtype=td)
            steps = {col: prepare(m, x, graph=name.endswith("graph")) for col, m in modules.items()}
            res = time_steps(steps, args.iters)
            del steps, modules
            base = res["torch"]
            cell = lambda k: f"{res[k]:8.3f} ({100 * (res[k] / base - 1):+6.2f}%)" if k in res else ""
            print(f"{name:26s} {dt:5s} {base:9.3f} {cell('invact'):>18s} {cell('pbit'):>18s} {cell('fused'):>18s}", flush=True)
            if "sbit" in res:
                print(f"{'  sign-bit, fused products':26s} {dt:5s} {'':9s} {cell('sbit'):>18s}", flush=True)
            del x
            torch.cuda.empty_cache()
    for which in ("bert", "llama"):
        if which in args.blocks:
            name, dt, res = model_rows(which, max(2, args.iters // 5))
            base = res["torch"]
            cell = lambda k: f"{res[k]:8.3f} ({100 * (res[k] / base - 1):+6.2f}%)"
            print(f"{name:26s} {dt:5s} {base:9.3f} {cell('invact'):>18s} {cell('pbit'):>18s} "
                  f"{cell('fused') if 'fused' in res else '':>18s}", flush=True)
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
