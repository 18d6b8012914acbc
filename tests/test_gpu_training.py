"""The layers inside a training loop (Experiments, "gradient approximation does not affect training"):
a small transformer trained on a synthetic next-token task with torch's activation and with the InvAct
layers in its place, same seed, same batches.  The paper shows its loss curves on public datasets; here
the data are a seeded random Markov chain, which is enough to see whether the approximate derivative
bends the optimisation: both runs must learn, and their losses must stay together."""
import pytest
import torch
import torch.nn.functional as F

import parity as PT
from paper_2407_15545_amd import nn as inv

pytestmark = pytest.mark.gpu
VOCAB, DIM, HEADS, LAYERS, SEQ, BATCH, STEPS = 64, 128, 4, 2, 64, 32, 150


class Block(torch.nn.Module):
    def __init__(self, act, gated):
        super().__init__()
        self.ln1, self.ln2 = torch.nn.LayerNorm(DIM), torch.nn.LayerNorm(DIM)
        self.qkv, self.proj = torch.nn.Linear(DIM, 3 * DIM), torch.nn.Linear(DIM, DIM)
        self.gated = gated
        self.fc1 = torch.nn.Linear(DIM, 4 * DIM * (2 if gated else 1))
        self.fc2 = torch.nn.Linear(4 * DIM, DIM)
        self.act = act

    def forward(self, x):
        b, s, _ = x.shape
        q, k, v = self.qkv(self.ln1(x)).view(b, s, 3, HEADS, DIM // HEADS).permute(2, 0, 3, 1, 4)
        a = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(b, s, DIM)
        x = x + self.proj(a)
        h = self.fc1(self.ln2(x))
        if self.gated:
            gate, up = h.chunk(2, dim=-1)
            h = self.act(gate.contiguous(), up.contiguous())
        else:
            h = self.act(h)
        return x + self.fc2(h)


class TinyLM(torch.nn.Module):
    def __init__(self, make_act, gated=False):
        super().__init__()
        self.emb = torch.nn.Embedding(VOCAB, DIM)
        self.pos = torch.nn.Parameter(torch.zeros(SEQ, DIM))
        self.blocks = torch.nn.ModuleList(Block(make_act(), gated) for _ in range(LAYERS))
        self.head = torch.nn.Linear(DIM, VOCAB)

    def forward(self, ids):
        x = self.emb(ids) + self.pos
        for blk in self.blocks:
            x = blk(x)
        return self.head(x)


def markov_batches(steps, seed):
    """Sequences of a fixed random first-order Markov chain (entropy well below log VOCAB, so there is something to learn)."""
    g = torch.Generator().manual_seed(seed)
    trans = torch.softmax(3.0 * torch.randn(VOCAB, VOCAB, generator=g), dim=-1)
    out = []
    for _ in range(steps):
        ids = torch.empty(BATCH, SEQ + 1, dtype=torch.long)
        ids[:, 0] = torch.randint(0, VOCAB, (BATCH,), generator=g)
        for t in range(SEQ):
            ids[:, t + 1] = torch.multinomial(trans[ids[:, t]], 1, generator=g).squeeze(1)
        out.append(ids.cuda())
    return out


def train(make_act, batches, gated=False, dtype=torch.float32):
    torch.manual_seed(0)
    model = TinyLM(make_act, gated).cuda()
    opt = torch.optim.AdamW(model.parameters(), lr=3e-3)
    losses = []
    for ids in batches:
        with torch.autocast("cuda", dtype=dtype, enabled=dtype != torch.float32):
            logits = model(ids[:, :-1])
        loss = F.cross_entropy(logits.float().reshape(-1, VOCAB), ids[:, 1:].reshape(-1))
        opt.zero_grad(set_to_none=True)
        loss.backward()
        opt.step()
        losses.append(loss.item())
    return losses


class TorchGLU(torch.nn.Module):
    def forward(self, gate, up):
        return F.silu(gate) * up


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_training_curves_stay_together(dtype):
    batches = markov_batches(STEPS, seed=11)
    PT.say(f"training loop {dtype}")
    ref = train(lambda: torch.nn.GELU(), batches, dtype=dtype)
    runs = {
        "InvActGELU": train(lambda: inv.InvActGELU(), batches, dtype=dtype),
        "InvActGELU precision bit": train(lambda: inv.InvActGELU(precision_bit=True), batches, dtype=dtype),
    }
    tail = lambda xs: sum(xs[-20:]) / 20
    assert tail(ref) < 0.8 * ref[0], "the reference run did not learn"
    for name, losses in runs.items():
        gap = abs(tail(losses) - tail(ref)) / tail(ref)
        PT.say(f"  {name}: final loss {tail(losses):.4f} vs torch {tail(ref):.4f} ({100 * gap:.2f} % apart)")
        assert all(l == l for l in losses)
        assert gap < 0.02, (name, gap)


def test_training_with_the_fused_swiglu_layer():
    batches = markov_batches(STEPS, seed=12)
    PT.say("training loop, gated MLP")
    ref = train(lambda: TorchGLU(), batches, gated=True, dtype=torch.bfloat16)
    got = train(lambda: inv.InvActGLU("silu"), batches, gated=True, dtype=torch.bfloat16)
    tail = lambda xs: sum(xs[-20:]) / 20
    gap = abs(tail(got) - tail(ref)) / tail(ref)
    PT.say(f"  InvActGLU: final loss {tail(got):.4f} vs torch {tail(ref):.4f} ({100 * gap:.2f} % apart)")
    assert tail(ref) < 0.8 * ref[0] and gap < 0.02, gap
