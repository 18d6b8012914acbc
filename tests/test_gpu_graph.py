"""The entry points enqueue exactly one kernel and nothing else (no allocation, no memset, no
synchronisation), so a caller may capture them in a HIP graph.  Replays are interleaved with
eager work and synchronisation and every replay is checked against the eager result."""
import pytest
import torch

import parity as PT
from paper_2407_15545_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_forward_backward_replay_from_a_graph(dtype):
    n = 4 * 128 * 3072 + 37                               # the small, launch-bound workload plus a ragged tail
    torch.manual_seed(0)
    x = torch.randn(n, device="cuda").to(dtype)
    up = torch.randn(n, device="cuda").to(dtype)
    g = torch.randn(n, device="cuda").to(dtype)
    outs = [torch.empty_like(x) for _ in range(6)]
    masks = [torch.empty(B.mask_bytes(n), dtype=torch.uint8, device="cuda") for _ in range(2)]

    def run():
        y, gx, act, h, gg, gu = outs
        B.invact_fwd("gelu_tanh", x, y=y, mask=masks[0])
        B.invact_bwd("gelu_tanh", y, masks[0], g, grad_x=gx)
        B.swiglu_invact_fwd(x, up, act=act, h=h, mask=masks[1])
        B.swiglu_invact_bwd(act, up, masks[1], g, grad_gate=gg, grad_up=gu)

    PT.say(f"graph capture {dtype}: eager reference")
    run()
    torch.cuda.synchronize()
    want = [t.clone() for t in outs + masks]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run()                                              # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()

    for replay in range(4):
        for t in outs + masks:
            t.fill_(0 if t.dtype == torch.uint8 else 7.0)   # eager work between replays
        x2 = torch.roll(x, 1)                              # more eager work, results unused
        torch.cuda.synchronize()
        PT.say(f"  replay {replay}")
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs + masks, want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), replay
        del x2
