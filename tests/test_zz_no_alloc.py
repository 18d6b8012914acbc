"""The entry point that allocates nothing (invact_sbit_linear_wgrad_static): the same bits as
invact_sbit_linear_wgrad_ws with a caller's workspace, on calls in a row that share the library's per-GPU array."""
import pytest
import torch

import parity as PT
import synth
from paper_2407_15545_amd import binding as B

pytestmark = pytest.mark.gpu


def tagged_and_gradient(kind, M, N, K, seed):
    """Device tensors: the saved tensor of the sign-bit forward on seeded N(0, 2^2) pre-activations, and dOut ~ N(0, 1)."""
    x = PT.to_device(synth.to_storage(synth.normal(M * K, seed, 2.0), "bf16"), "bf16")
    yt = B.invact_sbit_fwd(kind, x).view(M, K)
    g = PT.to_device(synth.to_storage(synth.normal(M * N, seed + 1, 1.0), "bf16"), "bf16").view(M, N)
    return yt, g


def test_static_scratch_gives_the_bits_of_a_caller_workspace_call_after_call():
    kind = "gelu_erf"
    # 64 MiB of partial sums (four parts of 64 large tiles), then a smaller product in the same array (16 MiB:
    # four parts of 64 small tiles), then one that does not split, then the first again
    shapes = [(8192, 1024, 4096), (4096, 1024, 1024), (8192, 4096, 4096), (8192, 1024, 4096)]
    expected_bytes = [64 << 20, 16 << 20, 0, 64 << 20]
    for (M, N, K), nbytes in zip(shapes, expected_bytes):
        PT.say(f"invact_sbit_linear_wgrad_static {kind} M={M} N={N} K={K}")
        assert B.sbit_linear_wgrad_workspace(M, N, K) == nbytes
        yt, g = tagged_and_gradient(kind, M, N, K, 4100 + K)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda") if nbytes else None
        want = B.invact_sbit_linear_wgrad_ws(kind, yt, g, workspace=workspace)
        got = torch.full((N, K), float("nan"), dtype=torch.bfloat16, device="cuda")
        allocations = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]      # a count that only grows
        before = allocations()
        B.invact_sbit_linear_wgrad_static(kind, yt, g, grad_weight=got)
        assert allocations() == before
        torch.cuda.synchronize()
        assert torch.equal(got, want), (M, N, K)
        assert bool(torch.isfinite(got.float()).all())


def test_static_scratch_refuses_what_does_not_fit():
    kind, M, N, K = "silu", 8192, 1024, 4096
    yt, g = tagged_and_gradient(kind, M, N, K, 4200)
    out = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    B.set_linear_tile(4)
    B.set_linear_splits(8)                                   # 8 parts of 64 large tiles: 128 MiB
    try:
        assert B.sbit_linear_wgrad_workspace(M, N, K) == 128 << 20
        with pytest.raises(B.InvactError) as err:
            B.invact_sbit_linear_wgrad_static(kind, yt, g, grad_weight=out)
        assert err.value.status == 5                          # INVACT_ERR_SIZE, before anything is launched
    finally:
        B.set_linear_tile(0)
        B.set_linear_splits(0)


def test_static_scratch_replays_from_a_graph():
    """What the entry point is for: captured in a HIP graph (both of its kernels, no allocation), replayed on
    inputs that change between replays, with eager work and synchronisation in between; every replay against
    the eager result on the same inputs."""
    kind, M, N, K = "gelu_tanh", 4096, 1024, 1024
    assert B.sbit_linear_wgrad_workspace(M, N, K) > 0
    yt, g = tagged_and_gradient(kind, M, N, K, 4300)
    out = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        B.invact_sbit_linear_wgrad_static(kind, yt, g, grad_weight=out)          # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            B.invact_sbit_linear_wgrad_static(kind, yt, g, grad_weight=out)
    torch.cuda.synchronize()
    for replay in range(3):
        PT.say(f"invact_sbit_linear_wgrad_static from a graph, replay {replay}")
        fresh_yt, fresh_g = tagged_and_gradient(kind, M, N, K, 4310 + 2 * replay)
        yt.copy_(fresh_yt)
        g.copy_(fresh_g)
        out.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = B.invact_sbit_linear_wgrad_ws(kind, yt, g)
        torch.cuda.synchronize()
        assert torch.equal(out, want), replay
