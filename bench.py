#!/usr/bin/env python3
"""Throughput of the Inverted-Activations hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
swiglu_invact_fwd (gate, up -> act, h, mask) followed by swiglu_invact_bwd
(act, up, mask, grad_h -> grad_gate, grad_up) on the bf16 Llama-3-8B-shaped
tensor 4 x 4096 x 14336, inputs resident in HBM before the timed region.

Prints ONE JSON line.  `value` is algorithmic bytes moved per second over the
wall-clock time of the timed steps (18.25 bytes per element and step: forward
8.125, backward 10.125); nothing but the two launches of each step happens
inside that region.  `roofline` is the same figure for the dominant kernel
alone (the backward): after the timed region each kernel is launched
--kernel-launches times back to back between ONE pair of HIP events recorded
on the launching stream, --kernel-groups times over, and the median group gives
the average launch duration (so the events' own cost is spread over the group and the sample does not
depend on --steps).  `cpu_baseline` is the double-precision oracle timed on the host on a
bounded slice of the same workload.

    python bench.py --entries [NAME ...] [--kinds ...] [--dtypes ...] [--log2-sizes ...] [--elements ...]
                    [--resident ...] [--blocks-per-cu ...] [--lib PATH ...] [--graph]

prints one line per (library build, entry point, kind, dtype, size, launch shape) instead: time per launch,
algorithmic GB/s and the share of the 8 TB/s peak, every launch of a group on the next of enough buffer
sets that the group's working set is at least three times the 256 MB Infinity Cache.

    python bench.py --consumer M,N,K [M,N,K ...]

times the sign-bit variant's fused matrix products against the decode kernel followed by torch's GEMM.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
WORKLOAD = "swiglu_bf16_4x4096x14336"
BYTES_FWD, BYTES_BWD = 8.125, 10.125          # per element, bf16
PROFILE = os.path.join("profiles", WORKLOAD + ".md")
INFINITY_CACHE = 256 << 20

# algorithmic bytes per element of every entry point: (fp32, bf16)
ENTRY_BYTES = {
    "invact_fwd": (8.125, 4.125), "invact_bwd": (12.125, 6.125),
    "geglu_invact_fwd": (16.125, 8.125), "geglu_invact_bwd": (20.125, 10.125),
    "invact_pbit_fwd": (8.0, 4.0), "invact_pbit_bwd": (12.0, 6.0),
    "invact_sbit_fwd": (8.0, 4.0), "invact_sbit_decode": (8.0, 4.0), "invact_sbit_bwd": (12.0, 6.0),
}


def profiled_traffic():
    """HBM bytes one swiglu_invact_bwd launch moves on the full workload, as rocprofv3's FETCH_SIZE and
    WRITE_SIZE counters (scaled by their readings for a plain copy) gave them in the committed profile:
    the line `traffic_bwd_bytes: <number>` of profiles/swiglu_bf16_4x4096x14336.md.  Counters cannot be
    read from inside this process, so the figure is the profile's, not this run's; None if the file is absent."""
    try:
        text = open(os.path.join(ROOT, PROFILE)).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bwd_bytes:\s*([0-9.eE+]+)\s*$", text, re.M)
    return float(m.group(1)) if m else None


def cpu_baseline(w, n_slice):
    """The oracle's gated forward + backward on the first n_slice elements, all host threads."""
    import numpy as np
    import oracle as O
    import synth
    gate, up, gh = (synth.storage_to_f64(w[k][:n_slice], "bf16") for k in ("gate", "up", "grad_h"))
    t0 = time.perf_counter()
    ae, as_, he, m = O.glu_fwd("silu", "bf16", gate, up)
    gg, gu = O.glu_bwd("silu", as_, up, m, gh)
    dt = time.perf_counter() - t0
    out = {"value": round(n_slice * (BYTES_FWD + BYTES_BWD) / dt / 1e9, 4), "unit": "GB/s",
           "cores": O.num_threads(), "kind": "oracle",
           "sample": f"first {n_slice} elements of the workload, forward+backward, {dt:.2f} s"}
    # the same code on one thread, on a smaller slice (the OpenMP runtime is told so; the oracle is untouched)
    n1 = min(n_slice, 1 << 22)
    try:
        import ctypes
        omp = ctypes.CDLL("libgomp.so.1")
        threads = O.num_threads()
        omp.omp_set_num_threads(1)
        t0 = time.perf_counter()
        _, as1, _, m1 = O.glu_fwd("silu", "bf16", gate[:n1], up[:n1])
        O.glu_bwd("silu", as1, up[:n1], m1, gh[:n1])
        dt1 = time.perf_counter() - t0
        omp.omp_set_num_threads(threads)
        out["single_thread"] = {"value": round(n1 * (BYTES_FWD + BYTES_BWD) / dt1 / 1e9, 4), "unit": "GB/s",
                                "sample": f"first {n1} elements, {dt1:.2f} s"}
    except OSError:
        pass
    # the exact branch-wise inverse (bisection), which only the accuracy reports use, timed on its own
    n2 = min(n_slice, 1 << 20)
    y_st = np.ascontiguousarray(as_[:n2])
    s_bits = O.unpack(m, n_slice)[:n2]
    t0 = time.perf_counter()
    O.finv("silu", y_st, s_bits)
    dt2 = time.perf_counter() - t0
    out["inverse_by_bisection"] = {"value": round(n2 / dt2 / 1e6, 3), "unit": "M elements/s",
                                   "sample": f"first {n2} saved activations, {dt2:.2f} s"}
    return out


def group_ms(torch, stream, launch, launches, groups):
    """Average launch duration in ms: `launches` back-to-back calls between one pair of events on `stream`,
    `groups` times; returns (median, min, max) of the groups' averages."""
    out = []
    for _ in range(groups):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(launches):
            launch()
        e1.record(stream)
        e1.synchronize()
        out.append(e0.elapsed_time(e1) / launches)
    out.sort()
    return out[len(out) // 2], out[0], out[-1]


def entry_sweep(args):
    """One line per entry point, kind, dtype, size and launch shape (see the module docstring)."""
    import torch
    from paper_2407_15545_amd import binding as B
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    sizes = [1 << s for s in args.log2_sizes] + list(args.elements_list)
    entries = args.entries or list(ENTRY_BYTES)
    warm = torch.empty(1 << 28, device="cuda", dtype=torch.bfloat16)      # bring the clocks up before timing
    for _ in range(300):
        B.invact_pbit_fwd("silu", warm, y=warm)
    torch.cuda.synchronize()
    del warm
    for lib in args.lib or [None]:
        if lib is not None:
            B._lib, B._LIB_PATH = None, os.path.abspath(lib)
        B.lib()
        tag = os.path.basename(lib) if lib else "libinvact.so"
        for n in sizes:
            for dt in args.dtypes:
                td = B.DTYPE_NAMES[dt]
                width = 4 if dt == "fp32" else 2
                # enough buffer sets that no launch finds its operands in the Infinity Cache
                sets = max(1, min(48, -(-3 * INFINITY_CACHE // (n * width * 2))))
                bufs = [dict(a=torch.randn(n, device="cuda").to(td), b=torch.randn(n, device="cuda").to(td),
                             c=torch.randn(n, device="cuda").to(td), o1=torch.empty(n, device="cuda", dtype=td),
                             o2=torch.empty(n, device="cuda", dtype=td),
                             mask=torch.empty(B.mask_bytes(n), dtype=torch.uint8, device="cuda")) for _ in range(sets)]
                launches = max(sets, 20, min(400, (1 << 35) // (n * width)))   # 30 ms or more per group
                for kind in args.kinds:
                    for s in bufs:                                         # valid saved tensors for the backward calls
                        s["y"], s["ymask"] = B.invact_fwd(kind, s["a"])
                        s["yp"] = B.invact_pbit_fwd(kind, s["a"])
                        s["ys"] = B.invact_sbit_fwd(kind, s["a"])
                    calls = {
                        "invact_fwd": lambda s: B.invact_fwd(kind, s["a"], y=s["o1"], mask=s["mask"]),
                        "invact_bwd": lambda s: B.invact_bwd(kind, s["y"], s["ymask"], s["b"], grad_x=s["o1"]),
                        "geglu_invact_fwd": lambda s: B.geglu_invact_fwd(kind, s["a"], s["b"], act=s["o1"], h=s["o2"], mask=s["mask"]),
                        "geglu_invact_bwd": lambda s: B.geglu_invact_bwd(kind, s["y"], s["b"], s["ymask"], s["c"],
                                                                         grad_gate=s["o1"], grad_up=s["o2"]),
                        "invact_pbit_fwd": lambda s: B.invact_pbit_fwd(kind, s["a"], y=s["o1"]),
                        "invact_pbit_bwd": lambda s: B.invact_pbit_bwd(kind, s["yp"], s["b"], grad_x=s["o1"]),
                        "invact_sbit_fwd": lambda s: B.invact_sbit_fwd(kind, s["a"], y_tagged=s["o1"]),
                        "invact_sbit_decode": lambda s: B.invact_sbit_decode(kind, s["ys"], y=s["o1"]),
                        "invact_sbit_bwd": lambda s: B.invact_sbit_bwd(kind, s["ys"], s["b"], grad_x=s["o1"]),
                    }
                    for entry in entries:
                        for bpc in args.blocks_per_cu_list:
                            for res in args.resident:
                                B.set_blocks_per_cu(bpc)
                                B.set_resident_blocks(res)
                                turn = [0]

                                def launch():
                                    calls[entry](bufs[turn[0] % sets])
                                    turn[0] += 1
                                if args.graph:                             # what a launch-bound caller would do
                                    side = torch.cuda.Stream()
                                    side.wait_stream(stream)
                                    g = torch.cuda.CUDAGraph()
                                    with torch.cuda.stream(side):
                                        launch()
                                        side.synchronize()
                                        with torch.cuda.graph(g, stream=side):
                                            for _ in range(launches):
                                                launch()
                                    torch.cuda.synchronize()
                                    g.replay()
                                    ms = group_ms(torch, stream, g.replay, 1, 3)[0] / launches
                                else:
                                    group_ms(torch, stream, launch, launches, 1)       # untimed: clocks, TLBs
                                    ms = group_ms(torch, stream, launch, launches, 5)[0]
                                gbs = n * ENTRY_BYTES[entry][0 if dt == "fp32" else 1] / ms / 1e6
                                note = ("launch-bound" if n < (1 << 24) else "") + (" graph" if args.graph else "")
                                print(f"{tag} {entry:18s} {kind:9s} {dt} n={n:<10d} sets={sets:<2d} bpc={bpc:<2d} res={res:<2d} "
                                      f"{ms * 1e3:9.2f} us {gbs:7.0f} GB/s {100 * gbs / HBM_PEAK_GBS:5.1f}% {note}", flush=True)
                    B.set_blocks_per_cu(0)
                    B.set_resident_blocks(0)
                del bufs


def consumer_timing(args):
    """The sign-bit variant's consumer: the fused products against invact_sbit_decode followed by torch's GEMM
    (hipBLASLt / rocBLAS; for the input gradient: torch's GEMM followed by invact_sbit_bwd), and torch's GEMM
    alone.  One line per product and shape M,N,K."""
    import torch
    from paper_2407_15545_amd import binding as B
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    kind = "gelu_erf"
    warm = torch.randn(8192, 8192, device="cuda").bfloat16()                   # bring the chip out of idle before timing
    for _ in range(40):
        torch.mm(warm, warm)
    torch.cuda.synchronize()
    del warm
    print(f"{'M x N x K':>22s}  {'product':8s} {'fused ms':>9s} {'TFLOP/s':>8s} {'decode + GEMM ms':>17s} {'TFLOP/s':>8s} "
          f"{'GEMM alone ms':>14s} {'TFLOP/s':>8s}", flush=True)
    for spec in args.consumer:
        M, N, K = (int(v) for v in spec.split(","))
        x = torch.randn(M, K, device="cuda").bfloat16()
        yt = B.invact_sbit_fwd(kind, x.view(-1)).view(M, K)
        w = (torch.randn(N, K, device="cuda") * K ** -0.5).bfloat16()
        g = torch.randn(M, N, device="cuda").bfloat16()
        y = B.invact_sbit_decode(kind, yt.view(-1)).view(M, K)
        out, gw, tmp = torch.empty(M, N, device="cuda", dtype=torch.bfloat16), torch.empty_like(w), torch.empty_like(y)
        flops = 2.0 * M * N * K
        launches = max(10, min(200, int(2e12 / flops)))
        cases = {
            "forward": (lambda: B.invact_sbit_linear_fwd(kind, yt, w, None, out=out),
                        lambda: torch.mm(B.invact_sbit_decode(kind, yt.view(-1), y=tmp.view(-1)).view(M, K), w.t(), out=out),
                        lambda: torch.mm(y, w.t(), out=out)),
            "dW": (lambda: B.invact_sbit_linear_wgrad(kind, yt, g, grad_weight=gw),
                   lambda: torch.mm(g.t(), B.invact_sbit_decode(kind, yt.view(-1), y=tmp.view(-1)).view(M, K), out=gw),
                   lambda: torch.mm(g.t(), y, out=gw)),
        }
        if N % 64 == 0 and K % 8 == 0:       # the input gradient; its comparison is torch's GEMM + invact_sbit_bwd
            gx, gy = torch.empty_like(yt), torch.empty_like(yt)
            cases["dX"] = (lambda: B.invact_sbit_linear_dgrad(kind, yt, g, w, grad_x=gx),
                           lambda: B.invact_sbit_bwd(kind, yt.view(-1), torch.mm(g, w, out=gy).view(-1), grad_x=gx.view(-1)),
                           lambda: torch.mm(g, w, out=gy))
        compared = set()                                       # the two comparisons are timed once per product
        for tile in args.linear_tile:
            B.set_linear_tile(tile)
            for name, (fused, *others) in cases.items():
                for splits in args.linear_splits if name == "dW" else [0]:
                    B.set_linear_splits(splits)
                    ws = B.sbit_linear_wgrad_workspace(M, N, K) if name == "dW" else 0
                    workspace = torch.empty(ws, dtype=torch.uint8, device="cuda") if ws else None
                    split = lambda: B.invact_sbit_linear_wgrad_ws(kind, yt, g, grad_weight=gw, workspace=workspace)
                    ms = []
                    for fn in [split if ws else fused] + ([] if name in compared else others):
                        group_ms(torch, stream, fn, launches, 1)
                        ms.append(group_ms(torch, stream, fn, launches, 5)[0])
                    compared.add(name)
                    cells = "  ".join(f"{t:>12.4f} {flops / t / 1e9:8.1f}" for t in ms)
                    note = ", ".join(([f"tile {tile}"] if tile else []) + ([f"splits {splits}"] if splits else []) +
                                     ([f"workspace {ws >> 20} MiB"] if ws else []))
                    print(f"{M:>8d} x {N:>5d} x {K:>5d}  {name:8s} {cells}" + (f"   [{note}]" if note else ""), flush=True)
        B.set_linear_tile(0)
        B.set_linear_splits(0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--cpu-elems", type=int, default=1 << 28, help="elements of the CPU-baseline slice (0 = skip)")
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--elements", type=int, default=0, help="override the element count (debugging only)")
    ap.add_argument("--kernel-launches", type=int, default=60,
                    help="back-to-back launches of each kernel between one event pair, after the timed steps")
    ap.add_argument("--kernel-groups", type=int, default=5, help="such groups per kernel; the median one is reported")
    ap.add_argument("--unfused-iters", type=int, default=20,
                    help="after the timed steps, time the unfused forward (invact_fwd + a separate multiply) this "
                         "many times for comparison (0 = skip); never part of `value`")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="after the timed steps, run this many plain device copies of one tensor (reads and "
                         "writes 2 bytes per element each): the known traffic that rocprofv3's FETCH_SIZE / "
                         "WRITE_SIZE readings are scaled by")
    sw = ap.add_argument_group("entry-point sweep (prints a table instead of the JSON line)")
    sw.add_argument("--entries", nargs="*", default=None, help="entry points to time (no name = all)")
    sw.add_argument("--kinds", nargs="+", default=["gelu_tanh", "gelu_erf", "silu"])
    sw.add_argument("--dtypes", nargs="+", default=["bf16", "fp32"])
    sw.add_argument("--log2-sizes", type=int, nargs="*", default=[], help="log2 of element counts")
    sw.add_argument("--elements-list", type=int, nargs="*", default=[], help="element counts, e.g. 50331648")
    sw.add_argument("--resident", type=int, nargs="+", default=[0],
                    help="cap on resident workgroups per compute unit (0 = the library's default, 32 = none)")
    sw.add_argument("--blocks-per-cu-list", type=int, nargs="+", default=[0],
                    help="persistent grids of this many workgroups per compute unit (0 = one tile per workgroup)")
    sw.add_argument("--lib", nargs="*", default=None, help="alternative builds of libinvact.so to compare")
    sw.add_argument("--graph", action="store_true", help="time replays of a HIP graph holding the launches")
    sw.add_argument("--consumer", nargs="+", default=None, metavar="M,N,K",
                    help="time the sign-bit variant's fused products (forward and weight gradient) at these shapes "
                         "against invact_sbit_decode + torch's GEMM")
    sw.add_argument("--linear-tile", type=int, nargs="+", default=[0], choices=[0, 2, 3, 4],
                    help="with --consumer: force the fused products' workgroup tile (4: 256 x 256, 2: 128 x 128, 0: the library's choice)")
    sw.add_argument("--linear-splits", type=int, nargs="+", default=[0],
                    help="with --consumer: force the number of parts the weight gradient's contraction is split into "
                         "(0: the library's choice; 1: none)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path is element-wise and needs no exchange between GPUs, "
                 "so this build has no multi-GPU mode (--gpus must be 1).")

    import torch
    import parity as PT
    from paper_2407_15545_amd import binding as B
    import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    from paper_2407_15545_amd import build as hip_build
    if not os.path.exists(hip_build.LIB):               # nothing built yet: build, never fall back
        hip_build.build(force=True)
    B.lib()                                              # fails loudly if the HIP library is missing
    if args.consumer:
        return consumer_timing(args)
    if args.entries is not None:
        if not (args.log2_sizes or args.elements_list):
            args.log2_sizes = [26, 28]
        return entry_sweep(args)
    if args.blocks_per_cu:
        B.set_blocks_per_cu(args.blocks_per_cu)

    n = args.elements or synth.numel(WORKLOAD)
    w = synth.make(WORKLOAD, n=n)
    gate, up, gh = (PT.to_device(w[k], "bf16") for k in ("gate", "up", "grad_h"))
    act, h = torch.empty_like(gate), torch.empty_like(gate)
    gg, gu = torch.empty_like(gate), torch.empty_like(gate)
    mask = torch.empty(B.mask_bytes(n), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def fwd():
        B.swiglu_invact_fwd(gate, up, act=act, h=h, mask=mask, stream=stream)

    def bwd():
        B.swiglu_invact_bwd(act, up, mask, gh, grad_gate=gg, grad_up=gu, stream=stream)

    for _ in range(args.warmup):
        fwd(); bwd()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fwd(); bwd()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # per-kernel durations, outside the timed region
    fwd_ms, fwd_lo, fwd_hi = group_ms(torch, stream, fwd, args.kernel_launches, args.kernel_groups)
    bwd_ms, bwd_lo, bwd_hi = group_ms(torch, stream, bwd, args.kernel_launches, args.kernel_groups)

    # The forward as two launches, for comparison: invact_fwd(silu) saves act and the mask, then a
    # separate element-wise multiply (torch's) reads act and up and writes h: 4.125 + 6 bytes per element.
    unfused = None
    if args.unfused_iters:
        def unfused_fwd():
            B.invact_fwd("silu", gate, y=act, mask=mask, stream=stream)
            torch.mul(act, up, out=h)
        for _ in range(3):
            unfused_fwd()
        unfused = group_ms(torch, stream, unfused_fwd, args.unfused_iters, 1)[0]

    for _ in range(args.calibration_copies):
        act.copy_(gate)
    torch.cuda.synchronize()

    ms_step = wall * 1e3 / args.steps
    value = n * (BYTES_FWD + BYTES_BWD) / (ms_step * 1e-3) / 1e9
    bwd_gbs = n * BYTES_BWD / (bwd_ms * 1e-3) / 1e9
    fwd_gbs = n * BYTES_FWD / (fwd_ms * 1e-3) / 1e9
    full = n == synth.numel(WORKLOAD)

    out = {
        "metric": "effective HBM GB/s (fwd+bwd), bf16 SwiGLU 4x4096x14336",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD, "storage": "bf16", "registers": "f32", "elements": n,
                   "inputs": "gate~N(0,1) seed 0, up~N(0,1) seed 2, grad_h~N(0,0.01^2) seed 1",
                   "bytes_per_element": {"fwd": BYTES_FWD, "bwd": BYTES_BWD},
                   "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
                   "kernel_timing": f"median of {args.kernel_groups} groups of {args.kernel_launches} back-to-back "
                                    "launches, one HIP event pair per group, after the timed steps",
                   "fwd_kernel": {"ms": round(fwd_ms, 5), "GB/s": round(fwd_gbs, 1),
                                  "ms_min_max_over_groups": [round(fwd_lo, 5), round(fwd_hi, 5)]},
                   "bwd_kernel": {"ms": round(bwd_ms, 5), "GB/s": round(bwd_gbs, 1),
                                  "ms_min_max_over_groups": [round(bwd_lo, 5), round(bwd_hi, 5)]}},
        "roofline": {"bound": "hbm", "kernel": "stream_kernel<GluBwdOp<silu,bf16>> (swiglu_invact_bwd)",
                     "achieved": round(bwd_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(bwd_gbs / HBM_PEAK_GBS, 4),
                     "traffic": profiled_traffic() if full else None,
                     "traffic_source": (PROFILE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, a run of their own: "
                                        "counters cannot be read from inside this process)") if full else None,
                     "algorithmic_bytes": n * BYTES_BWD, "avg_launch_ms": round(bwd_ms, 5),
                     "launches": args.kernel_launches * args.kernel_groups},
    }
    if unfused is not None:
        out["config"]["unfused_fwd"] = {"ms": round(unfused, 5), "bytes_per_element": 10.125,
                                        "GB/s": round(n * 10.125 / (unfused * 1e-3) / 1e9, 1),
                                        "what": "invact_fwd(silu) + torch.mul, for comparison with fwd_kernel"}
    if args.cpu_elems:
        out["cpu_baseline"] = cpu_baseline(w, min(args.cpu_elems, n))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
