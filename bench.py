#!/usr/bin/env python3
"""Throughput of the Inverted-Activations hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
swiglu_invact_fwd (gate, up -> act, h, mask) followed by swiglu_invact_bwd
(act, up, mask, grad_h -> grad_gate, grad_up) on the bf16 Llama-3-8B-shaped
tensor 4 x 4096 x 14336, inputs resident in HBM before the timed region.

Prints ONE JSON line.  `value` is algorithmic bytes moved per second
(18.25 bytes per element and step: forward 8.125, backward 10.125); `roofline`
is the same figure for the dominant kernel alone (the backward), from HIP
events recorded around the launches of every 4th timed step on the stream the
kernels run on;
`cpu_baseline` is the double-precision oracle timed on the host on a bounded
slice of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
WORKLOAD = "swiglu_bf16_4x4096x14336"
BYTES_FWD, BYTES_BWD = 8.125, 10.125          # per element, bf16
# HBM bytes one swiglu_invact_bwd launch moves on the full workload, from rocprofv3's
# FETCH_SIZE and WRITE_SIZE counters scaled by their readings for a plain copy
# (profiles/swiglu_bf16_4x4096x14336.md): 1468.0 MB read + 939.5 MB written.  The read side is
# 29.4 MB (1.2 %) above the algorithmic bytes: the 64 mask bytes of a wave tile are half a cache
# line, and the two wavefronts sharing a line run on different XCDs, so the mask is fetched twice.
TRAFFIC_BWD_FULL = 2407.5e6


def cpu_baseline(w, n_slice):
    """The oracle's gated forward + backward on the first n_slice elements, all host threads."""
    import numpy as np
    import oracle as O
    from paper_2407_15545_amd import synth
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--cpu-elems", type=int, default=1 << 28, help="elements of the CPU-baseline slice (0 = skip)")
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--elements", type=int, default=0, help="override the element count (debugging only)")
    ap.add_argument("--unfused-iters", type=int, default=20,
                    help="after the timed steps, time the unfused forward (invact_fwd + a separate multiply) this "
                         "many times for comparison (0 = skip); never part of `value`")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="after the timed steps, run this many plain device copies of one tensor (reads and "
                         "writes 2 bytes per element each): the known traffic that rocprofv3's FETCH_SIZE / "
                         "WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path is element-wise and needs no exchange between GPUs, "
                 "so this build has no multi-GPU mode (--gpus must be 1).")

    import torch
    import parity as PT
    from paper_2407_15545_amd import binding as B
    from paper_2407_15545_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    from paper_2407_15545_amd import build as hip_build
    if not os.path.exists(hip_build.LIB):               # nothing built yet: build, never fall back
        hip_build.build(force=True)
    B.lib()                                              # fails loudly if the HIP library is missing
    if args.blocks_per_cu:
        B.set_blocks_per_cu(args.blocks_per_cu)

    n = args.elements or synth.numel(WORKLOAD)
    w = synth.make(WORKLOAD, n=n)
    gate, up, gh = (PT.to_device(w[k], "bf16") for k in ("gate", "up", "grad_h"))
    act, h = torch.empty_like(gate), torch.empty_like(gate)
    gg, gu = torch.empty_like(gate), torch.empty_like(gate)
    mask = torch.empty(B.mask_bytes(n), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def step(ev=None):
        if ev: ev[0].record(stream)
        B.swiglu_invact_fwd(gate, up, act=act, h=h, mask=mask, stream=stream)
        if ev: ev[1].record(stream)
        B.swiglu_invact_bwd(act, up, mask, gh, grad_gate=gg, grad_up=gu, stream=stream)
        if ev: ev[2].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # per-kernel durations come from HIP events around the launches of every 4th step of the timed region
    # (an event costs the stream a few microseconds; the other steps run exactly as a caller would run them)
    timed = [i for i in range(args.steps) if i % 4 == 0]
    events = {i: [torch.cuda.Event(enable_timing=True) for _ in range(3)] for i in timed}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events.get(i))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    events = list(events.values())

    # The forward as two launches, for comparison: invact_fwd(silu) saves act and the mask, then a
    # separate element-wise multiply (torch's) reads act and up and writes h: 4.125 + 6 bytes per element.
    unfused = None
    if args.unfused_iters:
        def unfused_fwd():
            B.invact_fwd("silu", gate, y=act, mask=mask, stream=stream)
            torch.mul(act, up, out=h)
        for _ in range(3):
            unfused_fwd()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.unfused_iters):
            unfused_fwd()
        e1.record(stream)
        torch.cuda.synchronize()
        unfused = e0.elapsed_time(e1) / args.unfused_iters

    for _ in range(args.calibration_copies):
        act.copy_(gate)
    torch.cuda.synchronize()

    ms_step = wall * 1e3 / args.steps
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in events) / len(events)
    bwd_ms = sum(e[1].elapsed_time(e[2]) for e in events) / len(events)
    value = n * (BYTES_FWD + BYTES_BWD) / (ms_step * 1e-3) / 1e9
    bwd_gbs = n * BYTES_BWD / (bwd_ms * 1e-3) / 1e9
    fwd_gbs = n * BYTES_FWD / (fwd_ms * 1e-3) / 1e9

    out = {
        "metric": "effective HBM GB/s (fwd+bwd), bf16 SwiGLU 4x4096x14336",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD, "storage": "bf16", "elements": n,
                   "inputs": "gate~N(0,1) seed 0, up~N(0,1) seed 2, grad_h~N(0,0.01^2) seed 1",
                   "bytes_per_element": {"fwd": BYTES_FWD, "bwd": BYTES_BWD},
                   "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
                   "launches_timed_with_events": len(events),
                   "fwd_kernel": {"ms": round(fwd_ms, 5), "GB/s": round(fwd_gbs, 1)},
                   "bwd_kernel": {"ms": round(bwd_ms, 5), "GB/s": round(bwd_gbs, 1)}},
        "roofline": {"bound": "hbm", "kernel": "stream_kernel<GluBwdOp<silu,bf16>> (swiglu_invact_bwd)",
                     "achieved": round(bwd_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(bwd_gbs / HBM_PEAK_GBS, 4),
                     "traffic": TRAFFIC_BWD_FULL if n == synth.numel(WORKLOAD) else None,
                     "algorithmic_bytes": n * BYTES_BWD, "avg_launch_ms": round(bwd_ms, 5)},
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
