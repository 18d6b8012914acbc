"""Throughput of every entry point over kinds, dtypes and sizes (one GPU).

    python -m paper_2407_15545_amd.sweep [--sizes 20 24 26 28] [--blocks-per-cu 0 1 2] [--lib PATH ...]

Prints one line per (library, entry point, kind, dtype, size, launch shape):
time per launch (median of 3 groups of launches, HIP events on the launching
stream), algorithmic GB/s and the share of the 8 TB/s HBM peak.  Inputs are
N(0,1) draws made on the device: throughput does not depend on the values
beyond the branch mix.  Sizes up to 2^24 elements fit in the 256 MB Infinity
Cache together with their outputs and are marked "cache".
"""
import argparse
import os

import torch

from . import binding as B

PEAK = 8000.0
BYTES = {  # algorithmic bytes per element: (fp32, bf16)
    "invact_fwd": (8.125, 4.125), "invact_bwd": (12.125, 6.125),
    "geglu_invact_fwd": (16.125, 8.125), "geglu_invact_bwd": (20.125, 10.125),
    "invact_pbit_fwd": (8.0, 4.0), "invact_pbit_bwd": (12.0, 6.0),
    "invact_sbit_fwd": (8.0, 4.0), "invact_sbit_decode": (8.0, 4.0), "invact_sbit_bwd": (12.0, 6.0),
}


def timeit(fn, iters, graph=False):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    if graph:
        # the launches are recorded once and replayed: what a launch-bound caller would do
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            fn()
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                for _ in range(iters):
                    fn()
        torch.cuda.synchronize()
        fn, iters_per_call = g.replay, iters
        ts = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / iters_per_call)
        return sorted(ts)[1]
    ts = []
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) / iters)
    return sorted(ts)[1]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes", type=int, nargs="*", default=[20, 22, 24, 26, 28], help="log2 of the element counts")
    ap.add_argument("--elements", type=int, nargs="*", default=[], help="extra element counts (e.g. 234881024)")
    ap.add_argument("--kinds", nargs="+", default=["gelu_tanh", "gelu_erf", "silu"])
    ap.add_argument("--dtypes", nargs="+", default=["bf16", "fp32"])
    ap.add_argument("--entries", nargs="+", default=list(BYTES))
    ap.add_argument("--blocks-per-cu", type=int, nargs="+", default=[0])
    ap.add_argument("--resident", type=int, nargs="+", default=[0],
                    help="cap on resident workgroups per compute unit (0 = the library's default, 8 = none)")
    ap.add_argument("--lib", nargs="*", default=[None], help="alternative builds of libinvact.so to compare")
    ap.add_argument("--graph", action="store_true", help="time replays of a HIP graph holding the launches")
    args = ap.parse_args()
    torch.cuda.set_device(0)
    sizes = [1 << s for s in args.sizes] + list(args.elements)
    warm = torch.empty(1 << 28, device="cuda", dtype=torch.bfloat16)      # bring the clocks up before timing
    for _ in range(300):
        B.invact_pbit_fwd("silu", warm, y=warm)
    torch.cuda.synchronize()
    del warm
    for lib in args.lib:
        if lib is not None:
            B._lib, B._LIB_PATH = None, os.path.abspath(lib)
        B.lib()
        tag = os.path.basename(lib) if lib else "libinvact.so"
        for n in sizes:
            for dt in args.dtypes:
                td = B.DTYPE_NAMES[dt]
                a, b, c = (torch.randn(n, device="cuda", dtype=torch.float32).to(td) for _ in range(3))
                o1, o2 = torch.empty_like(a), torch.empty_like(a)
                mask = torch.empty(B.mask_bytes(n), dtype=torch.uint8, device="cuda")
                iters = max(5, min(200, (1 << 31) // (n * (4 if dt == "fp32" else 2))))
                for kind in args.kinds:
                    B.invact_fwd(kind, a, y=o1, mask=mask)          # a valid (y, mask) pair for the backward
                    y_saved = o1.clone()
                    y_tagged = B.invact_pbit_fwd(kind, a)
                    y_signed = B.invact_sbit_fwd(kind, a)
                    calls = {
                        "invact_sbit_fwd": lambda: B.invact_sbit_fwd(kind, a, y_tagged=o1),
                        "invact_sbit_decode": lambda: B.invact_sbit_decode(kind, y_signed, y=o1),
                        "invact_sbit_bwd": lambda: B.invact_sbit_bwd(kind, y_signed, b, grad_x=o1),
                        "invact_pbit_fwd": lambda: B.invact_pbit_fwd(kind, a, y=o1),
                        "invact_pbit_bwd": lambda: B.invact_pbit_bwd(kind, y_tagged, b, grad_x=o1),
                        "invact_fwd": lambda: B.invact_fwd(kind, a, y=o1, mask=mask),
                        "invact_bwd": lambda: B.invact_bwd(kind, y_saved, mask, b, grad_x=o1),
                        "geglu_invact_fwd": lambda: B.geglu_invact_fwd(kind, a, b, act=o1, h=o2, mask=mask),
                        "geglu_invact_bwd": lambda: B.geglu_invact_bwd(kind, y_saved, b, mask, c, grad_gate=o1, grad_up=o2),
                    }
                    shapes = [(bpc, res) for bpc in args.blocks_per_cu for res in args.resident]
                    for entry in args.entries:
                        for bpc, res in shapes:
                            B.set_blocks_per_cu(bpc)
                            B.set_resident_blocks(res)
                            B.invact_fwd(kind, a, y=o2, mask=mask)  # restore the mask the backward reads
                            ms = timeit(calls[entry], iters, args.graph)
                            nbytes = n * BYTES[entry][0 if dt == "fp32" else 1]
                            gbs = nbytes / ms / 1e6
                            note = ("cache" if n <= (1 << 24) else "") + (" graph" if args.graph else "")
                            print(f"{tag} {entry:17s} {kind:9s} {dt} n={n:<10d} bpc={bpc:<2d} res={res:<2d} {ms * 1e3:9.2f} us "
                                  f"{gbs:7.0f} GB/s {100 * gbs / PEAK:5.1f}% {note}", flush=True)
                B.set_blocks_per_cu(0)
                B.set_resident_blocks(0)
                del a, b, c, o1, o2, mask


if __name__ == "__main__":
    main()
