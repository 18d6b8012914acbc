"""Builds libinvact.so (the HIP kernels and their C ABI) for gfx950, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "csrc", "invact_kernels.hip"),      # the element-wise kernels and their C ABI
        os.path.join(HERE, "csrc", "invact_gemm.hip")]         # the sign-bit variant's fused consumer (MFMA GEMMs)
DEPS = SRCS + [os.path.join(HERE, "csrc", "invact_math.h"), os.path.join(HERE, "csrc", "invact_constants.h"),
               os.path.join(os.path.dirname(HERE), "include", "invact.h")]
LIB = os.path.join(HERE, "libinvact.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # hipcc must not form packed-FP32 instructions on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def up_to_date():
    return os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS)


def build(force=True, verbose=False, extra=(), out=LIB):
    """Compile the library.  Returns its path."""
    if not force and out == LIB and up_to_date():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra, "-o", out, *SRCS]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


TORCH_EXT_SRC = os.path.join(HERE, "csrc", "invact_torch.cpp")
TORCH_EXT = os.path.join(HERE, "libinvact_torch.so")


def build_torch_extension(verbose=False):
    """Compile the C++ autograd wiring of the layers (host code only) against libtorch and libinvact.so."""
    import torch
    tdir = os.path.dirname(torch.__file__)
    cxx = os.environ.get("CXX", "g++")
    cmd = [cxx, "-O2", "-std=c++17", "-fPIC", "-shared", "-D__HIP_PLATFORM_AMD__=1", "-DUSE_ROCM=1",
           f"-D_GLIBCXX_USE_CXX11_ABI={int(torch._C._GLIBCXX_USE_CXX11_ABI)}",
           f"-I{tdir}/include", f"-I{tdir}/include/torch/csrc/api/include", "-I/opt/rocm/include",
           "-o", TORCH_EXT, TORCH_EXT_SRC,
           f"-L{tdir}/lib", "-ltorch", "-ltorch_cpu", "-lc10", "-lc10_hip", "-ltorch_hip",
           f"-L{HERE}", "-linvact", "-Wl,-rpath,$ORIGIN", f"-Wl,-rpath,{tdir}/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return TORCH_EXT


if __name__ == "__main__":
    # python -m paper_2407_15545_amd.build [-o variant.so] [-DINVACT_UNROLL_ALL=2 ...]
    argv = sys.argv[1:]
    if "-o" in argv:                       # a build variant for sweeps: only the library, at the given path
        i = argv.index("-o")
        out = os.path.abspath(argv[i + 1])
        build(force=True, verbose=True, extra=argv[:i] + argv[i + 2:], out=out)
        print(out)
    else:
        print(build(force=True, verbose=True, extra=argv))
        print(build_torch_extension(verbose=True))
