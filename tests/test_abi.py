"""The C ABI without a GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2407_15545_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "invact.h")

OK, ERR_KIND, ERR_DTYPE, ERR_NULL, ERR_ALIGN, ERR_SIZE, ERR_HIP = range(7)


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b((?:invact|swiglu_invact|geglu_invact)\w*)\s*\(", text)))


def test_header_is_valid_c():
    src = '#include "invact.h"\nint main(void) { return (int)invact_mask_bytes(3); }\n'
    subprocess.run(["gcc", "-x", "c", "-fsyntax-only", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                    "-I" + os.path.join(ROOT, "include"), "-"], input=src.encode(), check=True)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"invact_fwd", "invact_bwd", "swiglu_invact_fwd", "swiglu_invact_bwd", "geglu_invact_fwd",
            "geglu_invact_bwd", "invact_mask_bytes", "invact_strerror"} <= set(names)
    lib = B.lib()
    for name in names:
        assert hasattr(lib, name), name
        assert name in B._PROTOTYPES, f"binding has no prototype for {name}"


def test_mask_bytes():
    for n, want in [(0, 0), (1, 8), (63, 8), (64, 8), (65, 16), (128, 16), (129, 24), (1 << 28, 1 << 25),
                    (234881024, 29360128)]:
        assert B.mask_bytes(n) == want
    assert B.mask_bytes(2 ** 64 - 1) == 8 * ((2 ** 64 - 1 + 63) // 64)


def test_strerror_texts_are_distinct():
    texts = [B.strerror(i) for i in range(7)]
    assert len(set(texts)) == 7 and texts[0] == "success"
    assert B.strerror(99) == "unknown status"


def test_argument_validation_happens_before_any_launch():
    lib = B.lib()
    a16, a8, odd = 0x1000, 0x1008, 0x1004          # never dereferenced: every call below is rejected
    fwd, bwd = lib.invact_fwd, lib.invact_bwd
    assert fwd(3, 0, a16, a16, a16, 8, None) == ERR_KIND
    assert fwd(-1, 0, a16, a16, a16, 8, None) == ERR_KIND
    assert fwd(0, 2, a16, a16, a16, 8, None) == ERR_DTYPE
    assert fwd(0, 0, None, a16, a16, 8, None) == ERR_NULL
    assert fwd(0, 0, a16, None, a16, 8, None) == ERR_NULL
    assert fwd(0, 0, a16, a16, None, 8, None) == ERR_NULL
    assert fwd(0, 0, a8, a16, a16, 8, None) == ERR_ALIGN
    assert fwd(0, 1, a16, a8, a16, 8, None) == ERR_ALIGN
    assert fwd(0, 1, a16, a16, odd, 8, None) == ERR_ALIGN
    assert fwd(0, 0, a16, a16, a16, 2 ** 64 - 1, None) == ERR_SIZE
    assert bwd(0, 0, a16, a16, None, a16, 8, None) == ERR_NULL
    assert bwd(0, 0, a16, odd, a16, a16, 8, None) == ERR_ALIGN
    assert bwd(2, 5, a16, a16, a16, a16, 8, None) == ERR_DTYPE
    assert lib.geglu_invact_fwd(9, 1, a16, a16, a16, a16, a16, 8, None) == ERR_KIND
    assert lib.geglu_invact_bwd(0, 1, a16, a16, a16, a16, a16, None, 8, None) == ERR_NULL
    assert lib.swiglu_invact_fwd(1, a16, a16, a16, a8, a16, 8, None) == ERR_ALIGN
    assert lib.swiglu_invact_bwd(7, a16, a16, a16, a16, a16, a16, 8, None) == ERR_DTYPE
    assert lib.invact_pbit_fwd(0, 0, a16, None, 8, None) == ERR_NULL
    assert lib.invact_pbit_fwd(0, 1, a8, a16, 8, None) == ERR_ALIGN
    assert lib.invact_pbit_bwd(3, 1, a16, a16, a16, 8, None) == ERR_KIND
    assert lib.invact_pbit_bwd(0, 1, a16, a16, a16, 0, None) == OK
    lin, wg = lib.invact_sbit_linear_fwd, lib.invact_sbit_linear_wgrad
    assert lin(5, 1, a16, a16, None, a16, 128, 128, 64, None) == ERR_KIND
    assert lin(1, 0, a16, a16, None, a16, 128, 128, 64, None) == ERR_DTYPE          # bfloat16 only
    assert lin(1, 1, a16, a16, None, a16, 128, 128, 65, None) == ERR_SIZE           # K in whole steps of 64
    assert lin(1, 1, a16, a16, None, a16, 1 << 20, 128, 1 << 12, None) == ERR_SIZE  # 2^32 elements
    assert lin(1, 1, None, a16, None, a16, 128, 128, 64, None) == ERR_NULL
    assert lin(1, 1, a16, a8, None, a16, 128, 128, 64, None) == ERR_ALIGN
    assert lin(1, 1, a16, a16, None, a16, 0, 128, 64, None) == OK
    assert wg(1, 1, a16, a16, a16, 100, 128, 64, None) == ERR_SIZE                  # M in whole steps of 64
    assert wg(1, 1, a16, a16, a16, 128, 100, 64, None) == ERR_SIZE                  # N, K multiples of 8
    assert wg(1, 0, a16, a16, a16, 128, 128, 64, None) == ERR_DTYPE
    assert wg(1, 1, a16, None, a16, 128, 128, 64, None) == ERR_NULL
    assert wg(1, 1, a16, a16, odd, 128, 128, 64, None) == ERR_ALIGN
    assert wg(1, 1, a16, a16, a16, 128, 0, 64, None) == OK
    dg = lib.invact_sbit_linear_dgrad
    assert dg(1, 1, a16, a16, a16, a16, 128, 100, 64, None) == ERR_SIZE              # N in whole steps of 64
    assert dg(1, 1, a16, a16, a16, a16, 128, 64, 100, None) == ERR_SIZE              # K a multiple of 8
    assert dg(1, 0, a16, a16, a16, a16, 128, 64, 64, None) == ERR_DTYPE
    assert dg(4, 1, a16, a16, a16, a16, 128, 64, 64, None) == ERR_KIND
    assert dg(1, 1, a16, a16, None, a16, 128, 64, 64, None) == ERR_NULL
    assert dg(1, 1, a16, a16, a16, a8, 128, 64, 64, None) == ERR_ALIGN
    assert dg(1, 1, a16, a16, a16, a16, 0, 64, 64, None) == OK
    # the weight gradient that may split its contraction: what it asks for, and what it refuses (host logic only)
    ws, need = lib.invact_sbit_linear_wgrad_ws, lib.invact_sbit_linear_wgrad_workspace
    assert need(8192, 4096, 4096) == 0                           # 256 tiles of 256 x 256: not split
    assert need(8192, 1024, 4096) == 4 * 64 * 256 * 256 * 4      # 64 tiles: four parts of binary32 partial tiles
    assert need(2048, 1024, 4096) == 2 * 64 * 256 * 256 * 4      # parts of at least 16 steps
    assert need(64, 128, 128) == 0 and need(100, 128, 64) == 0 and need(0, 8, 8) == 0
    assert ws(1, 1, a16, a16, a16, 8192, 1024, 4096, a16, (1 << 26) - 16, None) == ERR_SIZE
    assert ws(1, 1, a16, a16, a16, 8192, 1024, 4096, None, 1 << 26, None) == ERR_NULL
    assert ws(1, 1, a16, a16, a16, 8192, 1024, 4096, a8, 1 << 26, None) == ERR_ALIGN
    assert ws(1, 1, a16, a16, a16, 100, 128, 64, a16, 1 << 26, None) == ERR_SIZE
    assert ws(1, 0, a16, a16, a16, 8192, 1024, 4096, a16, 1 << 26, None) == ERR_DTYPE
    assert ws(1, 1, a16, a16, a16, 8192, 0, 4096, None, 0, None) == OK
    # n == 0 is a successful no-op, whatever the pointers
    assert fwd(0, 0, None, None, None, 0, None) == OK
    assert bwd(2, 1, None, None, None, None, 0, None) == OK
    assert lib.swiglu_invact_bwd(1, None, None, None, None, None, None, 0, None) == OK


def test_blocks_per_cu_range():
    try:
        assert B.set_blocks_per_cu(4) == 4
        assert B.set_blocks_per_cu(65) < 0 and B.set_blocks_per_cu(-1) < 0
    finally:
        assert B.set_blocks_per_cu(0) == 0


def test_resident_blocks_range():
    try:
        assert B.set_resident_blocks(16) == 16 and B.set_resident_blocks(32) == 32
        assert B.set_resident_blocks(33) < 0 and B.set_resident_blocks(-1) < 0
    finally:
        assert B.set_resident_blocks(0) == 0


def test_binding_raises_with_the_library_message():
    with pytest.raises(B.InvactError) as e:
        B._check(ERR_ALIGN)
    assert "aligned" in str(e.value) and e.value.status == ERR_ALIGN


def test_torch_extension_loads_and_refuses_cpu_tensors():
    """The C++ autograd wiring of the layers: the operators exist, and there is no CPU path behind them."""
    import torch
    from paper_2407_15545_amd import nn
    previous = nn.set_wiring("c++")
    try:
        assert nn.wiring() == "c++"
        for name in ("act", "act_pbit", "glu"):
            assert hasattr(torch.ops.invact, name)
        with pytest.raises(RuntimeError, match="GPU tensors"):
            nn.invact(torch.randn(8), "gelu_erf")
        with pytest.raises(RuntimeError, match="float32 and bfloat16|GPU tensors"):
            nn.invact_glu(torch.randn(8), torch.randn(8), "silu")
    finally:
        nn.set_wiring(previous)


def test_linear_tuning_knobs_and_the_workspace_they_imply():
    """Host logic only: the forced tile and number of splits, their ranges, and the workspace size that follows."""
    need = B.lib().invact_sbit_linear_wgrad_workspace
    try:
        assert B.lib().invact_set_linear_tile(1) < 0 and B.lib().invact_set_linear_tile(5) < 0
        assert B.lib().invact_set_linear_splits(-1) < 0 and B.lib().invact_set_linear_splits(65) < 0
        assert B.lib().invact_set_linear_splits(8) == 8
        assert need(8192, 1024, 4096) == 8 * 64 * 256 * 256 * 4               # the library's tile (large), eight parts
        assert need(128, 1024, 4096) == 2 * 64 * 256 * 256 * 4                # capped at the number of 64-row steps
        assert B.lib().invact_set_linear_tile(2) == 2
        assert need(8192, 1024, 4096) == 8 * 256 * 128 * 128 * 4              # 128 x 128 tiles: 8 x 32 of them
        assert B.lib().invact_set_linear_splits(1) == 1
        assert need(8192, 1024, 4096) == 0
        assert B.lib().invact_set_linear_splits(0) == 0
        assert need(8192, 1024, 4096) == 0                                    # a forced tile alone: no split
    finally:
        assert B.lib().invact_set_linear_tile(0) == 0 and B.lib().invact_set_linear_splits(0) == 0
    assert need(8192, 1024, 4096) == 4 * 64 * 256 * 256 * 4
    assert need(4096, 1024, 1024) == 4 * 64 * 128 * 128 * 4                   # too short for large tiles: small ones, four parts
