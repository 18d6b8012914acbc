"""Host-side checks: the seeded workloads are reproducible and have the stated structure, the
storage conversions are exact, and bench.py refuses more than one GPU."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_workload_table_matches_the_benchmark_configs():
    assert synth.numel("gelu_tanh_fp32_4x128x3072") == 1572864
    assert synth.numel("gelu_erf_bf16_32x512x3072") == 50331648
    assert synth.numel("silu_bf16_8x2048x11008") == 180355072
    assert synth.numel("swiglu_bf16_4x4096x14336") == 234881024
    assert synth.numel("stress_2p28") == 1 << 28


@pytest.mark.parametrize("name", ["gelu_tanh_fp32_4x128x3072", "gelu_erf_bf16_32x512x3072",
                                  "silu_bf16_8x2048x11008", "swiglu_bf16_4x4096x14336"])
def test_workloads_are_seeded_and_shaped(name):
    n = 200000
    a, b = synth.make(name, n=n), synth.make(name, n=n)
    keys = [k for k in a if isinstance(a[k], np.ndarray)]
    assert keys and all(np.array_equal(a[k], b[k]) for k in keys)
    assert all(a[k].size == n for k in keys)
    dtype = a["dtype"]
    assert all(a[k].dtype == (np.float32 if dtype == "fp32" else np.uint16) for k in keys)
    x = synth.storage_to_f64(a["x" if "x" in a else "gate"], dtype)
    if name == "gelu_erf_bf16_32x512x3072":
        assert abs(x.std() - 1.5) < 0.02
        assert abs(synth.storage_to_f64(a["grad_y"], dtype).std() - 0.02) < 1e-3
    elif name == "silu_bf16_8x2048x11008":
        # 10 % of the elements come from U[-6, -0.5]: the left-branch share is well above a Gaussian's
        assert 0.28 < (x < -1.2785).mean() < 0.36 and x.min() > -12
    elif name == "swiglu_bf16_4x4096x14336":
        assert abs(x.std() - 1.0) < 0.01
        assert abs(synth.storage_to_f64(a["grad_h"], dtype).std() - 0.01) < 5e-4
        assert not np.array_equal(a["gate"], a["up"])
    else:
        assert abs(x.std() - 1.0) < 0.01


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_stress_workload_structure(dtype):
    T = -0.75179154
    n = 1 << 21
    w = synth.make("stress_2p28", n=n, kind="gelu_erf", dtype=dtype, T=T)
    x = synth.storage_to_f64(w["x"], dtype)
    dense = n // 4
    assert np.all(np.abs(x[:dense] - T) <= 0.05 + 1e-2)                  # dense block around the minimum
    tail = x[dense + 400:]
    assert 0.005 < (tail == 0).mean() < 0.02                              # 1 % exact zeros
    assert np.abs(tail).max() > 50                                        # heavy tails (Student-t, 3 degrees)
    near = x[dense:dense + 300]
    assert np.any(near == np.float64(np.float32(T))) or dtype == "bf16"   # T itself and its neighbours follow
    assert np.any(near == 0.0)


def test_storage_conversions_are_exact_and_round_to_nearest_even():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(1 << 16) * 10.0 ** rng.integers(-30, 30, 1 << 16)).astype(np.float32)
    bits = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    big = np.tile(x, 1 << 7)                                              # takes the multi-threaded path
    assert np.array_equal(synth.to_storage(big, "bf16"), np.tile(ref, 1 << 7))
    back = synth.bf16_bits_to_f32(bits)
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)            # fixed point
    assert np.array_equal(synth.f64_to_storage_exact(back.astype(np.float64), "bf16"), bits)
    assert np.array_equal(synth.storage_to_f64(x, "fp32"), x.astype(np.float64))
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], np.float32)  # ties go to even
    assert list(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(ties))) == [1.0, 1.0 + 2.0 ** -6]
    nb = synth.neighbours(-0.75, "bf16", 2)
    assert list(nb) == [-0.7421875, -0.74609375, -0.75, -0.75390625, -0.7578125]


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_bench_takes_its_traffic_figure_from_the_committed_profile():
    """`roofline.traffic` is the HBM byte count of the rocprofv3 counter runs summarised under profiles/:
    bench.py reads it from there, and the figure must be the sum of that file's own read and write columns."""
    import re
    sys.path.insert(0, ROOT)
    import bench
    text = open(os.path.join(ROOT, bench.PROFILE)).read()
    row = re.search(r"^\| swiglu_invact_bwd \| ([0-9.]+) \| ([0-9.]+) \| ([0-9.]+) \| ([0-9.]+) \|", text, re.M)
    assert row, "the profile's traffic table has no backward row"
    read_mb, write_mb, total_mb, algorithmic_mb = map(float, row.groups())
    assert abs(read_mb + write_mb - total_mb) < 0.11
    assert bench.profiled_traffic() == pytest.approx(total_mb * 1e6, rel=1e-4)
    assert algorithmic_mb == pytest.approx(synth.numel(bench.WORKLOAD) * bench.BYTES_BWD / 1e6, rel=1e-4)
    assert 1.0 <= total_mb / algorithmic_mb < 1.05        # no wasted re-reads to speak of
