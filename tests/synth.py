"""Seeded synthetic inputs for the tests and the benchmark.

Holds none of the method's arithmetic: only random draws, the storage-format
conversions (binary32 <-> bfloat16 bit patterns) and the list of workloads.
Both the CPU oracle's tests and the GPU path's tests draw from here, so that
the two sides always see the same bits.

The workloads stand in for the transformer-MLP activation tensors the paper
measures on (BERT / Llama MLP blocks, Appendix "Experiment Setups"); models
and datasets are not used.
"""
import numpy as np

# name -> kind, storage dtype, shape.  Element count is the product of shape.
WORKLOADS = {
    # small parity case
    "gelu_tanh_fp32_4x128x3072": dict(kind="gelu_tanh", dtype="fp32", shape=(4, 128, 3072)),
    # BERT-base MLP activation
    "gelu_erf_bf16_32x512x3072": dict(kind="gelu_erf", dtype="bf16", shape=(32, 512, 3072)),
    # standalone SiLU, Llama-2-7B-like intermediate width
    "silu_bf16_8x2048x11008": dict(kind="silu", dtype="bf16", shape=(8, 2048, 11008)),
    # Llama-3-8B SwiGLU activation (headline)
    "swiglu_bf16_4x4096x14336": dict(kind="silu", dtype="bf16", shape=(4, 4096, 14336), gated=True),
    # accuracy-stress / peak-bandwidth sweep
    "stress_2p28": dict(kind=None, dtype=None, shape=(1 << 28,)),
}


def numel(name):
    return int(np.prod(WORKLOADS[name]["shape"]))


# ----------------------------------------------------------------------
# storage formats
# ----------------------------------------------------------------------

def f32_to_bf16_bits(x):
    """binary32 array -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = ((u + (0x7FFF + ((u >> 16) & 1))) >> 16).astype(np.uint16)
    r[nan] = ((u[nan] >> 16) | 0x0040).astype(np.uint16)
    return r


def bf16_bits_to_f32(b):
    """bfloat16 bit patterns (uint16) -> binary32 array (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def to_storage(x32, dtype):
    """binary32 values -> storage array: float32 for fp32, uint16 bit patterns for bf16."""
    if dtype == "fp32":
        return np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "bf16":
        x32 = np.ascontiguousarray(x32, dtype=np.float32)
        if x32.size >= 1 << 22:
            # same rounding (nearest even), multi-threaded; tests check the two against each other
            import torch
            return torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        return f32_to_bf16_bits(x32)
    raise ValueError(dtype)


def storage_to_f64(a, dtype):
    """storage array -> float64 array holding the exact stored values."""
    if dtype == "fp32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    raise ValueError(dtype)


def f64_to_storage_exact(v, dtype):
    """float64 values that already lie on the storage grid -> storage array."""
    v32 = np.asarray(v, dtype=np.float64).astype(np.float32)
    if dtype == "fp32":
        return v32
    return (v32.view(np.uint32) >> 16).astype(np.uint16)


# ----------------------------------------------------------------------
# random draws
# ----------------------------------------------------------------------

_CHUNK = 1 << 24


def normal(n, seed, std=1.0):
    rng = np.random.default_rng(seed)
    out = np.empty(n, dtype=np.float32)
    for o in range(0, n, _CHUNK):
        m = min(_CHUNK, n - o)
        out[o:o + m] = rng.standard_normal(m, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def silu_mixture(n, seed):
    """90 % N(0, 2^2) + 10 % U[-6, -0.5], chosen per element by a Bernoulli(0.1) draw."""
    rng = np.random.default_rng(seed)
    out = np.empty(n, dtype=np.float32)
    for o in range(0, n, _CHUNK):
        m = min(_CHUNK, n - o)
        g = rng.standard_normal(m, dtype=np.float32) * np.float32(2.0)
        u = rng.random(m, dtype=np.float32) * np.float32(5.5) - np.float32(6.0)
        pick = rng.random(m, dtype=np.float32) < np.float32(0.1)
        out[o:o + m] = np.where(pick, u, g)
    return out


def neighbours(center, dtype, radius=64):
    """All representable values of `dtype` within +-radius ulps of `center` (binary32 array)."""
    c = np.float32(center)
    if dtype == "fp32":
        u = int(np.array([c], dtype=np.float32).view(np.uint32)[0])
        pats = np.arange(u - radius, u + radius + 1, dtype=np.int64).astype(np.uint32)
        return pats.view(np.float32)
    b = int(f32_to_bf16_bits(np.array([c], dtype=np.float32))[0])
    pats = np.arange(b - radius, b + radius + 1, dtype=np.int64).astype(np.uint16)
    return bf16_bits_to_f32(pats)


_heavy_cache = {}


def heavy_tailed(n, seed):
    """2 * Student-t(3) with 1 % exact zeros (cached: the 2^28 draw takes a while)."""
    if (n, seed) not in _heavy_cache:
        rng = np.random.default_rng(seed)
        out = np.empty(n, dtype=np.float32)
        for o in range(0, n, _CHUNK):
            m = min(_CHUNK, n - o)
            t = (2.0 * rng.standard_t(3, m)).astype(np.float32)
            t[rng.random(m, dtype=np.float32) < np.float32(0.01)] = 0.0
            out[o:o + m] = t
        _heavy_cache.clear()
        _heavy_cache[(n, seed)] = out
    return _heavy_cache[(n, seed)]


def stress(n, seed, dtype, T):
    """Heavy-tailed stress input: 2 * Student-t(3) with 1 % exact zeros; the
    first min(2^20, n/4) elements are replaced by a dense block uniform on
    [T-0.05, T+0.05], followed by every representable value within 64 ulps of T
    and of -T, the values next to 0, and +-0 and T themselves."""
    out = heavy_tailed(n, seed).copy()
    rng = np.random.default_rng(seed + 1000)
    dense = min(1 << 20, n // 4)
    if dense:
        out[:dense] = (T - 0.05 + 0.1 * rng.random(dense)).astype(np.float32)
    special = np.concatenate([neighbours(T, dtype), neighbours(0.0, "fp32", 8),
                              neighbours(-T, dtype),
                              np.array([0.0, -0.0, T], dtype=np.float32)])
    k = min(special.size, n - dense)
    out[dense:dense + k] = special[:k]
    return out


# ----------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------

def make(name, n=None, kind=None, dtype=None, T=None):
    """Inputs of workload `name`, as storage arrays (see to_storage), flat.

    n overrides the element count (same recipe, fewer elements).  For the
    stress workload pass kind, dtype and that kind's T.
    Returns a dict with keys among x, grad_y, gate, up, grad_h plus kind,
    dtype, n.
    """
    w = WORKLOADS[name]
    n = numel(name) if n is None else int(n)
    kind = w["kind"] or kind
    dtype = w["dtype"] or dtype
    out = dict(kind=kind, dtype=dtype, n=n, name=name)
    if name == "gelu_tanh_fp32_4x128x3072":
        out["x"] = to_storage(normal(n, 0), dtype)
        out["grad_y"] = to_storage(normal(n, 1), dtype)
    elif name == "gelu_erf_bf16_32x512x3072":
        out["x"] = to_storage(normal(n, 0, 1.5), dtype)
        out["grad_y"] = to_storage(normal(n, 1, 0.02), dtype)
    elif name == "silu_bf16_8x2048x11008":
        out["x"] = to_storage(silu_mixture(n, 0), dtype)
        out["grad_y"] = to_storage(normal(n, 1), dtype)
    elif name == "swiglu_bf16_4x4096x14336":
        out["gate"] = to_storage(normal(n, 0), dtype)
        out["up"] = to_storage(normal(n, 2), dtype)
        out["grad_h"] = to_storage(normal(n, 1, 0.01), dtype)
    elif name == "stress_2p28":
        out["x"] = to_storage(stress(n, 0, dtype, T), dtype)
        out["grad_y"] = to_storage(normal(n, 1), dtype)
    else:
        raise KeyError(name)
    return out
