"""Seeded synthetic input generators for the V-ABFT verified-GEMM workloads.

This module holds NO arithmetic of the method (no checksums, statistics,
thresholds, hashes or bit flips).  It only draws matrices from documented
distributions and rounds them to the storage type of a configuration.  It is
the one module that both the CPU oracle's tests and the HIP path's tests /
benchmark import; the oracle and the HIP path share nothing else.

Storage conventions returned by every generator
  "f64"  -> numpy float64 array
  "f32"  -> numpy float32 array
  "f16"  -> numpy float16 array (IEEE binary16, round-to-nearest-even)
  "bf16" -> numpy uint16 array holding bfloat16 bit patterns
            (round-to-nearest-even from float32)

Distributions follow the paper's evaluation set-up (section "Experimental
Setup", "Distributions tested") and the five benchmark configurations:
N(mu, sigma), U(lo, hi), |N(1,1)| (the calibration protocol's positive
matrices), truncated normals (true truncation by rejection, not clipping) and
"outlier channel" activations (a seeded 1 % of the K columns scaled by 20).
"""
from __future__ import annotations

import numpy as np

DTYPES = ("f64", "f32", "f16", "bf16")


def rng(seed: int, stream: int = 0) -> np.random.Generator:
    """Counter-based generator; (seed, stream) name an independent stream."""
    return np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), int(stream)]))


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float64 sample to the storage type of a configuration."""
    if dtype == "f64":
        return np.ascontiguousarray(x, dtype=np.float64)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))
    if dtype == "f8":
        return f64_to_e4m3_bits(np.asarray(x, dtype=np.float64))
    if dtype == "f8e5m2":
        return f64_to_e5m2_bits(np.asarray(x, dtype=np.float64))
    raise ValueError(f"unknown dtype {dtype!r}")


def _e4m3_positive_values() -> np.ndarray:
    """The 127 finite non-negative values of OCP FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3
    mantissa bits, no infinities, code 0x7F is NaN), indexed by code 0x00 .. 0x7E."""
    codes = np.arange(0x7F)
    e, m = codes >> 3, codes & 7
    return np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7))


def f64_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code, ties to the even code, magnitudes beyond 448 saturate to +-448 (uint8)."""
    vals = _e4m3_positive_values()
    a = np.minimum(np.abs(x), vals[-1])
    hi = np.clip(np.searchsorted(vals, a, side="left"), 1, len(vals) - 1)
    lo = hi - 1
    dlo, dhi = a - vals[lo], vals[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code = np.where(a == 0, 0, code).astype(np.uint8)
    return (code | np.where(np.signbit(x), 0x80, 0).astype(np.uint8)).astype(np.uint8)


def f64_to_e5m2_bits(x: np.ndarray) -> np.ndarray:
    """Nearest OCP FP8 E5M2 code (1 sign, 5 exponent bits with bias 15, 2 mantissa bits; codes 0x00 .. 0x7B are the
    finite non-negative values in increasing order), ties to the even code, magnitudes beyond 57344 saturate to
    +-57344 (uint8)."""
    codes = np.arange(0x7C)
    e, m = codes >> 2, codes & 3
    vals = np.where(e == 0, m * 2.0 ** -16, (1.0 + m / 4.0) * 2.0 ** (e.astype(np.float64) - 15))
    a = np.minimum(np.abs(x), vals[-1])
    hi = np.clip(np.searchsorted(vals, a, side="left"), 1, len(vals) - 1)
    lo = hi - 1
    dlo, dhi = a - vals[lo], vals[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code = np.where(a == 0, 0, code).astype(np.uint8)
    return (code | np.where(np.signbit(x), 0x80, 0).astype(np.uint8)).astype(np.uint8)


# --------------------------------------------------------------------------
# distributions (all return float64 samples of the requested shape)
# --------------------------------------------------------------------------
def normal(g: np.random.Generator, shape, mean=0.0, std=1.0) -> np.ndarray:
    return g.normal(mean, std, size=shape)


def uniform(g: np.random.Generator, shape, lo=-1.0, hi=1.0) -> np.ndarray:
    return g.uniform(lo, hi, size=shape)


def abs_normal(g: np.random.Generator, shape, mean=1.0, std=1.0) -> np.ndarray:
    """|N(mean, std)|: the positive matrices of the calibration protocol."""
    return np.abs(g.normal(mean, std, size=shape))


def truncated_normal(g: np.random.Generator, shape, mean=0.0, std=1.0, bound_sigmas=1.0) -> np.ndarray:
    """N(mean, std) conditioned on |x - mean| <= bound_sigmas * std (rejection)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float64)
    filled = 0
    while filled < n:
        need = n - filled
        z = g.normal(0.0, 1.0, size=int(need * 1.6) + 16)
        z = z[np.abs(z) <= bound_sigmas][:need]
        out[filled:filled + z.size] = z
        filled += z.size
    return (mean + std * out).reshape(shape)


def outlier_activations(g: np.random.Generator, shape, frac=0.01, scale=20.0):
    """N(0,1) activations with round(frac*K) seeded columns multiplied by scale.

    Returns (sample, outlier_column_indices)."""
    m, k = shape
    x = g.normal(0.0, 1.0, size=shape)
    n_out = int(round(frac * k))
    cols = np.sort(g.choice(k, size=n_out, replace=False))
    x[:, cols] *= scale
    return x, cols


# --------------------------------------------------------------------------
# the benchmark configurations
# --------------------------------------------------------------------------
CONFIGS = {
    # name: dtype, M, N, K, transB
    "c1_f32_256": dict(dtype="f32", M=256, N=256, K=256, transB=0),
    "c2_bf16_4096": dict(dtype="bf16", M=4096, N=4096, K=4096, transB=0),
    "c3_bf16_ffn": dict(dtype="bf16", M=4096, N=11008, K=4096, transB=1),
    "c4_f16_8192": dict(dtype="f16", M=8192, N=8192, K=8192, transB=0),
    "c5_f64_2048": dict(dtype="f64", M=2048, N=2048, K=2048, transB=0),
    # beyond the five benchmark configurations: FP8 E4M3 inputs, FP32 accumulation, FP16 output
    "c6_f8_4096": dict(dtype="f8", M=4096, N=4096, K=4096, transB=1),
    "c8_f8e5m2_4096": dict(dtype="f8e5m2", M=4096, N=4096, K=4096, transB=1),
    # ... and an FP32 problem large enough to be bound by the FP32 matrix instruction rather than by latency
    "c7_f32_4096": dict(dtype="f32", M=4096, N=4096, K=4096, transB=0),
}


def make_config(name: str, seed: int = 0, variant: int = 0, shape=None):
    """Inputs of one trial of a benchmark configuration.

    Returns dict(dtype, M, N, K, transB, A, B) with A of shape (M, K) and B of
    shape (K, N) when transB == 0, or (N, K) when transB == 1 (the "weight"
    layout), both already rounded to storage.  `shape=(M, N, K)` overrides
    the size (used by tests to run a configuration's distributions at a size
    the oracle finishes quickly).  `variant` selects the second B of c5.
    """
    cfg = dict(CONFIGS[name])
    if shape is not None:
        cfg["M"], cfg["N"], cfg["K"] = (int(v) for v in shape)
    M, N, K, dt = cfg["M"], cfg["N"], cfg["K"], cfg["dtype"]
    ga, gb = rng(seed, 1), rng(seed, 2)
    if name in ("c1_f32_256", "c2_bf16_4096", "c7_f32_4096"):
        A = normal(ga, (M, K))
        B = normal(gb, (K, N))
    elif name == "c3_bf16_ffn":
        A, cols = outlier_activations(ga, (M, K))
        cfg["outlier_cols"] = cols
        # weights drawn directly in the (N, K) layout a linear layer stores
        B = truncated_normal(gb, (N, K), 0.0, 0.02, 2.0)
    elif name in ("c6_f8_4096", "c8_f8e5m2_4096"):
        A = normal(ga, (M, K))
        B = normal(gb, (N, K))  # weight layout
    elif name == "c4_f16_8192":
        A = uniform(ga, (M, K))
        B = uniform(gb, (K, N))
    elif name == "c5_f64_2048":
        A = normal(ga, (M, K))
        if variant == 0:
            B = truncated_normal(gb, (K, N), 0.0, 1.0, 3.0)
        else:
            B = uniform(gb, (K, N), 0.0, 1.0)
    else:
        raise KeyError(name)
    cfg["A"] = to_storage(A, dt)
    cfg["B"] = to_storage(B, dt)
    return cfg


def paper_distribution(g: np.random.Generator, which: str, shape) -> np.ndarray:
    """The four fault-free test distributions of the paper's evaluation."""
    if which == "n_1e-6_1":
        return normal(g, shape, 1e-6, 1.0)
    if which == "n_1_1":
        return normal(g, shape, 1.0, 1.0)
    if which == "u_-1_1":
        return uniform(g, shape, -1.0, 1.0)
    if which == "trunc_n_0_1":
        return truncated_normal(g, shape, 0.0, 1.0, 1.0)
    if which == "u_0_1":
        return uniform(g, shape, 0.0, 1.0)
    if which == "abs_n_1_1":
        return abs_normal(g, shape)
    raise KeyError(which)


PAPER_DISTRIBUTIONS = ("n_1e-6_1", "n_1_1", "u_-1_1", "trunc_n_0_1")


# --------------------------------------------------------------------------
# the same configurations drawn on the device (fresh matrices for many-trial statistics)
# --------------------------------------------------------------------------
def _device_truncated_normal(torch, g, shape, std, bound_sigmas, dtype):
    """N(0, std) conditioned on |x| <= bound_sigmas * std, by rejection (rejected entries are redrawn)."""
    z = torch.randn(shape, generator=g, device="cuda", dtype=dtype)
    while True:
        bad = z.abs() > bound_sigmas
        n_bad = int(bad.sum().item())
        if n_bad == 0:
            break
        z[bad] = torch.randn(n_bad, generator=g, device="cuda", dtype=dtype)
    return z.mul_(std)


def device_trial(name: str, g, variant: int = 0, shape=None):
    """One trial's (A, B) of a benchmark configuration as torch tensors on the GPU, in storage type and layout,
    from the torch generator `g` (seeded by the caller).  Same distributions as make_config: N(0,1);
    c3: round(0.01 K) seeded outlier columns of A times 20 and weights N(0, 0.02) truncated at 2 sigma by
    rejection, N x K layout; c4: U(-1,1); c5: B ~ N(0,1) truncated at 3 sigma (variant 0) or U(0,1) (variant 1)."""
    import torch

    cfg = dict(CONFIGS[name])
    if shape is not None:
        cfg["M"], cfg["N"], cfg["K"] = (int(v) for v in shape)
    M, N, K, dt, tb = cfg["M"], cfg["N"], cfg["K"], cfg["dtype"], cfg["transB"]
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32, "f64": torch.float64,
           "f8": torch.float8_e4m3fn, "f8e5m2": torch.float8_e5m2}[dt]
    gen = torch.float64 if dt == "f64" else torch.float32
    bshape = (N, K) if tb else (K, N)
    if name in ("c1_f32_256", "c2_bf16_4096", "c6_f8_4096", "c7_f32_4096", "c8_f8e5m2_4096"):
        A = torch.randn((M, K), generator=g, device="cuda", dtype=gen)
        B = torch.randn(bshape, generator=g, device="cuda", dtype=gen)
    elif name == "c3_bf16_ffn":
        A = torch.randn((M, K), generator=g, device="cuda", dtype=gen)
        cols = torch.randperm(K, generator=g, device="cuda")[:int(round(0.01 * K))]
        A[:, cols] *= 20.0
        B = _device_truncated_normal(torch, g, bshape, 0.02, 2.0, gen)
    elif name == "c4_f16_8192":
        A = torch.rand((M, K), generator=g, device="cuda", dtype=gen).mul_(2.0).sub_(1.0)
        B = torch.rand(bshape, generator=g, device="cuda", dtype=gen).mul_(2.0).sub_(1.0)
    elif name == "c5_f64_2048":
        A = torch.randn((M, K), generator=g, device="cuda", dtype=gen)
        B = (_device_truncated_normal(torch, g, bshape, 1.0, 3.0, gen) if variant == 0 else
             torch.rand(bshape, generator=g, device="cuda", dtype=gen))
    else:
        raise KeyError(name)
    return A.to(tdt), B.to(tdt)
