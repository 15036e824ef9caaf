"""Seeded synthetic activation tensors shaped like ViT stage-boundary outputs.

These stand in for the ImageNet activations of a trained ViT that the paper
quantizes (Sec. 3, Sec. 4.1): shapes are [microbatch, tokens, hidden] and the
value distributions are heavy-tailed and outlier-bearing, which is the regime
the paper describes for naive PTQ versus ACIQ (Sec. 3, "Naive PTQ and ACIQ").

This module holds no arithmetic of the method itself (no statistics, clipping,
quantization or packing); it only draws numbers.  Both the CPU oracle's tests
and the HIP path's tests and benchmark import it so that the two sides see the
same host arrays.

Everything is drawn with numpy.random.default_rng(seed) (PCG64) in float64 and
cast once to float32 (round to nearest even); bf16 tensors are the float32
values rounded to nearest even on the upper 16 bits and returned as uint16.
"""
from __future__ import annotations

import math

import numpy as np

# name -> (shape, dtype, seed)
CONFIG_SHAPES = {
    "C1": ((1, 197, 768), "f32", 0),
    "C2": ((64, 197, 768), "f32", 1),
    "C3": ((64, 197, 1024), "f32", 2),
    "C4": ((32, 257, 1280), "f32", 3),
    "C5": ((256, 577, 1024), "bf16", 4),
}
CONFIG_BITS = {
    "C1": (2, 4, 8),
    "C2": (2, 3, 4, 6, 8, 16),
    "C3": (2, 4, 8),
    "C4": (2, 4, 6, 8, 16),
    "C5": (2, 3, 4, 8),
}


def numel(name: str) -> int:
    return int(np.prod(CONFIG_SHAPES[name][0]))


def f32_to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _scale_outliers(x: np.ndarray, rng: np.random.Generator, frac: float, factor: float) -> None:
    k = int(round(frac * x.size))
    if k > 0:
        idx = rng.choice(x.size, size=k, replace=False)
        x[idx] *= factor


def laplace_outliers(n: int, seed: int, b: float = 0.5, frac: float = 0.001, factor: float = 20.0) -> np.ndarray:
    """C1 recipe: Laplace(0, b) with a fraction of the values multiplied by `factor`."""
    rng = np.random.default_rng(seed)
    x = rng.laplace(0.0, b, size=n)
    _scale_outliers(x, rng, frac, factor)
    return x.astype(np.float32)


def laplace_gauss_mixture(n: int, seed: int, p_laplace: float = 0.7, b: float = 0.4,
                          g_mean: float = 0.1, g_std: float = 1.0,
                          frac: float = 0.0005, factor: float = 30.0) -> np.ndarray:
    """C2 recipe: per element Laplace(0,b) with prob. p else N(g_mean,g_std); outliers scaled."""
    rng = np.random.default_rng(seed)
    pick = rng.random(n) < p_laplace
    lap = rng.laplace(0.0, b, size=n)
    gau = rng.normal(g_mean, g_std, size=n)
    x = np.where(pick, lap, gau)
    del lap, gau, pick
    _scale_outliers(x, rng, frac, factor)
    return x.astype(np.float32)


def post_gelu(n: int, seed: int, std: float = 1.5) -> np.ndarray:
    """C3 recipe: exact (erf) GELU of N(0, std): skewed, one-sided, spike near zero."""
    from scipy.special import erf  # library routine, used only to shape the inputs
    rng = np.random.default_rng(seed)
    g = rng.normal(0.0, std, size=n)
    x = g * 0.5 * (1.0 + erf(g / math.sqrt(2.0)))
    return x.astype(np.float32)


def unit_laplace(n: int, seed: int) -> np.ndarray:
    """C4 base buffer: Laplace(0, 1); the stream scales it per microbatch."""
    rng = np.random.default_rng(seed)
    return rng.laplace(0.0, 1.0, size=n).astype(np.float32)


def student_t_bf16(n: int, seed: int, df: float = 3.0, scale: float = 0.5) -> np.ndarray:
    """C5 recipe: Student-t(df) * scale, stored as bfloat16 bit patterns (uint16)."""
    rng = np.random.default_rng(seed)
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        m = min(step, n - s)
        out[s:s + m] = f32_to_bf16_bits((rng.standard_t(df, size=m) * scale).astype(np.float32))
    return out


def make_config(name: str, n: int | None = None) -> np.ndarray:
    """Flattened tensor of BASELINE config `name` (or its first-n-sized analogue).

    Returns float32, except C5 which returns bfloat16 bit patterns as uint16.
    For C4 this is microbatch 0's base buffer (unit Laplace); see c4_stream().
    """
    shape, _, seed = CONFIG_SHAPES[name]
    n = int(np.prod(shape)) if n is None else int(n)
    if name == "C1":
        return laplace_outliers(n, seed)
    if name == "C2":
        return laplace_gauss_mixture(n, seed)
    if name == "C3":
        return post_gelu(n, seed)
    if name == "C4":
        return unit_laplace(n, seed)
    if name == "C5":
        return student_t_bf16(n, seed)
    raise KeyError(name)


def c4_stream(n_microbatches: int = 500, seed: int = 3, ring: int = 8,
              images: int = 32, rate: float = 100.0, n_per_mb: int | None = None):
    """C4 recipe: per-microbatch (ring buffer index, Laplace b, bandwidth Mbit/s, bitwidth).

    Bandwidth is a seeded random walk in log space clipped to [5, 1000] Mbit/s.
    The bitwidth is the largest of {2,4,6,8,16} whose payload n*k bits fits in
    what the link carries during one microbatch period images/rate seconds,
    else 2.  (A stand-in for the paper's controller, Eq. 2, which also picks the
    highest bitwidth that sustains the target rate.)
    """
    n_per_mb = numel("C4") if n_per_mb is None else n_per_mb
    rng = np.random.default_rng(seed + 1000)
    b = rng.uniform(0.2, 2.0, size=n_microbatches)
    steps = rng.normal(0.0, 0.25, size=n_microbatches)
    logbw = np.empty(n_microbatches)
    cur = math.log(200.0)
    lo, hi = math.log(5.0), math.log(1000.0)
    for m in range(n_microbatches):
        cur = min(max(cur + steps[m], lo), hi)
        logbw[m] = cur
    bw = np.exp(logbw)
    budget_bits = bw * 1e6 * (images / rate)
    bits = np.full(n_microbatches, 2, dtype=np.int64)
    for k in (4, 6, 8, 16):
        bits[n_per_mb * k <= budget_bits] = k
    return [(m % ring, float(b[m]), float(bw[m]), int(bits[m])) for m in range(n_microbatches)]


# Small adversarial inputs used by both sides' edge-case tests -----------------

def edge_cases(seed: int = 7):
    """(name, float32 array) pairs: ragged sizes, degenerate and extreme tensors."""
    rng = np.random.default_rng(seed)
    out = []
    for n in (1, 2, 3, 5, 31, 32, 33, 63, 255, 257, 1023, 1025, 4097, 8191, 8193, 70001):
        out.append((f"laplace_n{n}", rng.laplace(0.0, 0.7, size=n).astype(np.float32)))
    out.append(("constant", np.full(1000, 1.25, dtype=np.float32)))
    out.append(("zeros", np.zeros(777, dtype=np.float32)))
    out.append(("all_negative", (-np.abs(rng.normal(3.0, 1.0, size=5000)) - 0.5).astype(np.float32)))
    x = rng.laplace(0.0, 0.1, size=20000).astype(np.float32)
    x[1234] = 1.0e6
    out.append(("huge_outlier", x))
    out.append(("two_point", np.tile(np.array([-2.0, 2.0], dtype=np.float32), 3000)))
    out.append(("tiny_values", (rng.laplace(0.0, 1.0, size=3000) * 1e-30).astype(np.float32)))
    out.append(("large_values", (rng.laplace(0.0, 1.0, size=3000) * 1e30).astype(np.float32)))
    out.append(("ramp", np.arange(6000, dtype=np.float32)))
    # so small that the clipping range is a subnormal float and its reciprocal overflows
    out.append(("subnormal_values", (rng.laplace(0.0, 1.0, size=3000) * 1e-41).astype(np.float32)))
    return out
