"""Seeded synthetic gradients shaped like the paper's workloads (Section 4.1, Table 2: sparse
linear-model gradients over millions of features, plus dense per-layer gradients).

This module holds input generation only -- none of the codec's arithmetic -- so both the HIP path's
tests and the CPU oracle's tests may draw their inputs from it.  The paper's datasets are not
available, so these stand in for them.  Every draw uses numpy's Generator(PCG64(seed)); values are
drawn in float64 and cast to float32; "N(0, x)" and "Laplace(0, x)" take x as the standard
deviation and the scale respectively.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

TAU = 128       # paper default (Section 4.2, effect of tau)
FLAG_BITS = 2   # paper default (Table 6)


@dataclass
class Workload:
    name: str
    keys: np.ndarray                 # uint32, strictly increasing (per segment)
    values: np.ndarray               # float32
    dim: int                         # D_m, the dense dimension the keys index into
    seg_offsets: Optional[np.ndarray] = None   # uint64 [n_segments+1] for a segmented batch
    meta: dict = field(default_factory=dict)


def solve_base(values: np.ndarray, keep_fraction: float, tau: int = TAU) -> float:
    """Base b for which about `keep_fraction` of `values` pass the threshold filter.

    The filter keeps |v| >= sum/b^tau, so b = (sum / x)^(1/tau) with x the ceil(p*n)-th largest |v|.
    This is parameter selection for the benchmark, not part of the codec: the result is handed to
    both sides as a float64 and only has to land near the target.  Clamped to the library's range.
    """
    a = np.abs(values.astype(np.float64))
    n = a.size
    k = min(max(int(np.ceil(keep_fraction * n)), 1), n)
    x = np.partition(a, n - k)[n - k]
    s = float(a.sum())
    if not (x > 0.0) or not (s > 0.0):
        return 1.1
    b = (s / x) ** (1.0 / tau) * (1.0 + 1e-9)
    return float(min(max(b, 1.0 + 2.0 ** -19), 16.0))


def solve_bases(values: np.ndarray, keep_fractions, tau: int = TAU) -> List[float]:
    """solve_base for several keep fractions with one partition of |values| (large arrays)."""
    a = np.abs(values)                                   # float32: the order statistics are exact
    n = a.size
    s = float(a.sum(dtype=np.float64))
    ks = [min(max(int(np.ceil(f * n)), 1), n) for f in keep_fractions]
    part = np.partition(a, sorted(set(n - k for k in ks)))
    out = []
    for k in ks:
        x = float(part[n - k])
        b = (s / x) ** (1.0 / tau) * (1.0 + 1e-9) if x > 0.0 and s > 0.0 else 1.1
        out.append(float(min(max(b, 1.0 + 2.0 ** -19), 16.0)))
    return out


def config1(seed: int = 1001, dim: int = 1_000_000, nnz: int = 100_000) -> Workload:
    """Tiny sparse gradient: uniform keys without replacement, Laplace(0, 1e-3) values."""
    rng = np.random.Generator(np.random.PCG64(seed))
    keys = np.sort(rng.choice(dim, nnz, replace=False)).astype(np.uint32)
    values = rng.laplace(0.0, 1e-3, nnz).astype(np.float32)
    return Workload("c1_tiny_sparse", keys, values, dim, meta={"keep": [0.10]})


def config2(seed: int = 1002, n: int = 25_600_000) -> Workload:
    """Dense flat gradient of a 25.6M-parameter model: N(0,1e-4) with 1% outliers N(0,1e-2)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    values = rng.normal(0.0, 1e-4, n)
    out = rng.random(n) < 0.01
    values[out] = rng.normal(0.0, 1e-2, int(out.sum()))
    return Workload("c2_dense_25m", np.arange(n, dtype=np.uint32), values.astype(np.float32), n,
                    meta={"keep": [0.01]})


def zipf_gaps(rng, count: int, s: float, target_mean: float) -> np.ndarray:
    """iid gaps from Zipf(s) truncated to {1..Gmax}, Gmax the largest support with mean <= target."""
    g = np.arange(1, 100_000, dtype=np.float64)
    w = g ** (-s)
    means = np.cumsum(g * w) / np.cumsum(w)
    gmax = int(np.searchsorted(means, target_mean, side="right"))  # means[gmax-1] <= target
    gmax = max(gmax, 1)
    cdf = np.cumsum(w[:gmax]) / np.sum(w[:gmax])
    u = rng.random(count)
    return (np.searchsorted(cdf, u, side="right") + 1).clip(1, gmax).astype(np.int64)


def config3(seed: int = 1003, dim: int = 100_000_000, nnz: int = 10_000_000) -> Workload:
    """High-dimensional sparse linear-model gradient: Zipf(1.2) key gaps, Laplace(0,1e-5) values."""
    rng = np.random.Generator(np.random.PCG64(seed))
    gaps = zipf_gaps(rng, nnz, 1.2, 0.99 * dim / nnz)
    keys64 = np.cumsum(gaps) - 1
    assert keys64[-1] < dim, "truncated Zipf gaps overran the dimension"
    values = rng.laplace(0.0, 1e-5, nnz).astype(np.float32)
    return Workload("c3_sparse_zipf", keys64.astype(np.uint32), values, dim, meta={"keep": [0.001]})


def config4(seed: int = 1004, n: int = 124_000_000) -> Workload:
    """Large dense flat gradient: 90% N(0,1e-5) + 10% N(0,1e-3); keep fractions are swept."""
    rng = np.random.Generator(np.random.PCG64(seed))
    values = np.empty(n, np.float32)
    step = 1 << 24
    for lo in range(0, n, step):   # chunked so the float64 temporaries stay small
        m = min(step, n - lo)
        z = rng.standard_normal(m)
        wide = rng.random(m) < 0.10
        values[lo:lo + m] = (z * np.where(wide, 1e-3, 1e-5)).astype(np.float32)
    return Workload("c4_dense_124m", np.arange(n, dtype=np.uint32), values, n,
                    meta={"keep": [0.10, 0.01, 0.001, 0.0001]})


def config5(seed: int = 1005, n_tensors: int = 160, lo: int = 4096, hi: int = 4_194_304,
            total_range=(57_000_000, 63_000_000)) -> Workload:
    """Per-layer segmented batch: log-uniform tensor sizes, per-tensor Laplace scale log-uniform
    in [1e-6, 1e-2], keys 0..n_i-1 in every tensor."""
    rng = np.random.Generator(np.random.PCG64(seed))
    target = 0.5 * (total_range[0] + total_range[1])
    sizes = np.exp(rng.uniform(np.log(lo), np.log(hi), n_tensors))
    sizes = np.clip(np.round(sizes * (target / sizes.sum())), lo, hi).astype(np.int64)
    for _ in range(64):            # clipping moves the total a little: pull it back into range
        total = int(sizes.sum())
        if total_range[0] <= total <= total_range[1]:
            break
        sizes = np.clip(np.round(sizes * (target / total)), lo, hi).astype(np.int64)
    scales = np.exp(rng.uniform(np.log(1e-6), np.log(1e-2), n_tensors))
    offs = np.zeros(n_tensors + 1, np.uint64)
    offs[1:] = np.cumsum(sizes)
    total = int(offs[-1])
    keys = np.empty(total, np.uint32)
    values = np.empty(total, np.float32)
    for i in range(n_tensors):
        a, b = int(offs[i]), int(offs[i + 1])
        keys[a:b] = np.arange(b - a, dtype=np.uint32)
        values[a:b] = rng.laplace(0.0, scales[i], b - a).astype(np.float32)
    return Workload("c5_segmented", keys, values, int(sizes.max()), seg_offsets=offs,
                    meta={"keep": [0.01], "scales": scales})


def small_mixture(seed: int, n: int, dim: Optional[int] = None) -> Workload:
    """Reduced-size stand-in used by parity tests: sparse sorted keys, heavy-tailed values spanning
    many binades (a few exact zeros and denormals included)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    dim = dim or max(4 * n, 16)
    keys = np.sort(rng.choice(dim, n, replace=False)).astype(np.uint32) if n else np.zeros(0, np.uint32)
    scale = np.exp(rng.uniform(np.log(1e-7), np.log(1e-2), n))
    values = (rng.laplace(0.0, 1.0, n) * scale).astype(np.float32)
    if n >= 64:
        values[rng.integers(0, n, n // 64)] = 0.0
        values[rng.integers(0, n, 4)] = np.float32(1e-42)   # denormal
    return Workload(f"small_{seed}_{n}", keys, values, dim)
