"""Seeded synthetic workloads for the SD-KDE hot path.

This module only draws inputs (samples, queries, bandwidth); it contains none of the
estimator's arithmetic and is the single piece shared by the CPU oracle's tests and the
HIP path's tests and benchmark.

The paper's experiments use a "simple 16-D Gaussian mixture" with n_test = n_train/8
(Results section) and a 1-D mixture (Appendix A) without stating their parameters; the
mixtures below stand in for them.  The bandwidth follows Silverman's rule of thumb, which
the paper names (Introduction) but does not spell out; the multivariate normal-reference
form is used here.

Draw order for a given seed (numpy Generator, PCG64), all in float64 then cast to fp32:
  1. component means  K x d ~ N(0, 9)
  2. (diagonal-covariance configs only) variances K x d ~ U[0.5, 2]
  3. sample labels, 4. sample normals, 5. query labels, 6. query normals
The 1-D config draws labels (Bernoulli 0.3) and normals for the samples only; its queries are
a uniform grid.
"""
from __future__ import annotations

import dataclasses
import numpy as np


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    n: int
    m: int
    d: int
    kind: str          # "mix_iso" | "mix_diag" | "mix_1d"
    components: int


CONFIGS = {
    "C1": Config("C1", 4096, 1024, 16, "mix_iso", 4),
    "C2": Config("C2", 32768, 32768, 16, "mix_iso", 4),
    "C3": Config("C3", 32768, 65536, 1, "mix_1d", 2),
    "C4": Config("C4", 262144, 65536, 64, "mix_diag", 8),
    "C5": Config("C5", 1048576, 131072, 16, "mix_iso", 4),
}


def silverman_bandwidth(x: np.ndarray) -> float:
    """Normal-reference rule: h = sigma * (4 / ((d + 2) n))^(1 / (d + 4)),
    sigma^2 = mean over dimensions of the unbiased per-dimension sample variance."""
    x = np.asarray(x, dtype=np.float64)
    n, d = x.shape
    sigma = float(np.sqrt(np.mean(np.var(x, axis=0, ddof=1))))
    return sigma * (4.0 / ((d + 2.0) * n)) ** (1.0 / (d + 4.0))


def _mixture(rng, count, means, variances):
    k, d = means.shape
    labels = rng.integers(0, k, size=count)
    z = rng.standard_normal((count, d))
    if variances is None:
        return means[labels] + z
    return means[labels] + z * np.sqrt(variances[labels])


def gaussian_mixture(n: int, m: int, d: int, components: int = 4, seed: int = 0,
                     diag_cov: bool = False):
    """Equal-weight mixture; means ~ N(0, 9 I); unit covariance, or diagonal with variances
    uniform on [0.5, 2] when diag_cov.  Returns (samples[n,d], queries[m,d], h) as fp32/fp32/float."""
    rng = np.random.default_rng(seed)
    means = 3.0 * rng.standard_normal((components, d))
    variances = rng.uniform(0.5, 2.0, size=(components, d)) if diag_cov else None
    x = _mixture(rng, n, means, variances).astype(np.float32)
    q = _mixture(rng, m, means, variances).astype(np.float32)
    return x, q, silverman_bandwidth(x)


def mixture_1d(n: int, m: int, seed: int = 0, lo: float = -5.0, hi: float = 6.0):
    """0.7 N(0,1) + 0.3 N(3, variance 0.25); queries on a uniform grid over [lo, hi]."""
    rng = np.random.default_rng(seed)
    second = rng.random(n) < 0.3
    z = rng.standard_normal(n)
    x = np.where(second, 3.0 + 0.5 * z, z).astype(np.float32).reshape(n, 1)
    q = np.linspace(lo, hi, m).astype(np.float32).reshape(m, 1)
    return x, q, silverman_bandwidth(x)


def mixture_parameters(name: str, seed: int = 0):
    """(weights[K], means[K,d], variances[K,d]) of the mixture that make(name, seed) draws from
    (the same first draws of the same generator)."""
    cfg = CONFIGS[name]
    if cfg.kind == "mix_1d":
        return np.array([0.7, 0.3]), np.array([[0.0], [3.0]]), np.array([[1.0], [0.25]])
    rng = np.random.default_rng(seed)
    means = 3.0 * rng.standard_normal((cfg.components, cfg.d))
    if cfg.kind == "mix_diag":
        variances = rng.uniform(0.5, 2.0, size=(cfg.components, cfg.d))
    else:
        variances = np.ones((cfg.components, cfg.d))
    return np.full(cfg.components, 1.0 / cfg.components), means, variances


def true_log_density(q, weights, means, variances) -> np.ndarray:
    """Log density of the generating mixture at q[m,d] (float64, log-sum-exp over components)."""
    q = np.asarray(q, dtype=np.float64)
    logs = []
    for w, mu, var in zip(weights, means, variances):
        z = (q - mu) ** 2 / var
        logs.append(np.log(w) - 0.5 * z.sum(1) - 0.5 * np.log(2 * np.pi * var).sum())
    logs = np.stack(logs, axis=0)
    top = logs.max(0)
    return top + np.log(np.exp(logs - top).sum(0))


def draw_from_mixture(weights, means, variances, count: int, seed: int) -> np.ndarray:
    """count draws (float64 [count, d]) from the Gaussian mixture with these weights, means [K,d] and diagonal
    variances [K,d]: labels first, then the normals."""
    rng = np.random.default_rng(seed)
    means, variances = np.asarray(means, dtype=np.float64), np.asarray(variances, dtype=np.float64)
    labels = rng.choice(len(weights), size=count, p=np.asarray(weights, dtype=np.float64))
    z = rng.standard_normal((count, means.shape[1]))
    return means[labels] + z * np.sqrt(variances[labels])


def mixture_samples(name: str, n: int, seed: int):
    """n fp32 samples of the mixture that config `name` draws from with seed 0 (fixed true density), the draws
    themselves depending on `seed`; with their rule-of-thumb bandwidth.  For the known-density benchmark."""
    w, mu, var = mixture_parameters(name, 0)
    x = draw_from_mixture(w, mu, var, n, 7919 + seed).astype(np.float32)
    return x, silverman_bandwidth(x)


def standard_normal_cloud(rows: int, d: int, seed: int = 0, scale: float = 1.0) -> np.ndarray:
    """rows x d fp32 draws of N(0, scale^2), generated in fp32 chunk by chunk (for arrays too large to
    go through float64): the index-range tests use it for hundreds of millions of rows."""
    rng = np.random.default_rng(seed)
    out = np.empty((rows, d), dtype=np.float32)
    step = 1 << 22
    for lo in range(0, rows, step):
        hi = min(rows, lo + step)
        out[lo:hi] = rng.standard_normal((hi - lo, d), dtype=np.float32)
    if scale != 1.0:
        out *= np.float32(scale)
    return out


def sample_rows(count: int, extra: int, seed: int = 0) -> np.ndarray:
    """Row indices for sampled checks at sizes where the oracle cannot cover every row: `extra` random rows plus
    the rows next to tile, row-block and split boundaries (first and last rows, powers of two and their
    neighbours from both ends, the eighths of the range).  Sorted, unique."""
    edges = [0, 1, 15, 16, 17, 63, 64, 127, 128, 255, 256, 511, 512, 1023, 1024, 2047, 2048]
    rows = {e for e in edges if e < count}
    rows |= {count - 1 - e for e in edges if e < count}
    rows |= {(count // 8) * k for k in range(1, 8)} | {(count // 8) * k - 1 for k in range(1, 8)}
    rows = {r for r in rows if 0 <= r < count}
    rng = np.random.default_rng(seed)
    rows |= set(int(v) for v in rng.integers(0, count, size=extra))
    return np.array(sorted(rows), dtype=np.int64)


def make(name: str, seed: int = 0, n: int | None = None, m: int | None = None):
    """Inputs of a named config; n/m may be overridden to get a scaled-down case of the
    same distribution."""
    cfg = CONFIGS[name]
    n = cfg.n if n is None else n
    m = cfg.m if m is None else m
    if cfg.kind == "mix_1d":
        return mixture_1d(n, m, seed)
    return gaussian_mixture(n, m, cfg.d, cfg.components, seed, diag_cov=(cfg.kind == "mix_diag"))
