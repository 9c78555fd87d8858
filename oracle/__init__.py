"""ctypes front end of the double-precision CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package;
the product package never does.  Inputs of any float dtype are widened to float64 first, so
the oracle sees exactly the fp32 values the GPU path is given.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdkde_oracle.c")
_LIB = os.path.join(_HERE, "libsdkde_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _configure(lib):
    dp = ctypes.POINTER(ctypes.c_double)
    i64, i32, f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_double
    lib.sdkde_oracle_threads.restype = ctypes.c_int
    lib.sdkde_oracle_score.argtypes = [dp, i64, dp, i64, i32, f64, dp]
    lib.sdkde_oracle_debias.argtypes = [dp, dp, i64, i32, f64, dp]
    lib.sdkde_oracle_eval.argtypes = [dp, i64, dp, i64, i32, f64, dp, dp]
    lib.sdkde_oracle_eval_laplace.argtypes = [dp, i64, dp, i64, i32, f64, dp]
    lib.sdkde_oracle_eval_laplace_abs.argtypes = [dp, i64, dp, i64, i32, f64, dp]
    return lib


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _configure(ctypes.CDLL(_LIB))
    return _lib


def use_library(path):
    """Test hook: route every call through another build of the oracle source (a deliberately
    broken one, to check that the pins notice); path=None restores the real library."""
    global _lib
    _lib = None if path is None else _configure(ctypes.CDLL(path))


def _f64(a):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if a.ndim == 1:
        a = a.reshape(-1, 1)
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: oracle returned status {rc}")


def threads() -> int:
    return int(_load().sdkde_oracle_threads())


def score(samples, h: float, points=None) -> np.ndarray:
    """Empirical KDE score at `points` (default: at the samples themselves)."""
    x = _f64(samples)
    p = x if points is None else _f64(points)
    n, d = x.shape
    m = p.shape[0]
    if p.shape[1] != d:
        raise ValueError("points and samples differ in dimension")
    out = np.empty((m, d), dtype=np.float64)
    _check(_load().sdkde_oracle_score(_p(x), n, _p(p), m, d, float(h), _p(out)), "score")
    return out


def debias(samples, score_values, h: float) -> np.ndarray:
    x = _f64(samples)
    s = _f64(score_values)
    if s.shape != x.shape:
        raise ValueError("score and samples differ in shape")
    out = np.empty_like(x)
    _check(_load().sdkde_oracle_debias(_p(x), _p(s), x.shape[0], x.shape[1], float(h), _p(out)),
           "debias")
    return out


def eval_log_density(samples, queries, h: float) -> np.ndarray:
    x, q = _f64(samples), _f64(queries)
    if q.shape[1] != x.shape[1]:
        raise ValueError("queries and samples differ in dimension")
    out = np.empty(q.shape[0], dtype=np.float64)
    _check(_load().sdkde_oracle_eval(_p(x), x.shape[0], _p(q), q.shape[0], x.shape[1], float(h),
                                     _p(out), None), "eval")
    return out


def eval_density(samples, queries, h: float) -> np.ndarray:
    x, q = _f64(samples), _f64(queries)
    if q.shape[1] != x.shape[1]:
        raise ValueError("queries and samples differ in dimension")
    out = np.empty(q.shape[0], dtype=np.float64)
    _check(_load().sdkde_oracle_eval(_p(x), x.shape[0], _p(q), q.shape[0], x.shape[1], float(h),
                                     None, _p(out)), "eval")
    return out


def eval_laplace_density(samples, queries, h: float) -> np.ndarray:
    x, q = _f64(samples), _f64(queries)
    if q.shape[1] != x.shape[1]:
        raise ValueError("queries and samples differ in dimension")
    out = np.empty(q.shape[0], dtype=np.float64)
    _check(_load().sdkde_oracle_eval_laplace(_p(x), x.shape[0], _p(q), q.shape[0], x.shape[1],
                                             float(h), _p(out)), "eval_laplace")
    return out


def eval_laplace_abs_density(samples, queries, h: float) -> np.ndarray:
    """Sum of K_h |1 + d/2 - r^2/2h^2| / n: the scale of the terms the signed Laplace sum cancels."""
    x, q = _f64(samples), _f64(queries)
    out = np.empty(q.shape[0], dtype=np.float64)
    _check(_load().sdkde_oracle_eval_laplace_abs(_p(x), x.shape[0], _p(q), q.shape[0], x.shape[1],
                                                 float(h), _p(out)), "eval_laplace_abs")
    return out


def sd_kde_log_density(samples, queries, h: float):
    """Whole pipeline: score at the samples, shift, KDE of the shifted samples at the queries.
    Returns (score, shifted samples, log density)."""
    s = score(samples, h)
    x_sd = debias(samples, s, h)
    return s, x_sd, eval_log_density(x_sd, queries, h)
