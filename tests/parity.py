"""Comparison helpers for GPU-vs-oracle parity (no estimator arithmetic here).

Tolerances (from the benchmark spec: max relative error <= 1e-3 on density, <= 1e-3 * |s| on
score for the fp32-accumulate path):
  score   : per point, |s_gpu - s_ref|_2 <= 1e-3 * max(|s_ref|_2, 1e-3 * rms_i |s_ref,i|_2)
            (degenerate data whose true score vanishes against 1/h: also the absolute score_resolution below)
  density : |p_gpu - p_ref| <= 1e-3 * p_ref wherever p_ref >= 1e-30 (fp32-representable with margin)
  log dens: |log p_gpu - log p_ref| <= 1e-3 (used where the density itself is below fp32 range)
"""
import numpy as np

TOL = 1e-3


def score_resolution(x, points, h):
    """What fp32 arithmetic resolves of a score, per point and in absolute terms: the paper's identity
    sum_j (p - x_j) phi_j = p sum_j phi_j - sum_j phi_j x_j subtracts two sums of size |p - c| sum_j phi_j (coordinates
    are relative to a centre c of the samples), each carried through fp32 accumulators, so about
    16 * 2^-24 * (1 + |p - c| / h) / h is lost whatever the size of the result (16: the roundings of the two sums,
    measured up to 10).  It matters only where the true score is that small against 1/h: a sample whose only
    neighbours are its own exact duplicates, a point where the pulls of two clusters cancel."""
    x = np.asarray(x, dtype=np.float64)
    p = np.asarray(points, dtype=np.float64)
    c = x.mean(axis=0)
    return 2.0**-20 * (1.0 + np.linalg.norm(p - c, axis=1) / h) / h


def score_error(s_gpu, s_ref, resolution=None):
    """Largest per-point error relative to its allowance (<= 1 passes) and the global relative
    Frobenius error.  resolution (per point, score_resolution): an absolute allowance beside the relative one."""
    s_gpu = np.asarray(s_gpu, dtype=np.float64)
    s_ref = np.asarray(s_ref, dtype=np.float64)
    err = np.linalg.norm(s_gpu - s_ref, axis=1)
    ref = np.linalg.norm(s_ref, axis=1)
    rms = float(np.sqrt(np.mean(ref**2))) if len(ref) else 0.0
    allow = TOL * np.maximum(ref, 1e-3 * rms)
    if resolution is not None:
        allow = np.maximum(allow, resolution)
    allow = np.where(allow > 0, allow, np.finfo(np.float64).tiny)
    frob = float(np.linalg.norm(s_gpu - s_ref) / max(np.linalg.norm(s_ref), 1e-300))
    return float(np.max(err / allow)) if len(err) else 0.0, frob


def assert_score_close(s_gpu, s_ref, what="", resolution=None):
    assert np.all(np.isfinite(s_gpu)), f"{what}: non-finite score"
    worst, frob = score_error(s_gpu, s_ref, resolution)
    assert worst <= 1.0, f"{what}: score error {worst:.3g}x the allowance (global rel {frob:.3g})"
    return worst, frob


def assert_density_close(p_gpu, logp_ref, what=""):
    p_gpu = np.asarray(p_gpu, dtype=np.float64)
    p_ref = np.exp(logp_ref)
    big = p_ref >= 1e-30
    rel = np.abs(p_gpu[big] - p_ref[big]) / p_ref[big]
    worst = float(rel.max()) if rel.size else 0.0
    assert worst <= TOL, f"{what}: density rel error {worst:.3g}"
    return worst


def assert_log_density_close(lp_gpu, logp_ref, what=""):
    lp_gpu = np.asarray(lp_gpu, dtype=np.float64)
    assert np.all(np.isfinite(lp_gpu)), f"{what}: non-finite log density"
    worst = float(np.max(np.abs(lp_gpu - logp_ref))) if lp_gpu.size else 0.0
    assert worst <= TOL, f"{what}: log-density abs error {worst:.3g}"
    return worst


def assert_shifted_close(x_sd_gpu, x_sd_ref, s_ref, h, what=""):
    """Shifted samples: the shift (h^2/2) s carries the score tolerance; on top of it the fp32
    result cannot resolve less than one rounding (2^-24 relative) of x_sd itself."""
    x_sd_gpu = np.asarray(x_sd_gpu, dtype=np.float64)
    ref = np.linalg.norm(s_ref, axis=1)
    rms = float(np.sqrt(np.mean(ref**2)))
    allow = 0.5 * h * h * TOL * np.maximum(ref, 1e-3 * rms) + 2.0**-24 * np.linalg.norm(x_sd_ref, axis=1)
    err = np.linalg.norm(x_sd_gpu - x_sd_ref, axis=1)
    worst = float(np.max(err / allow))
    assert worst <= 1.0, f"{what}: shifted-sample error {worst:.3g}x the allowance"
    return worst


def gram_exponent_error(x, q, h, low_precision_inputs=False):
    """Bound, per query, on the absolute error of the exponent -|q - x_j|^2 / 2h^2 (in nats) as the matrix path
    forms it in fp32: |q~|^2 + |x~|^2 - 2 q~.x~ on coordinates relative to a centre c of the samples.  With
    E = (|q - c|^2 + max_j |x_j - c|^2) / 2h^2 the size of the terms that cancel, the two stored norms are rounded
    relative to their own sizes (together at most one half-ulp of E), their sum once, and each of the d/4 MFMA
    steps rounds an accumulator of at most that size: (2 + d/4) half-ulps of E, i.e. (2 + d/4) E 2^-24.  The fp16
    hi + lo input modes drop the lo.lo products, 2^-22 of |q~||x~| <= E per pair: four more units.  The thin path
    (d <= 3) forms the differences directly, and what it rounds is the squared distance itself, d + 2 times:
    (2 + d) u 2^-24 with u <= 88, beyond which the weight is zero in fp32."""
    x = np.asarray(x, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    d = x.shape[1]
    if d <= 3:
        return np.full(q.shape[0], (2.0 + d) * 88.0 * 2.0**-24)
    c = x.mean(axis=0)
    big = ((q - c) ** 2).sum(axis=1) + float(((x - c) ** 2).sum(axis=1).max())
    return (2.0 + d / 4.0 + (4.0 if low_precision_inputs else 0.0)) * big / (2.0 * h * h) * 2.0**-24


def assert_laplace_close(p_gpu, p_ref, p_abs_ref, what="", exponent_error=None, p_kde_ref=None):
    """Signed Laplace-corrected density: |error| <= max(1e-3 |p_ref|, 1e-6 p_abs_ref, e (p_abs_ref + p_kde_ref)),
    where p_abs_ref sums the magnitudes of the terms that cancel in p_ref and e = exponent_error (per query,
    gram_exponent_error) is what the fp32 Gram expansion can lose in every term's exponent: a term
    phi (1 + d/2 - u) with u off by e changes by at most e (|1 + d/2 - u| + 1) phi, which sums to
    e (p_abs_ref + p_kde_ref) over the samples (p_kde_ref: the plain KDE at the same queries)."""
    p_gpu = np.asarray(p_gpu, dtype=np.float64)
    big = p_abs_ref >= 1e-30
    allow = np.maximum(TOL * np.abs(p_ref), TOL * 1e-3 * p_abs_ref)
    if exponent_error is not None:
        allow = np.maximum(allow, exponent_error * (p_abs_ref + p_kde_ref))
    worst = float(np.max(np.abs(p_gpu[big] - p_ref[big]) / allow[big])) if big.any() else 0.0
    assert worst <= 1.0, f"{what}: Laplace density error {worst:.3g}x the allowance"
    return worst
