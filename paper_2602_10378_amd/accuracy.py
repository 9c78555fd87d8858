"""Integrated-error comparison of the estimators the paper studies (its known-density
benchmark": MISE / MIAE of KDE, Laplace-corrected KDE and SD-KDE against a known mixture density),
run through the GPU library.

With evaluation points q_k drawn from the true density p itself, the integrals become plain
averages (importance sampling with proposal p):
    ISE = int (p_hat - p)^2 dq  ~  mean_k (p_hat(q_k) - p(q_k))^2 / p(q_k)
    IAE = int |p_hat - p| dq    ~  mean_k |p_hat(q_k) - p(q_k)| / p(q_k)
Everything is formed in log space on the host in float64 from the library's fp32 log densities,
so the comparison also works where the densities themselves are far below the fp32 range.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _errors(log_est: np.ndarray, sign: np.ndarray, log_true: np.ndarray):
    ratio = sign * np.exp(log_est - log_true)             # p_hat / p
    p = np.exp(log_true)
    return {"ise": float(np.mean((ratio - 1.0) ** 2 * p)), "iae": float(np.mean(np.abs(ratio - 1.0))),
            "mean_sq_rel": float(np.mean((ratio - 1.0) ** 2))}


def integrated_errors(samples: torch.Tensor, queries: torch.Tensor, h: float, log_true_density: np.ndarray,
                      flags: int = B.SDKDE_PREC_FP32):
    """samples [n,d], queries [m,d] (drawn from the true density) on the GPU; log_true_density [m] on the host.
    Returns {estimator: {"ise", "iae", "mean_sq_rel"}} for
      kde            plain Gaussian KDE of the samples,
      sd_kde         score-debiased KDE (score and KDE with the same bandwidth h),
      sd_kde_half_t  as sd_kde but the score taken at bandwidth h/sqrt(2) (the t' = h^2/2 remark of the
                     Laplace-corrected KDE section),
      laplace        Laplace-corrected KDE (signed; only where d is small enough for fp32 densities).
    """
    n, d = samples.shape
    ws = B.make_workspace(n, queries.shape[0], d, device=samples.device)
    log_true = np.asarray(log_true_density, dtype=np.float64)
    out = {}
    ones = np.ones_like(log_true)

    _, logd = B.sdkde_eval(samples, queries, h, want="log", workspace=ws, flags=flags)
    out["kde"] = _errors(logd.double().cpu().numpy(), ones, log_true)

    for name, h_score in (("sd_kde", h), ("sd_kde_half_t", h / np.sqrt(2.0))):
        s = B.sdkde_score(samples, h_score, workspace=ws, flags=flags)
        x_sd = B.sdkde_debias(samples, s, h)
        _, logd = B.sdkde_eval(x_sd, queries, h, want="log", workspace=ws, flags=flags)
        out[name] = _errors(logd.double().cpu().numpy(), ones, log_true)

    lap = B.sdkde_eval_laplace(samples, queries, h, workspace=ws, flags=flags).double().cpu().numpy()
    if np.all(np.isfinite(lap)) and np.any(lap != 0.0) and log_true.max() > -60.0:
        with np.errstate(divide="ignore"):
            out["laplace"] = _errors(np.log(np.abs(lap)), np.sign(lap), log_true)
    return out
