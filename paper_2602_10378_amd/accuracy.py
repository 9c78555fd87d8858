"""Integrated-error comparison of the estimators the paper studies (Results section, the benchmark
against a known density: MISE / MIAE of KDE, Laplace-corrected KDE and SD-KDE against a known mixture density, with the
negative mass of the signed Laplace estimate logged separately), run through the GPU library.

With evaluation points q_k drawn from a proposal density g, every integral is a plain average:
    ISE      = int (p_hat - p)^2 dq     ~  mean_k (p_hat(q_k) - p(q_k))^2 / g(q_k)
    IAE      = int |p_hat - p| dq       ~  mean_k |p_hat(q_k) - p(q_k)| / g(q_k)
    neg mass = int max(-p_hat, 0) dq    ~  mean_k max(-p_hat(q_k), 0) / g(q_k)
A uniform grid is the case g = 1 / (length of the interval) (1-D: plain quadrature).  In higher dimension the
proposal is the true mixture with every component variance enlarged by h^2 (the expectation of the KDE), which
covers the region where the estimates live, tails included.  Everything is formed on the host in float64 from the
library's fp32 outputs.

  python -m paper_2602_10378_amd.accuracy        prints the table of the n-sweeps (3 seeds) as markdown
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _errors(p_hat: np.ndarray, p_true: np.ndarray, g: np.ndarray):
    diff = p_hat - p_true
    return {"ise": float(np.mean(diff * diff / g)), "iae": float(np.mean(np.abs(diff) / g)),
            "neg_mass": float(np.mean(np.maximum(-p_hat, 0.0) / g))}


def integrated_errors(samples: torch.Tensor, queries: torch.Tensor, h: float, log_true_density: np.ndarray,
                      log_proposal: np.ndarray | None = None, flags: int = B.SDKDE_PREC_FP32):
    """samples [n,d], queries [m,d] on the GPU; log_true_density [m] and log_proposal [m] (default: the true
    density itself) on the host.  Returns {estimator: {"ise", "iae", "neg_mass"}} for
      kde            plain Gaussian KDE of the samples,
      sd_kde         score-debiased KDE (score and KDE with the same bandwidth h),
      sd_kde_half_t  as sd_kde but the score taken at bandwidth h/sqrt(2) (the t' = h^2/2 remark of the
                     Laplace-corrected KDE section),
      laplace        Laplace-corrected KDE (signed).
    """
    n, d = samples.shape
    ws = B.make_workspace(n, queries.shape[0], d, device=samples.device)
    log_true = np.asarray(log_true_density, dtype=np.float64)
    g = np.exp(log_true if log_proposal is None else np.asarray(log_proposal, dtype=np.float64))
    p_true = np.exp(log_true)
    out = {}

    _, logd = B.sdkde_eval(samples, queries, h, want="log", workspace=ws, flags=flags)
    out["kde"] = _errors(np.exp(logd.double().cpu().numpy()), p_true, g)
    for name, h_score in (("sd_kde", h), ("sd_kde_half_t", h / np.sqrt(2.0))):
        s = B.sdkde_score(samples, h_score, workspace=ws, flags=flags)
        x_sd = B.sdkde_debias(samples, s, h)
        _, logd = B.sdkde_eval(x_sd, queries, h, want="log", workspace=ws, flags=flags)
        out[name] = _errors(np.exp(logd.double().cpu().numpy()), p_true, g)
    lap = B.sdkde_eval_laplace(samples, queries, h, workspace=ws, flags=flags).double().cpu().numpy()
    out["laplace"] = _errors(lap, p_true, g)
    return out


def benchmark_points(name: str, h: float, count: int, seed: int):
    """Evaluation points and their log proposal density for config `name` ("C3": 1-D, "C1": 16-D): a uniform
    grid over [-6, 7] in 1-D, draws from the h-smoothed mixture otherwise.  Returns (q fp32 [count, d],
    log_true [count], log_proposal [count])."""
    import sdkde_inputs
    w, mu, var = sdkde_inputs.mixture_parameters(name, 0)
    if mu.shape[1] == 1:
        lo, hi = -6.0, 7.0
        q = np.linspace(lo, hi, count).astype(np.float32).reshape(count, 1)
        log_g = np.full(count, -np.log(hi - lo))
    else:
        q = sdkde_inputs.draw_from_mixture(w, mu, var + h * h, count, seed).astype(np.float32)
        log_g = sdkde_inputs.true_log_density(q, w, mu, var + h * h)
    return q, sdkde_inputs.true_log_density(q, w, mu, var), log_g


def sweep(name: str, sizes, seeds=(0, 1, 2), bandwidth_factor: float = 1.0, points: int = 16384):
    """{n: {estimator: {metric: [value per seed]}}} for samples of config `name`'s mixture (parameters of seed 0,
    sample draws of each seed) with bandwidth = bandwidth_factor x the rule of thumb of each sample set."""
    import sdkde_inputs
    table = {}
    for n in sizes:
        rows = {}
        for seed in seeds:
            x, h = sdkde_inputs.mixture_samples(name, n, seed)
            h = float(h) * bandwidth_factor
            q, log_true, log_g = benchmark_points(name, h, points, 1000 + seed)
            res = integrated_errors(torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda(), h, log_true, log_g)
            for est, vals in res.items():
                for metric, v in vals.items():
                    rows.setdefault(est, {}).setdefault(metric, []).append(v)
        table[n] = rows
    return table


def _fmt(values):
    return f"{np.mean(values):.2e} ± {np.std(values):.1e}"


def markdown(table, title):
    ests = ("kde", "sd_kde", "sd_kde_half_t", "laplace")
    lines = [f"**{title}**", "", "| n | metric | KDE | SD-KDE | SD-KDE, score at h/√2 | Laplace-corrected | Laplace negative mass |",
             "|---|---|---|---|---|---|---|"]
    for n, rows in table.items():
        for metric, label in (("ise", "ISE"), ("iae", "IAE")):
            cells = " | ".join(_fmt(rows[e][metric]) for e in ests)
            neg = _fmt(rows["laplace"]["neg_mass"]) if metric == "iae" else ""
            lines.append(f"| {n} | {label} | {cells} | {neg} |")
    return "\n".join(lines)


def main():
    print(markdown(sweep("C3", (1024, 4096, 16384, 65536)), "1-D mixture (0.7 N(0,1) + 0.3 N(3, 0.25)), rule-of-thumb bandwidth"))
    print()
    print(markdown(sweep("C1", (2048, 8192, 32768)), "16-D mixture (4 unit-covariance components), rule-of-thumb bandwidth"))
    print()
    print(markdown(sweep("C1", (2048, 8192, 32768), bandwidth_factor=0.6),
                   "16-D mixture, 0.6 x the rule-of-thumb bandwidth"))


if __name__ == "__main__":
    main()
