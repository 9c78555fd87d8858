"""The estimators behave as the paper's oracle-density benchmark says (Results section): against a
known mixture density, score-debiased KDE and Laplace-corrected KDE have a clearly lower integrated
squared error than plain KDE at the same (Silverman) bandwidth.  Checked with the CPU oracle at a
small size and with the GPU library at a larger one.  This pins the readings of the method (self
term included, same bandwidth in score and KDE, shift of +h^2/2 s): with any of them wrong the
debiased estimate gets worse than the plain one, not better."""
import numpy as np
import pytest

import oracle
import sdkde_inputs


def _ise(log_est, log_true, sign=None):
    ratio = np.exp(log_est - log_true) if sign is None else sign * np.exp(log_est - log_true)
    return float(np.mean((ratio - 1.0) ** 2 * np.exp(log_true)))


def test_oracle_sd_kde_and_laplace_beat_kde_in_1d():
    w, mu, var = sdkde_inputs.mixture_parameters("C3")
    q = sdkde_inputs.mixture_1d(4000, 8, seed=100)[0]             # evaluation points drawn from the true density
    log_true = sdkde_inputs.true_log_density(q, w, mu, var)
    wins_sd, wins_lap = 0, 0
    for seed in range(3):
        x, _, h = sdkde_inputs.mixture_1d(2048, 8, seed=seed)
        kde = _ise(oracle.eval_log_density(x, q, h), log_true)
        _, _, logp_sd = oracle.sd_kde_log_density(x, q, h)
        sd = _ise(logp_sd, log_true)
        lap_dens = oracle.eval_laplace_density(x, q, h)
        lap = float(np.mean((lap_dens / np.exp(log_true) - 1.0) ** 2 * np.exp(log_true)))
        wins_sd += sd < 0.7 * kde
        wins_lap += lap < 0.7 * kde
    assert wins_sd == 3 and wins_lap == 3


@pytest.mark.gpu
@pytest.mark.parametrize("name,n,factor", [("C3", 16384, 0.4), ("C1", 32768, 1.0)])
def test_gpu_sd_kde_and_laplace_beat_kde(name, n, factor):
    import torch
    from paper_2602_10378_amd import accuracy
    w, mu, var = sdkde_inputs.mixture_parameters(name, 0)
    if name == "C3":
        x, _, h = sdkde_inputs.make(name, seed=0, n=n, m=8)
        q = sdkde_inputs.mixture_1d(8192, 8, seed=100)[0]
    else:
        x, q, h = sdkde_inputs.make(name, seed=0, n=n, m=8192)    # queries of the 16-D configs are mixture draws
    log_true = sdkde_inputs.true_log_density(q, w, mu, var)
    res = accuracy.integrated_errors(torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda(), h, log_true)
    print(name, n, {k: v["ise"] for k, v in res.items()}, flush=True)
    # 1-D: a large gain.  16-D with Silverman's bandwidth every estimator is heavily over-smoothed
    # (integrated absolute error above 1), so only the ordering of the squared errors is asserted.
    assert res["sd_kde"]["ise"] < factor * res["kde"]["ise"]
    assert res["laplace"]["ise"] < factor * res["kde"]["ise"]
    assert res["sd_kde_half_t"]["ise"] < factor * res["kde"]["ise"]
