"""Index range: more than 2^31 elements in the prepared point array (m_pad * dp) and in the partial
buffers, with few samples so that the pair count stays small.  Sampled points against the oracle."""
import time

import numpy as np
import pytest

import oracle
import sdkde_inputs
from parity import assert_log_density_close, assert_score_close

pytestmark = pytest.mark.gpu


def test_points_beyond_two_to_the_31_elements():
    import torch
    import paper_2602_10378_amd as P
    P.load()
    n, d = 200, 7
    m = (1 << 27) + 12345                      # m_pad * 16 floats > 2^31
    print(f"large index: n={n} m={m} d={d}", flush=True)
    plan = P.sdkde_describe_plan(n, m, d, 1)
    assert plan["m_pad"] * plan["dp"] > 2**31
    x = sdkde_inputs.standard_normal_cloud(n, d, seed=1)
    q = sdkde_inputs.standard_normal_cloud(m, d, seed=2, scale=1.5)
    h = 0.6
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ws = P.make_workspace(n, m, d)
    print(f"large index: workspace {ws.numel() / 2**30:.1f} GiB", flush=True)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([np.arange(0, 40), np.arange(m - 40, m), (1 << 27) + np.arange(-40, 40),
                                     (1 << 26) + np.arange(-8, 8), rng.integers(0, m, size=400)]))
    idx = torch.from_numpy(rows).cuda()

    dens, logd = P.sdkde_eval(xd, qd, h, want="both", workspace=ws)
    got = logd[idx].cpu().numpy()
    ok = np.isfinite(got)                      # a point 13 h from every sample underflows in fp32 (documented)
    assert ok.mean() > 0.9
    e = assert_log_density_close(got[ok], oracle.eval_log_density(x, q[rows[ok]], h), "large index eval")
    print(f"large index: eval log-density err {e:.3g} on {int(ok.sum())} points", flush=True)
    del dens, logd

    s = P.sdkde_score(xd, h, points=qd, workspace=ws)
    worst, _ = assert_score_close(s[idx].cpu().numpy()[ok], oracle.score(x, h, points=q[rows[ok]]), "large index score")
    print(f"large index: score at points worst {worst:.3g} of allowance", flush=True)


def test_samples_beyond_two_to_the_31_elements():
    import torch
    import paper_2602_10378_amd as P
    P.load()
    n, d, m = (1 << 27) + 777, 7, 300           # n_pad * 16 floats > 2^31; 8.4 million sample tiles
    print(f"large index: n={n} m={m} d={d}", flush=True)
    plan = P.sdkde_describe_plan(n, m, d, 2)
    assert plan["n_pad"] * plan["dp"] > 2**31
    x = sdkde_inputs.standard_normal_cloud(n, d, seed=4)
    q = sdkde_inputs.standard_normal_cloud(m, d, seed=5, scale=0.8)
    h = 0.1                                     # narrow: the sums are dominated by few of the 134 million samples
    t0 = time.time()
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    # sized for the two calls made here (the score at the samples themselves would need ~100 GiB at this n)
    need = max(plan["workspace_bytes"], P.sdkde_describe_plan(n, m, d, 1)["workspace_bytes"])
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    print(f"large index: workspace {need / 2**30:.1f} GiB, splits {plan['splits']}", flush=True)
    logd = P.sdkde_eval(xd, qd, h, want="log", workspace=ws)[1].cpu().numpy()
    sp = P.sdkde_score(xd, h, points=qd, workspace=ws).cpu().numpy()
    print(f"large index: GPU part {time.time() - t0:.1f} s", flush=True)
    rows = np.arange(0, m, 25)                  # the oracle takes a few tenths of a second per query at this n
    e = assert_log_density_close(logd[rows], oracle.eval_log_density(x, q[rows], h), "large index eval (samples)")
    worst, _ = assert_score_close(sp[rows], oracle.score(x, h, points=q[rows]), "large index score (samples)")
    print(f"large index: {len(rows)} queries against {n} samples: log-density err {e:.3g}, score worst {worst:.3g} "
          "of allowance", flush=True)
