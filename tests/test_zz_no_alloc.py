"""sdkde_fit_eval_static (the entry point for callers that cannot allocate: its scratch is a buffer built
into the library's device image) must give what sdkde_fit_eval gives with a caller-owned workspace, on two
calls in a row that share the built-in buffer, the second with a smaller input; and the oracle's results
within the parity tolerances."""
import numpy as np
import pytest

import sdkde_inputs
from parity import assert_density_close, assert_log_density_close, assert_score_close, assert_shifted_close

pytestmark = pytest.mark.gpu


def _run_both(P, torch, name, n, m, flags=0):
    print(f"static scratch: {name} n={n} m={m} flags={flags}", flush=True)
    x, q, h = sdkde_inputs.make(name, seed=3, n=n, m=m)
    d = x.shape[1]
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    outs = {}
    for which in ("workspace", "static"):
        s, x_sd = torch.full_like(xd, float("nan")), torch.full_like(xd, float("nan"))
        dens = torch.full((m,), float("nan"), device="cuda")
        logd = torch.full((m,), float("nan"), device="cuda")
        if which == "workspace":
            ws = torch.empty(P.sdkde_workspace_bytes(n, m, d, flags), dtype=torch.uint8, device="cuda")
            P.sdkde_fit_eval(xd, qd, h, score_out=s, samples_sd_out=x_sd, density_out=dens, log_density_out=logd,
                             workspace=ws, flags=flags)
        else:
            P.sdkde_fit_eval_static(xd, qd, h, x_sd, score_out=s, density_out=dens, log_density_out=logd, flags=flags)
        torch.cuda.synchronize()
        outs[which] = [t.cpu().numpy() for t in (s, x_sd, dens, logd)]
    for got, want, what in zip(outs["static"], outs["workspace"], ("score", "shifted samples", "density", "log density")):
        assert np.all(np.isfinite(got)), f"{what}: non-finite output"
        assert np.array_equal(got, want), f"{what} differs from sdkde_fit_eval's"
    return x, q, h, outs["static"]


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    import torch
    import oracle
    import paper_2602_10378_amd as P
    # first call: several row blocks and splits, a ragged tail; second call: smaller in every size, another d
    for name, n, m in (("C1", 9000, 2100), ("C3", 2500, 333)):
        x, q, h, (s, x_sd, dens, logd) = _run_both(P, torch, name, n, m)
        s_ref, x_sd_ref, logp_ref = oracle.sd_kde_log_density(x, q, h)
        assert_score_close(s, s_ref, name)
        assert_shifted_close(x_sd, x_sd_ref, s_ref, h, name)
        assert_log_density_close(logd, logp_ref, name)
        assert_density_close(dens, logp_ref, name)
    # and a lower-precision input mode on the same buffer
    _run_both(P, torch, "C1", 3000, 500, flags=P.SDKDE_PREC_FP16X2)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    import paper_2602_10378_amd as P
    n, m, d = 262144, 1024, 16
    assert P.sdkde_workspace_bytes(n, m, d) > P.SDKDE_STATIC_SCRATCH_BYTES
    xd = torch.zeros((n, d), device="cuda")
    qd = torch.zeros((m, d), device="cuda")
    out = torch.full_like(xd, 7.0)
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_fit_eval_static(xd, qd, 1.0, out, density_out=torch.empty(m, device="cuda"))
    assert e.value.status == P.SDKDE_ETOOLARGE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all()), "a refused call must not write"


def test_static_scratch_entry_point_replays_from_a_graph():
    """The callers this entry point is for include code under stream capture: after one call outside capture (it
    looks up the buffer's address), the call is captured into a HIP graph and every replay gives the eager bits."""
    import torch
    import paper_2602_10378_amd as P
    n, m = 5000, 700
    print(f"static scratch under capture: n={n} m={m}", flush=True)
    x, q, h = sdkde_inputs.make("C1", seed=4, n=n, m=m)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    s, x_sd = torch.empty_like(xd), torch.empty_like(xd)
    dens, logd = torch.empty(m, device="cuda"), torch.empty(m, device="cuda")

    def step():
        P.sdkde_fit_eval_static(xd, qd, h, x_sd, score_out=s, density_out=dens, log_density_out=logd)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (s, x_sd, dens, logd)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for replay in range(3):
        for t in (s, x_sd, dens, logd):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((s, x_sd, dens, logd), want):
            assert torch.equal(got, ref), f"replay {replay} differs from the eager result"
        # an eager call of another size on the same built-in buffer between replays
        P.sdkde_fit_eval_static(xd[:1500].contiguous(), qd[:100].contiguous(), h, torch.empty(1500, x.shape[1], device="cuda"),
                                density_out=torch.empty(100, device="cuda"))
        torch.cuda.synchronize()
