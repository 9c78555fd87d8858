"""The library only enqueues kernels on the caller's stream (no allocation, no host sync, no
memset), so a whole score -> debias -> eval pass can be captured in a HIP graph.  Every replay
is checked against the eager result, with eager work and synchronisations between replays."""
import numpy as np
import pytest

import sdkde_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,n,m,flags", [("C1", 4096, 1024, 0), ("C3", 5000, 700, 0), ("C1", 5000, 700, 32), ("C4", 3000, 500, 0)])
def test_pipeline_replays_from_a_graph(name, n, m, flags, tuning):
    import torch
    import paper_2602_10378_amd as P
    tuning(P.SDKDE_TUNE_SYM_MIN_ITEMS, 1)      # take the symmetric mode at this small size too
    print(f"graph {name} n={n} m={m} flags={flags}", flush=True)
    x, q, h = sdkde_inputs.make(name, seed=0, n=n, m=m)
    d = x.shape[1]
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ws = P.make_workspace(n, m, d, flags=flags)        # 32 = SDKDE_FLAG_SYMMETRIC: the score's symmetric mode
    s = torch.empty_like(xd)
    x_sd = torch.empty_like(xd)
    dens = torch.empty(m, device="cuda")
    logd = torch.empty(m, device="cuda")

    def step():
        P.sdkde_score(xd, h, out=s, workspace=ws, flags=flags)
        P.sdkde_debias(xd, s, h, out=x_sd)
        P.sdkde_eval(x_sd, qd, h, density_out=dens, log_density_out=logd, workspace=ws, flags=flags)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (s, x_sd, dens, logd)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                    # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    for replay in range(4):
        for t in (s, x_sd, dens, logd):
            t.fill_(float("nan"))
        ws.random_(0, 255)                        # scratch contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((s, x_sd, dens, logd), want):
            assert torch.equal(got, ref), f"replay {replay} differs from the eager result"
        # eager work of another shape between replays
        other = torch.from_numpy(np.ascontiguousarray(x[: n // 3])).cuda()
        P.sdkde_score(other, h)
        torch.cuda.synchronize()
