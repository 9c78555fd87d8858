"""Odd shapes and extreme bandwidths: sizes around the padding and tile boundaries, very few
samples against many points and the reverse, the largest supported dimension, bandwidths that
make every neighbour vanish or every pair weigh the same."""
import numpy as np
import pytest

import oracle
import sdkde_inputs
from parity import assert_log_density_close, assert_score_close

pytestmark = pytest.mark.gpu


def _run(P, torch, x, q, h):
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    s = P.sdkde_score(xd, h)
    sp = P.sdkde_score(xd, h, points=qd)
    _, logd = P.sdkde_eval(xd, qd, h, want="log")
    torch.cuda.synchronize()
    return s.cpu().numpy(), sp.cpu().numpy(), logd.cpu().numpy()


@pytest.mark.parametrize("n,m,d", [(100, 100000, 16), (50000, 1, 16), (1023, 31, 16), (1024, 32, 16), (1025, 33, 16),
                                   (31, 1025, 4), (33, 7, 128), (5000, 64, 128), (40000, 3, 1), (3, 40000, 2)])
def test_odd_shapes(n, m, d):
    import torch
    import paper_2602_10378_amd as P
    print(f"shape n={n} m={m} d={d}", flush=True)
    rng = np.random.default_rng(n + 7 * m + d)
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = (0.8 * rng.standard_normal((m, d))).astype(np.float32)
    h = float(max(sdkde_inputs.silverman_bandwidth(x), 0.3)) if n > 3 else 0.9
    if d == 128:
        # Silverman's rule puts c |x - y|^2 near 1.3 d for i.i.d. data: at d = 128 every pair weight is
        # below the fp32 range and the (documented) all-underflow result applies; use a wider kernel here.
        h = 2.5
    s, sp, logd = _run(P, torch, x, q, h)
    assert_score_close(s, oracle.score(x, h), f"self n={n} d={d}")
    assert_score_close(sp, oracle.score(x, h, points=q), f"points n={n} m={m} d={d}")
    assert_log_density_close(logd, oracle.eval_log_density(x, q, h), f"eval n={n} m={m} d={d}")


@pytest.mark.parametrize("d", [1, 16])
def test_extreme_bandwidths(d):
    import torch
    import paper_2602_10378_amd as P
    x, q, h0 = (sdkde_inputs.mixture_1d(2000, 100, 3) if d == 1 else sdkde_inputs.gaussian_mixture(2000, 100, 16, seed=3))
    # huge bandwidth: every pair weighs almost the same, the score tends to -(x - mean)/h^2
    big = 200.0 * h0
    s, sp, logd = _run(P, torch, x, q, big)
    assert_score_close(s, oracle.score(x, big), f"big h d={d}")
    assert_score_close(sp, oracle.score(x, big, points=q), f"big h points d={d}")
    assert_log_density_close(logd, oracle.eval_log_density(x, q, big), f"big h eval d={d}")
    # tiny bandwidth: no neighbour is left, the score at the samples is ~0 and stays finite
    tiny = 1e-3 * h0
    xd = torch.from_numpy(x).cuda()
    st = P.sdkde_score(xd, tiny).cpu().numpy()
    assert np.all(np.isfinite(st))
    ref = oracle.score(x, tiny)
    assert np.max(np.abs(st - ref)) <= 1e-3 * max(np.max(np.abs(ref)), 1e-30) + 1e-20
    if d == 1:
        # direct differences: the self distance is exactly 0, so the self-evaluated density is the self term
        # alone.  (On the MFMA path the Gram expansion loses |x~|^2 * 2^-23 in the exponent, which is only
        # small while (data radius / h)^2 is far below 2^23: not the case for this bandwidth.)
        _, ld = P.sdkde_eval(xd, xd, tiny, want="log")
        assert_log_density_close(ld.cpu().numpy(), oracle.eval_log_density(x, x, tiny), f"tiny h eval d={d}")


def test_debias_in_place_and_aliasing():
    import torch
    import paper_2602_10378_amd as P
    rng = np.random.default_rng(0)
    x = torch.from_numpy(rng.standard_normal((1000, 16)).astype(np.float32)).cuda()
    s = torch.from_numpy(rng.standard_normal((1000, 16)).astype(np.float32)).cuda()
    want = P.sdkde_debias(x, s, 1.3)
    xa = x.clone()
    P.sdkde_debias(xa, s, 1.3, out=xa)
    sa = s.clone()
    P.sdkde_debias(x, sa, 1.3, out=sa)
    assert torch.equal(xa, want) and torch.equal(sa, want)


@pytest.mark.parametrize("d", [1, 3, 16, 128])
def test_max_shift_mode_handles_points_whose_weights_all_underflow(d):
    # Without the flag these points get density 0 / log density -inf / score 0 (documented); with it the
    # sums are taken relative to the largest weight and match the oracle's max-shifted evaluation.
    import torch
    import paper_2602_10378_amd as P
    from parity import assert_laplace_close
    rng = np.random.default_rng(50 + d)
    n, m = 3000, 200
    x = rng.standard_normal((n, d)).astype(np.float32)
    h = float(sdkde_inputs.silverman_bandwidth(x))
    q = rng.standard_normal((m, d)).astype(np.float32)
    if d < 128:
        # push the queries out until c |q - x|^2 is a few hundred for every sample (i.i.d. data at d = 128
        # is there already with a rule-of-thumb bandwidth)
        direction = q / np.linalg.norm(q, axis=1, keepdims=True)
        q = (q + direction * (25.0 * h + 4.0)).astype(np.float32)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    _, plain = P.sdkde_eval(xd, qd, h, want="log")
    assert torch.isinf(plain).any()                   # the regime this test is about
    flags = P.SDKDE_FLAG_MAX_SHIFT
    dens, logd = P.sdkde_eval(xd, qd, h, want="both", flags=flags)
    ref = oracle.eval_log_density(x, q, h)
    assert_log_density_close(logd.cpu().numpy(), ref, f"shifted eval d={d}")
    sp = P.sdkde_score(xd, h, points=qd, flags=flags).cpu().numpy()
    assert_score_close(sp, oracle.score(x, h, points=q), f"shifted score at points d={d}")
    if d <= 16:
        lap = P.sdkde_eval_laplace(xd, qd, h, flags=flags).cpu().numpy()
        lref, labs = oracle.eval_laplace_density(x, q, h), oracle.eval_laplace_abs_density(x, q, h)
        assert np.all(np.isfinite(lap))
        ok = labs > 1e-36                               # where the signed density is representable in fp32 at all
        if ok.any():
            assert_laplace_close(lap[ok], lref[ok], labs[ok], f"shifted laplace d={d}")
        # a nearer ring of queries, where plain fp32 sums are tiny but the densities are representable
        q2 = (x[:m] + 6.0 * h * direction).astype(np.float32)
        lap2 = P.sdkde_eval_laplace(xd, torch.from_numpy(q2).cuda(), h, flags=flags).cpu().numpy()
        assert_laplace_close(lap2, oracle.eval_laplace_density(x, q2, h), oracle.eval_laplace_abs_density(x, q2, h),
                             f"shifted laplace ring d={d}")
    # the flag changes nothing where no shift is needed (queries among the samples), beyond rounding
    near = torch.from_numpy(x[:100].copy()).cuda()
    _, a = P.sdkde_eval(xd, near, h, want="log")
    _, b = P.sdkde_eval(xd, near, h, want="log", flags=flags)
    assert float((a - b).abs().max()) < 1e-4
    # and the fp16x2 input mode composes with it
    _, c = P.sdkde_eval(xd, qd, h, want="log", flags=flags | P.SDKDE_PREC_FP16X2)
    assert_log_density_close(c.cpu().numpy(), ref, f"shifted fp16x2 eval d={d}")


def test_profile_instrumentation_counts_launches_on_the_callers_stream():
    """sdkde_profile_enable / sdkde_profile_summary: one record per call and kind, on whatever stream the call was
    given, with durations that agree with stream events placed around the same calls."""
    import torch
    import paper_2602_10378_amd as P
    P.load()
    print("profile instrumentation", flush=True)
    x, q, h = sdkde_inputs.make("C1", seed=0, n=20000, m=3000)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ws = P.make_workspace(20000, 3000, 16)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    # Outputs allocated beforehand and three untimed calls on the side stream with recording on (which creates
    # the record's events), so that the timed region below holds launches only: the stream events also see
    # any gap the host leaves between launches.
    score = torch.empty_like(xd)
    P.sdkde_profile_enable(True)
    with torch.cuda.stream(side):
        for _ in range(3):
            P.sdkde_score(xd, h, out=score, workspace=ws)
    torch.cuda.synchronize()
    P.sdkde_profile_enable(False)
    # The stream events also see whatever pause the host takes between two launches (a garbage collection,
    # a page fault), so the comparison with them is made on the best of a few repetitions.
    share = 0.0
    for rep in range(5):
        P.sdkde_profile_enable(True)                   # starts an empty record
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(side):
            t0.record()
            for _ in range(3):
                P.sdkde_score(xd, h, out=score, workspace=ws)
            t1.record()
            P.sdkde_eval(xd, qd, h, workspace=ws)
        torch.cuda.synchronize()
        n_score, ms_score = P.sdkde_profile_summary(0)
        n_eval, ms_eval = P.sdkde_profile_summary(1)
        P.sdkde_profile_enable(False)
        assert (n_score, n_eval) == (3, 1)
        assert 0.0 < ms_score <= t0.elapsed_time(t1) and ms_eval > 0.0
        share = max(share, ms_score / t0.elapsed_time(t1))
    assert share > 0.5                                 # the pair kernel dominates a call of this size
    assert P.sdkde_profile_summary(0) == (0, 0.0)      # disabling reset the record


def test_concurrent_host_threads_with_their_own_streams(tuning):
    """Several host threads, each with its own workspace and stream, get the same bits as a lone call."""
    import threading
    import torch
    import paper_2602_10378_amd as P
    tuning(P.SDKDE_TUNE_SYM_MIN_ITEMS, 1)      # one of the threads runs the symmetric mode at a small size
    P.load()
    print("concurrent host threads", flush=True)
    cases = []
    for k, (n, m, d, flags) in enumerate([(6000, 800, 16, 0), (5000, 700, 20, 1), (7000, 900, 16, 32), (4000, 600, 2, 0)]):
        x, q, h = (sdkde_inputs.mixture_1d(n, m, 20 + k) if d == 1 else
                   sdkde_inputs.gaussian_mixture(n, m, d, 3, seed=20 + k))
        xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
        want_s = P.sdkde_score(xd, h, flags=flags)
        want_p = P.sdkde_eval(xd, qd, h, want="log", flags=flags)[1]
        cases.append((xd, qd, h, flags, want_s, want_p))
    torch.cuda.synchronize()
    failures = []

    def worker(case):
        xd, qd, h, flags, want_s, want_p = case
        try:
            stream = torch.cuda.Stream()
            ws = P.make_workspace(xd.shape[0], qd.shape[0], xd.shape[1], flags=flags)
            with torch.cuda.stream(stream):
                for _ in range(5):
                    s = P.sdkde_score(xd, h, workspace=ws, flags=flags, stream=stream)
                    p = P.sdkde_eval(xd, qd, h, want="log", workspace=ws, flags=flags, stream=stream)[1]
            stream.synchronize()
            if not (torch.equal(s, want_s) and torch.equal(p, want_p)):
                failures.append("result differs")
        except Exception as e:       # noqa: BLE001 - reported below, from the main thread
            failures.append(repr(e))

    threads = [threading.Thread(target=worker, args=(c,)) for c in cases]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads)
    assert not failures, failures


def test_outputs_need_no_more_than_float_alignment():
    """The C ABI takes plain float pointers: outputs (and the samples, for the shifted copy) that are only
    4-byte aligned must give the bits of the 16-byte aligned call (the epilogue then stores scalars)."""
    import torch
    import paper_2602_10378_amd as P
    P.load()
    print("unaligned outputs", flush=True)
    n, m, d = 3000, 100, 16
    x, q, h = sdkde_inputs.make("C1", seed=3, n=n, m=m)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ws = P.make_workspace(n, m, d)
    want_sd, _, want_log = P.sdkde_fit_eval(xd, qd, h, want="log", workspace=ws)
    want_s = P.sdkde_score(xd, h, workspace=ws)
    def shifted(t):
        buf = torch.empty(t.numel() + 1, dtype=torch.float32, device="cuda")
        view = buf[1:].view(t.shape)
        assert view.data_ptr() % 16 == 4
        return view
    s_out, sd_out, x_off = shifted(want_s), shifted(want_sd), shifted(xd)
    x_off.copy_(xd)
    P.sdkde_score(x_off, h, out=s_out, workspace=ws)
    assert torch.equal(s_out, want_s)
    _, _, got_log = P.sdkde_fit_eval(x_off, qd, h, score_out=s_out, samples_sd_out=sd_out, want="log", workspace=ws)
    assert torch.equal(sd_out, want_sd) and torch.equal(s_out, want_s) and torch.equal(got_log, want_log)


def test_default_workspace_serves_every_precision_mode():
    """A buffer from make_workspace with no flags must be accepted by every call in every precision mode: the
    number of partial-sum slots depends on the mode (at n = 100000 the fp32 plan takes more splits than the fp16
    ones), so the buffer is sized for the largest."""
    import torch
    import paper_2602_10378_amd as P
    P.load()
    print("default workspace, all precision modes", flush=True)
    n, m, d = 100000, 1000, 16
    x, q, h = sdkde_inputs.make("C1", seed=5, n=n, m=m)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ws = P.make_workspace(n, m, d)
    ref = None
    for flags in (P.SDKDE_PREC_FP32, P.SDKDE_PREC_FP16X2, P.SDKDE_PREC_FP16X2_ALL, P.SDKDE_PREC_FP16X2_PHI16, P.SDKDE_FLAG_MAX_SHIFT):
        s = P.sdkde_score(xd, h, workspace=ws, flags=flags)
        sp = P.sdkde_score(xd, h, points=qd, workspace=ws, flags=flags)
        _, logd = P.sdkde_eval(xd, qd, h, want="log", workspace=ws, flags=flags)
        if ref is None:
            ref = (s, sp, logd)
        else:       # the modes agree far inside the tolerance they are each held to against the oracle
            assert float((s - ref[0]).norm() / ref[0].norm()) < 1e-4
            assert float((sp - ref[1]).norm() / ref[1].norm()) < 1e-4
            assert float((logd - ref[2]).abs().max()) < 1e-3


def test_every_call_and_flag_accepts_the_default_workspace():
    """Seeded random shapes: a buffer from make_workspace (with the symmetric flag where that mode is asked for)
    is accepted by every entry point under every combination of flags, and the outputs are finite where they
    must be (no comparison with the oracle here: the parity tests do that)."""
    import random
    import torch
    import paper_2602_10378_amd as P
    P.load()
    rng = random.Random(7)
    for case in range(16):
        d = rng.choice([1, 3, 4, 6, 7, 8, 16, 17, 32, 48, 64, 96, 128])
        n = rng.choice([rng.randint(1, 3000), rng.randint(3000, 60000)])
        m = rng.choice([rng.randint(1, 300), rng.randint(300, 20000)])
        print(f"default workspace case {case}: n={n} m={m} d={d}", flush=True)
        gen = torch.Generator(device="cuda").manual_seed(case)
        x = torch.randn(n, d, device="cuda", generator=gen)
        q = torch.randn(m, d, device="cuda", generator=gen)
        h = 1.0 + 0.1 * d**0.5
        plain = P.make_workspace(n, m, d)
        symmetric = P.make_workspace(n, m, d, flags=P.SDKDE_FLAG_SYMMETRIC)
        for flags in (0, 1, 2, 3, 16, 17, 18, 19, 32, 48):
            ws = symmetric if flags & P.SDKDE_FLAG_SYMMETRIC else plain
            s = P.sdkde_score(x, h, workspace=ws, flags=flags)
            sp = P.sdkde_score(x, h, points=q, workspace=ws, flags=flags)
            _, logd = P.sdkde_eval(x, q, h, want="both", workspace=ws, flags=flags)
            lap = P.sdkde_eval_laplace(x, q, h, workspace=ws, flags=flags)
            x_sd, _, logd2 = P.sdkde_fit_eval(x, q, h, want="both", workspace=ws, flags=flags)
            for t in (s, sp, lap, x_sd):
                assert bool(torch.isfinite(t).all()), (case, flags)
            assert not bool(torch.isnan(logd).any()) and not bool(torch.isnan(logd2).any()), (case, flags)
            if flags & P.SDKDE_FLAG_MAX_SHIFT:
                assert bool(torch.isfinite(logd).all()), (case, flags)


def test_a_workspace_made_for_more_points_serves_fewer():
    """The decomposition is chosen per shape, and a smaller m can prefer more splits (more partial-sum slots) than
    the m a buffer was made for; the call then falls back to fewer splits instead of failing, with the same
    results to rounding."""
    import torch
    import paper_2602_10378_amd as P
    P.load()
    for n, m_made, m, d in ((72994, 73086, 54645, 16), (40000, 36000, 24000, 32)):
        size = P.sdkde_workspace_bytes(n, m_made, d)
        want_size = P.sdkde_describe_plan(n, m, d, 1)["workspace_bytes"]
        print(f"shared workspace n={n} made for m={m_made} ({size} B), used with m={m} (prefers {want_size} B)", flush=True)
        gen = torch.Generator(device="cuda").manual_seed(n)
        x = torch.randn(n, d, device="cuda", generator=gen)
        q = torch.randn(m, d, device="cuda", generator=gen)
        h = 1.5
        ws = torch.empty(size, dtype=torch.uint8, device="cuda")
        got_s = P.sdkde_score(x, h, points=q, workspace=ws)
        got_e = P.sdkde_eval(x, q, h, want="log", workspace=ws)[1]
        ref_s = P.sdkde_score(x, h, points=q)
        ref_e = P.sdkde_eval(x, q, h, want="log")[1]
        assert float((got_s - ref_s).norm() / ref_s.norm()) < 1e-5
        assert float((got_e - ref_e).abs().max()) < 1e-4
        assert torch.equal(got_s, P.sdkde_score(x, h, points=q, workspace=ws))      # still deterministic
    # the first shape is one where the preferred decomposition does not fit the shared buffer
    assert P.sdkde_describe_plan(72994, 54645, 16, 1)["workspace_bytes"] > P.sdkde_workspace_bytes(72994, 73086, 16)


def test_sweep_module_times_the_papers_shapes():
    """paper_2602_10378_amd.sweep (runtime and utilisation in the shapes of the paper's sweeps, n_test = n_train / 8):
    one small shape per dimension; times are positive, the whole SD-KDE pass costs more than the KDE alone, and no
    utilisation figure exceeds one."""
    from paper_2602_10378_amd import sweep
    for name, n, d in (("C1", 2048, 16), ("C3", 4096, 1)):
        print(f"sweep module: {name} n={n}", flush=True)
        rows = sweep.sweep(name, (n,), seeds=(0,), reps=5)
        assert len(rows) == 1 and rows[0]["n"] == n and rows[0]["m"] == n // 8 and rows[0]["d"] == d
        r = rows[0]
        assert 0.0 < r["kde_ms"] < r["sd_kde_ms"] < 50.0 and r["laplace_ms"] > 0.0
        assert 0.0 < r["share_of_bound"] < 1.0 and 0.0 < r["paper_model_utilisation"] < 1.0
        assert "| %d | %d |" % (n, n // 8) in sweep.markdown(rows, "t")
