"""GPU parity: the HIP library, called through its C ABI (ctypes binding), against the CPU
oracle on the same seeded inputs, element by element."""
import numpy as np
import pytest

import oracle
import sdkde_inputs
from parity import (TOL, gram_exponent_error, score_resolution, assert_density_close, assert_laplace_close, assert_log_density_close, assert_score_close,
                    assert_shifted_close)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import torch
    import paper_2602_10378_amd as P
    P.load()
    return P, torch


def _gpu_pipeline(P, torch, x, q, h):
    xd = torch.from_numpy(x).cuda()
    qd = torch.from_numpy(q).cuda()
    ws = P.make_workspace(x.shape[0], q.shape[0], x.shape[1])
    s = P.sdkde_score(xd, h, workspace=ws)
    x_sd = P.sdkde_debias(xd, s, h)
    dens, logd = P.sdkde_eval(x_sd, qd, h, want="both", workspace=ws)
    torch.cuda.synchronize()
    return s.cpu().numpy(), x_sd.cpu().numpy(), dens.cpu().numpy(), logd.cpu().numpy()


def _mixture(n, m, d, seed):
    if d == 1:
        return sdkde_inputs.mixture_1d(n, m, seed)
    return sdkde_inputs.gaussian_mixture(n, m, d, components=4, seed=seed, diag_cov=(d >= 64))


# sizes: several 16-sample tiles and row blocks plus ragged tails; d covers the thin path
# (1-3, and 4-6 for the score), the MFMA path with zero-padded columns (4-5 eval, 7, 20, 33, 100) and
# exact multiples of 16.
CASES = [
    (4096, 1024, 16, 0),     # config C1
    (1000, 333, 16, 1),
    (2049, 17, 16, 2),
    (3000, 777, 1, 0),
    (1500, 300, 2, 3),
    (1500, 300, 3, 4),
    (1200, 200, 4, 5),
    (1200, 200, 5, 6),
    (1300, 210, 6, 13),
    (1250, 190, 7, 14),
    (1100, 130, 20, 7),
    (1100, 130, 32, 8),
    (900, 100, 33, 9),
    (2048, 512, 64, 10),
    (700, 90, 100, 11),
    (700, 90, 128, 12),
]


@pytest.mark.parametrize("n,m,d,seed", CASES)
def test_pipeline_matches_oracle(lib, n, m, d, seed):
    P, torch = lib
    print(f"case n={n} m={m} d={d} seed={seed}", flush=True)
    x, q, h = _mixture(n, m, d, seed)
    s, x_sd, dens, logd = _gpu_pipeline(P, torch, x, q, h)
    s_ref, x_sd_ref, logp_ref = oracle.sd_kde_log_density(x, q, h)
    what = f"n={n} m={m} d={d}"
    assert_score_close(s, s_ref, what)
    assert_shifted_close(x_sd, x_sd_ref, s_ref, h, what)
    assert_log_density_close(logd, logp_ref, what)
    assert_density_close(dens, logp_ref, what)
    # stage-wise: eval alone on the oracle's shifted samples (rounded to fp32)
    x_sd32 = x_sd_ref.astype(np.float32)
    _, logd2 = P.sdkde_eval(torch.from_numpy(x_sd32).cuda(), torch.from_numpy(q).cuda(), h, want="log")
    assert_log_density_close(logd2.cpu().numpy(), oracle.eval_log_density(x_sd32, q, h), what + " eval-only")


@pytest.mark.parametrize("n,d", [(1, 16), (1, 1), (2, 16), (15, 16), (16, 16), (17, 5), (63, 2), (65, 64)])
def test_tiny_sample_sets(lib, n, d):
    P, torch = lib
    print(f"tiny n={n} d={d}", flush=True)
    rng = np.random.default_rng(100 + n + d)
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((9, d)).astype(np.float32)
    h = 0.8
    s, x_sd, dens, logd = _gpu_pipeline(P, torch, x, q, h)
    s_ref, _, logp_ref = oracle.sd_kde_log_density(x, q, h)
    if n == 1:
        assert np.all(s == 0.0)
    assert_score_close(s, s_ref, f"n={n} d={d}")
    assert_log_density_close(logd, logp_ref, f"n={n} d={d}")
    assert_density_close(dens, logp_ref, f"n={n} d={d}")


@pytest.mark.parametrize("d", [1, 3, 16, 40])
def test_score_at_separate_points(lib, d):
    P, torch = lib
    print(f"separate points d={d}", flush=True)
    x, q, h = _mixture(1300, 257, d, 21)
    got = P.sdkde_score(torch.from_numpy(x).cuda(), h, points=torch.from_numpy(q).cuda()).cpu().numpy()
    assert_score_close(got, oracle.score(x, h, points=q), f"points d={d}")


@pytest.mark.parametrize("n,m,d,seed", [(3000, 777, 1, 0), (1500, 300, 2, 3), (4096, 1024, 16, 0), (1000, 333, 16, 1),
                                        (1200, 200, 5, 6), (2048, 512, 64, 10), (17, 9, 16, 2)])
def test_laplace_corrected_kde_matches_oracle(lib, n, m, d, seed):
    P, torch = lib
    print(f"laplace n={n} m={m} d={d}", flush=True)
    x, q, h = _mixture(n, m, d, seed)
    got = P.sdkde_eval_laplace(torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda(), h).cpu().numpy()
    ref = oracle.eval_laplace_density(x, q, h)
    mag = oracle.eval_laplace_abs_density(x, q, h)
    assert_laplace_close(got, ref, mag, f"laplace n={n} d={d}")
    if d <= 16:
        assert (got < 0).any() or (ref >= 0).all()     # negative tails survive where the oracle has them


# fp16x2 input mode (inputs of the distance cross term split into two fp16 halves): a
# lower-precision-input mode, held to the same tolerances and with its error printed separately.
@pytest.mark.parametrize("d", [64, 70, 90, 112, 128])
@pytest.mark.parametrize("row_tiles", [2, 4])
def test_eval_kinds_at_large_dimension(lib, d, row_tiles, tuning):
    """From dp = 64 on the kinds without a second contraction run the kernel that stages the sample tile in
    LDS: plain, Laplace-corrected and max-shifted eval over several splits, with a ragged last tile and
    tiles of 320 / 384 / 448 / 512 float4s (not all multiples of the workgroup size)."""
    P, torch = lib
    n, m = 4500 + d, 301
    print(f"large-d eval kinds n={n} m={m} d={d} row tiles {row_tiles}", flush=True)
    tuning(P.SDKDE_TUNE_EVAL_ROW_TILES, row_tiles)       # both instantiations (the plan takes 2 at this size)
    x, q, h = _mixture(n, m, d, 70 + d)
    h = float(h) * (2.0 if d > 64 else 1.2)       # keep the sums inside the fp32 range without a shift
    plan = P.sdkde_describe_plan(n, m, d, 2)
    assert plan["splits"] >= 8 and plan["row_tiles"] == row_tiles
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ref = oracle.eval_log_density(x, q, h)
    lref, labs = oracle.eval_laplace_density(x, q, h), oracle.eval_laplace_abs_density(x, q, h)
    for flags in (0, P.SDKDE_FLAG_MAX_SHIFT):
        _, logd = P.sdkde_eval(xd, qd, h, want="log", flags=flags)
        assert_log_density_close(logd.cpu().numpy(), ref, f"large-d eval d={d} flags={flags}")
        lap = P.sdkde_eval_laplace(xd, qd, h, flags=flags).cpu().numpy()
        assert_laplace_close(lap, lref, labs, f"large-d laplace d={d} flags={flags}")
    # the score at separate points with the shift takes its row maxima from the same kernel
    sp = P.sdkde_score(xd, h, points=qd, flags=P.SDKDE_FLAG_MAX_SHIFT).cpu().numpy()
    assert_score_close(sp, oracle.score(x, h, points=q), f"large-d shifted score d={d}")


@pytest.mark.parametrize("mode", [1, 2, 3])
@pytest.mark.parametrize("n,m,d,seed", [(4096, 1024, 16, 0), (1000, 333, 16, 1), (1200, 200, 5, 6), (1100, 130, 20, 7),
                                        (2048, 512, 64, 10), (700, 90, 100, 11), (17, 9, 16, 2), (3000, 500, 1, 0)])
def test_fp16x2_input_mode_matches_oracle(lib, n, m, d, seed, mode):
    P, torch = lib
    flags = {1: P.SDKDE_PREC_FP16X2, 2: P.SDKDE_PREC_FP16X2_ALL, 3: P.SDKDE_PREC_FP16X2_PHI16}[mode]
    print(f"fp16x2 mode {mode} n={n} m={m} d={d}", flush=True)
    x, q, h = _mixture(n, m, d, seed)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    s = P.sdkde_score(xd, h, flags=flags)
    x_sd = P.sdkde_debias(xd, s, h)
    dens, logd = P.sdkde_eval(x_sd, qd, h, want="both", flags=flags)
    lap = P.sdkde_eval_laplace(xd, qd, h, flags=flags)
    sp = P.sdkde_score(xd, h, points=qd, flags=flags)
    s_ref, _, logp_ref = oracle.sd_kde_log_density(x, q, h)
    worst, frob = assert_score_close(s.cpu().numpy(), s_ref, f"fp16x2 d={d}")
    e_log = assert_log_density_close(logd.cpu().numpy(), logp_ref, f"fp16x2 d={d}")
    assert_density_close(dens.cpu().numpy(), logp_ref, f"fp16x2 d={d}")
    assert_laplace_close(lap.cpu().numpy(), oracle.eval_laplace_density(x, q, h), oracle.eval_laplace_abs_density(x, q, h),
                         f"fp16x2 laplace d={d}")
    assert_score_close(sp.cpu().numpy(), oracle.score(x, h, points=q), f"fp16x2 points d={d}")
    print(f"fp16x2 mode {mode} d={d}: score rel frobenius {frob:.3g} (worst {worst:.3g} of allowance), "
          f"log-density err {e_log:.3g}", flush=True)


# The fp16 second contraction (both the hi + lo split and the single-fp16 weights) also serves the score at
# separate points when the sums are max-shifted (largest weight 1): near points, far points (where the plain sums
# underflow and only the shift keeps a result), several splits and a ragged tail, at a full and a partly filled block.
@pytest.mark.parametrize("mode", [2, 3])
@pytest.mark.parametrize("n,m,d", [(5000, 1300, 16), (2100, 700, 9)])
def test_shifted_score_at_points_with_fp16_weights(lib, n, m, d, mode):
    P, torch = lib
    flags = mode | P.SDKDE_FLAG_MAX_SHIFT
    print(f"shifted score at points, mode {mode} n={n} m={m} d={d}", flush=True)
    x, q, h = _mixture(n, m, d, 23)
    q[: m // 2] += np.float32(9.0 * h / np.sqrt(d))       # half of the points 9 h away from where they were drawn
    plan = P.sdkde_describe_plan(n, m, d, 1, flags)
    assert plan["xt_scale"] == (2 if mode == 2 else 1) and plan["dp"] == 16
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    sp = P.sdkde_score(xd, h, points=qd, flags=flags)
    assert torch.equal(sp, P.sdkde_score(xd, h, points=qd, flags=flags))
    worst, frob = assert_score_close(sp.cpu().numpy(), oracle.score(x, h, points=q), f"mode {mode} shifted points d={d}")
    print(f"shifted score at points, mode {mode} d={d}: worst {worst:.3g} of allowance, rel frobenius {frob:.3g}", flush=True)


# A bandwidth well under the rule of thumb in 17-D leaves most samples without close neighbours: the
# weights that make up the score are then tiny (1e-7 and below), which is where a scaled fp16 split of
# Phi runs out of range.  The library uses that split only next to a weight of one (header, the
# FP16X2_ALL mode); the score at separate points must hold the plain tolerance in every mode, the score
# at the samples the tolerance plus the absolute term the header states.
@pytest.mark.parametrize("flags", [0, 1, 2, 18, 3, 19])
def test_score_with_narrow_bandwidth_in_every_mode(lib, flags):
    P, torch = lib
    n, m, d = 5445, 2306, 17
    print(f"narrow bandwidth n={n} m={m} d={d} flags={flags}", flush=True)
    x, q, h = sdkde_inputs.gaussian_mixture(n, m, d, components=1, seed=41)
    h *= 0.7
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    sp = P.sdkde_score(xd, h, points=qd, flags=flags).cpu().numpy()
    sp_ref = oracle.score(x, h, points=q)
    if flags & 16:
        keep = np.ones(m, bool)
    else:       # without the shift a point whose weights all underflow in fp32 gets the documented zero
        keep = np.isfinite(P.sdkde_eval(xd, qd, h, want="log", flags=flags)[1].cpu().numpy())
        assert keep.mean() > 0.5
    worst_p, _ = assert_score_close(sp[keep], sp_ref[keep], f"points flags={flags}")
    s = P.sdkde_score(xd, h, flags=flags).cpu().numpy().astype(np.float64)
    s_ref = oracle.score(x, h)
    ref = np.linalg.norm(s_ref, axis=1)
    allow = 1e-3 * np.maximum(ref, 1e-3 * np.sqrt(np.mean(ref**2)))
    if (flags & 15) in (2, 3):
        radius = np.linalg.norm(x - x.mean(0), axis=1).max()
        allow = allow + n * 2.0**-39 * radius / h**2
    worst_s = float(np.max(np.linalg.norm(s - s_ref, axis=1) / allow))
    print(f"narrow bandwidth flags={flags}: points {worst_p:.3g}, samples {worst_s:.3g} of allowance", flush=True)
    assert worst_s <= 1.0


# Evaluating one fitted estimate at batch after batch of queries: with SDKDE_FLAG_SAMPLES_PREPARED the samples
# prepared by the previous eval call on the same workspace are reused; the results must be the bits of a fresh call.
@pytest.mark.parametrize("n,d,flags", [(5000, 16, 0), (3000, 2, 0), (4000, 7, 0), (2500, 20, 1), (3000, 16, 16), (2000, 40, 17),
                                       (2500, 70, 0)])
def test_eval_with_samples_prepared_by_the_previous_call(lib, n, d, flags):
    P, torch = lib
    print(f"samples prepared n={n} d={d} flags={flags}", flush=True)
    x, q, h = _mixture(n, 1500, d, 12)
    xd = torch.from_numpy(x).cuda()
    batches = [torch.from_numpy(np.ascontiguousarray(q[a:b])).cuda() for a, b in ((0, 700), (700, 701), (701, 1500))]
    m_max = max(b.shape[0] for b in batches)
    ws = P.make_workspace(n, m_max, d, flags=flags)
    prepared = flags | P.SDKDE_FLAG_SAMPLES_PREPARED
    first = P.sdkde_eval(xd, batches[0], h, want="both", workspace=ws, flags=flags)
    for k, qb in enumerate(batches[1:]):
        got = P.sdkde_eval(xd, qb, h, want="both", workspace=ws, flags=prepared)
        lap = P.sdkde_eval_laplace(xd, qb, h, workspace=ws, flags=prepared)
        fresh_ws = P.make_workspace(n, m_max, d, flags=flags)
        want = P.sdkde_eval(xd, qb, h, want="both", workspace=fresh_ws, flags=flags)
        want_lap = P.sdkde_eval_laplace(xd, qb, h, workspace=fresh_ws, flags=flags)
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1]), f"batch {k + 1}"
        assert torch.equal(lap, want_lap), f"batch {k + 1} (Laplace)"
    assert_log_density_close(first[1].cpu().numpy(), oracle.eval_log_density(x, q[:700], h), "first batch")
    # the score calls do not take the flag, and the binding refuses to invent a workspace for it
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_score(xd, h, workspace=ws, flags=prepared)
    assert e.value.status == 2
    # A call whose precondition does not hold is answered with NaN in every output, not with numbers that belong
    # to other samples: another bandwidth, another sample array, a workspace last used by a score call, and a
    # workspace that never saw a preparation.
    qb = batches[0]
    def all_nan(result):
        return all(bool(torch.isnan(t).all()) for t in result)
    assert not all_nan(P.sdkde_eval(xd, qb, h, want="both", workspace=ws, flags=prepared))
    assert all_nan(P.sdkde_eval(xd, qb, h * 1.01, want="both", workspace=ws, flags=prepared))
    assert all_nan(P.sdkde_eval(xd.clone(), qb, h, want="both", workspace=ws, flags=prepared))
    assert all_nan([P.sdkde_eval_laplace(xd[:-1], qb, h, workspace=ws, flags=prepared)])
    P.sdkde_score(xd, h, workspace=ws, flags=flags)
    assert all_nan(P.sdkde_eval(xd, qb, h, want="both", workspace=ws, flags=prepared))
    assert all_nan(P.sdkde_eval(xd, qb, h, want="both", workspace=torch.zeros_like(ws), flags=prepared))
    with pytest.raises(ValueError):
        P.sdkde_eval(xd, batches[0], h, flags=prepared)


# Symmetric score (separate mode): every unordered pair of samples computed once.  Sizes span several sample
# blocks and groups of blocks with ragged tails; the tuning overrides force few groups (several blocks per
# work item, triangular items with more than one block) and the largest block size at small n.
@pytest.mark.parametrize("n,d,seed,env", [
    (5000, 16, 0, {}), (5000, 16, 1, {"SYM_GROUPS": 3}), (3000, 12, 2, {}), (7000, 20, 3, {}),
    (6100, 32, 4, {"SYM_GROUPS": 4}), (9000, 16, 5, {"SYM_BLOCK_ROWS": 2048}), (4000, 7, 6, {"SYM_GROUPS": 1}),
    (600, 16, 7, {}), (17, 8, 8, {}), (1, 16, 9, {})])
def test_symmetric_score_matches_oracle(lib, tuning, n, d, seed, env):
    P, torch = lib
    for key, value in env.items():
        tuning(getattr(P, "SDKDE_TUNE_" + key), value)
    tuning(P.SDKDE_TUNE_SYM_MIN_ITEMS, 1)      # the mode is otherwise declined below ~512 work items
    flags = P.SDKDE_FLAG_SYMMETRIC
    plan = P.sdkde_describe_plan(n, n, d, 0, flags)
    print(f"symmetric n={n} d={d} env={env} block={plan['sym_block_rows']} per_group={plan['sym_blocks_per_group']} "
          f"groups={plan['sym_groups']}", flush=True)
    assert plan["symmetric"] == 1
    if n == 1:      # the bandwidth rule needs two samples
        x, q, h = np.full((1, d), 0.25, np.float32), np.zeros((8, d), np.float32), 0.7
    else:
        x, q, h = _mixture(n, 8, d, seed)
    xd = torch.from_numpy(x).cuda()
    s = P.sdkde_score(xd, h, flags=flags)
    s_ref = oracle.score(x, h)
    worst, frob = assert_score_close(s.cpu().numpy(), s_ref, f"symmetric n={n} d={d}")
    assert torch.equal(s, P.sdkde_score(xd, h, flags=flags))       # deterministic: no atomics
    # the fused call takes the same path; its shifted samples carry the score
    ws = P.make_workspace(n, 8, d, flags=flags)
    s2 = torch.empty_like(xd)
    x_sd, _, _ = P.sdkde_fit_eval(xd, torch.from_numpy(q).cuda(), h, score_out=s2, want="both", workspace=ws, flags=flags)
    assert torch.equal(s2, s)
    assert_shifted_close(x_sd.cpu().numpy(), oracle.debias(x, s_ref, h), s_ref, h, f"symmetric x_sd n={n} d={d}")
    print(f"symmetric n={n} d={d}: worst {worst:.3g} of allowance, rel frobenius {frob:.3g}", flush=True)


def test_symmetric_flag_is_ignored_where_it_does_not_apply(lib, tuning):
    P, torch = lib
    sym = P.SDKDE_FLAG_SYMMETRIC
    # too few samples to fill the chip with its work items: declined
    assert P.sdkde_describe_plan(8192, 8192, 16, 0, sym)["symmetric"] == 0
    assert P.sdkde_describe_plan(32768, 32768, 16, 0, sym)["symmetric"] == 1
    tuning(P.SDKDE_TUNE_SYM_MIN_ITEMS, 1)
    for n, m, d, flags in ((3000, 500, 40, 0), (3000, 500, 16, P.SDKDE_PREC_FP16X2), (3000, 500, 2, 0)):
        print(f"symmetric flag ignored n={n} d={d} flags={flags}", flush=True)
        assert P.sdkde_describe_plan(n, n, d, 0, flags | sym)["symmetric"] == 0
        x, q, h = _mixture(n, m, d, 3)
        xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
        assert torch.equal(P.sdkde_score(xd, h, flags=flags | sym), P.sdkde_score(xd, h, flags=flags))
    # separate points and eval never take it
    x, q, h = _mixture(3000, 500, 16, 4)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    assert P.sdkde_describe_plan(3000, 500, 16, 1, sym)["symmetric"] == 0
    assert torch.equal(P.sdkde_score(xd, h, points=qd, flags=sym), P.sdkde_score(xd, h, points=qd))
    assert torch.equal(P.sdkde_eval(xd, qd, h, flags=sym)[0], P.sdkde_eval(xd, qd, h)[0])
    # where it applies it needs its own, larger workspace: one sized for the ordinary path is refused
    n_big = 40000
    xb = torch.from_numpy(_mixture(n_big, 8, 16, 5)[0]).cuda()
    small = torch.empty(P.sdkde_workspace_bytes(n_big, 8, 16, P.SDKDE_PREC_FP16X2_ALL), dtype=torch.uint8, device="cuda")
    assert P.sdkde_workspace_bytes(n_big, 8, 16, sym) > small.numel()
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_score(xb, 1.0, workspace=small, flags=sym)
    assert e.value.status == 3


@pytest.mark.parametrize("n,m,d,seed", [(4096, 1024, 16, 0), (1000, 333, 16, 1), (3000, 777, 1, 0), (2048, 512, 64, 10),
                                        (17, 9, 5, 2)])
def test_fused_call_matches_oracle_and_three_calls(lib, n, m, d, seed):
    P, torch = lib
    print(f"fused n={n} m={m} d={d}", flush=True)
    x, q, h = _mixture(n, m, d, seed)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    s = torch.empty_like(xd)
    x_sd, dens, logd = P.sdkde_fit_eval(xd, qd, h, score_out=s, want="both")
    s_ref, x_sd_ref, logp_ref = oracle.sd_kde_log_density(x, q, h)
    assert_score_close(s.cpu().numpy(), s_ref, f"fused d={d}")
    assert_shifted_close(x_sd.cpu().numpy(), x_sd_ref, s_ref, h, f"fused d={d}")
    assert_log_density_close(logd.cpu().numpy(), logp_ref, f"fused d={d}")
    assert_density_close(dens.cpu().numpy(), logp_ref, f"fused d={d}")
    # the separate calls give the same score and shifted samples bit for bit (same kernels, same order)
    s3 = P.sdkde_score(xd, h)
    assert torch.equal(s3, s) and torch.equal(P.sdkde_debias(xd, s3, h), x_sd)
    # without the optional score output
    x_sd2, _, logd2 = P.sdkde_fit_eval(xd, qd, h, want="log")
    assert torch.equal(x_sd2, x_sd) and torch.equal(logd2, logd)

@pytest.mark.parametrize("n,m,d,flags", [(4096, 1024, 16, 0), (3000, 333, 16, 0), (2048, 512, 9, 0), (1333, 77, 13, 0),
                                          (5000, 1, 7, 0), (3000, 700, 16, 1), (4096, 1024, 16, 2), (4096, 1024, 16, 3),
                                          (20000, 3000, 12, 0), (70000, 9000, 16, 0)])
def test_one_call_pass_with_and_without_the_folded_preparation(lib, tuning, n, m, d, flags):
    """sdkde_fit_eval prepares the eval pass's operands inside its score epilogue where the layouts allow it; with the
    knob that keeps the preparation in a launch of its own every output has the same bits, and the record the
    folded launch leaves lets a later SDKDE_FLAG_SAMPLES_PREPARED call reuse the prepared shifted samples."""
    P, torch = lib
    print(f"folded preparation n={n} m={m} d={d} flags={flags}", flush=True)
    assert P.sdkde_describe_plan(n, m, d, 2, flags)["fit_eval_fused_prep"] == 1
    x, q, h = _mixture(n, m, d, 91)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ws = P.make_workspace(n, m, d)
    outs = []
    for separate in (0, 1):
        tuning(P.SDKDE_TUNE_SEPARATE_PREP, separate)
        s = torch.full_like(xd, float("nan"))
        x_sd, dens, logd = P.sdkde_fit_eval(xd, qd, h, score_out=s, want="both", workspace=ws, flags=flags)
        if separate == 0:
            # the prepared shifted samples and their record are those of an eval call on x_sd
            _, again = P.sdkde_eval(x_sd, qd, h, want="log", workspace=ws, flags=flags | P.SDKDE_FLAG_SAMPLES_PREPARED)
            assert torch.equal(again, logd)
        outs.append([t.clone() for t in (s, x_sd, dens, logd)])
    for a, b, what in zip(outs[0], outs[1], ("score", "shifted samples", "density", "log density")):
        assert torch.isfinite(a).all() and torch.equal(a, b), f"{what} differs between the two forms"
    s_ref, x_sd_ref, logp_ref = oracle.sd_kde_log_density(x, q, h)
    if flags == 0:
        assert_score_close(outs[0][0].cpu().numpy(), s_ref, "folded preparation")
    assert_log_density_close(outs[0][3].cpu().numpy(), logp_ref, "folded preparation")


def test_single_sample_closed_form(lib):
    # n = 1: s(p) = -(p - x1)/h^2 exactly as in the paper's score formula.
    P, torch = lib
    x1 = np.array([[0.5, -1.0, 2.0, 0.25] * 4], dtype=np.float32)
    p = np.random.default_rng(3).standard_normal((50, 16)).astype(np.float32)
    h = 1.3
    got = P.sdkde_score(torch.from_numpy(x1).cuda(), h, points=torch.from_numpy(p).cuda()).cpu().numpy()
    assert_score_close(got, -(p.astype(np.float64) - x1) / h**2, "n=1")


def test_identical_samples_have_zero_score(lib):
    P, torch = lib
    x = np.tile(np.linspace(-1, 1, 16, dtype=np.float32), (200, 1))
    s = P.sdkde_score(torch.from_numpy(x).cuda(), 0.7).cpu().numpy()
    assert np.max(np.abs(s)) < 1e-5


@pytest.mark.parametrize("d", [1, 16])
def test_translation_far_from_origin(lib, d):
    # The library centres on a mean of the samples, so a large common offset must not cost accuracy
    # beyond the rounding of the shifted fp32 inputs themselves.
    P, torch = lib
    x, q, h = _mixture(2000, 200, d, 31)
    off = np.float32(1000.0)
    xo, qo = (x + off).astype(np.float32), (q + off).astype(np.float32)
    s, _, _, logd = _gpu_pipeline(P, torch, xo, qo, h)
    s_ref, _, logp_ref = oracle.sd_kde_log_density(xo, qo, h)
    assert_score_close(s, s_ref, f"offset d={d}")
    assert_log_density_close(logd, logp_ref, f"offset d={d}")


# The stated accuracy domain of the matrix path: the Gram expansion on centred coordinates loses about
# (R/h)^2 2^-24 in the exponent, R = distance from the centre, so the tolerances hold while R/h stays below ~100.
# Two unit-covariance clusters 2R apart put every point at distance ~R from the centre between them.
@pytest.mark.parametrize("ratio", [25.0, 50.0, 90.0])
@pytest.mark.parametrize("flags", [0, 1])
def test_accuracy_domain_of_the_gram_expansion(lib, ratio, flags):
    P, torch = lib
    n, m, d = 4000, 400, 16
    rng = np.random.default_rng(int(ratio))
    direction = rng.standard_normal(d)
    direction /= np.linalg.norm(direction)
    h = 1.1
    side = np.where(rng.random(n + m) < 0.5, -1.0, 1.0)[:, None]
    pts = (rng.standard_normal((n + m, d)) + side * ratio * h * direction).astype(np.float32)
    x, q = np.ascontiguousarray(pts[:n]), np.ascontiguousarray(pts[n:])
    print(f"accuracy domain R/h={ratio} flags={flags}", flush=True)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    s = P.sdkde_score(xd, h, flags=flags)
    _, logd = P.sdkde_eval(xd, qd, h, want="log", flags=flags)
    worst, frob = assert_score_close(s.cpu().numpy(), oracle.score(x, h), f"R/h={ratio}")
    e_log = assert_log_density_close(logd.cpu().numpy(), oracle.eval_log_density(x, q, h), f"R/h={ratio}")
    print(f"accuracy domain R/h={ratio} flags={flags}: score worst {worst:.3g} of allowance (rel frobenius {frob:.3g}), "
          f"log-density err {e_log:.3g}", flush=True)


@pytest.mark.parametrize("order", ["sorted", "periodic"])
@pytest.mark.parametrize("d", [16, 40])
def test_centre_of_a_strided_subsample_copes_with_ordered_samples(lib, d, order):
    """The centre is the mean of an evenly strided subsample of the samples.  Orderings that could fool a
    subsample must not cost accuracy: samples sorted by mixture component (a prefix would see one cluster), and
    samples arranged so that every row the subsample picks (stride n / rows) comes from the same component, which
    puts the centre inside one cluster instead of between them."""
    P, torch = lib
    n, m = 8192, 300
    x, q, h = sdkde_inputs.gaussian_mixture(n, m, d, components=4, seed=61)
    key = np.linalg.norm(x - x[0], axis=1)                  # the component of x[0] first, the others by distance
    by_cluster = np.argsort(key, kind="stable")
    if order == "sorted":
        x = np.ascontiguousarray(x[by_cluster])
    else:
        rows = max(32, 4096 // d)
        stride = n // rows
        picked = np.arange(rows) * stride                   # the rows the subsample reads
        rest = np.setdiff1d(np.arange(n), picked)
        arranged = np.empty_like(x)
        arranged[picked] = x[by_cluster[:rows]]             # all from the cluster of x[0]
        arranged[rest] = x[by_cluster[rows:]]
        x = arranged
    print(f"ordered samples d={d} {order}", flush=True)
    s, x_sd, dens, logd = _gpu_pipeline(P, torch, x, q, h)
    s_ref, x_sd_ref, logp_ref = oracle.sd_kde_log_density(x, q, h)
    worst, frob = assert_score_close(s, s_ref, f"{order} d={d}")
    assert_shifted_close(x_sd, x_sd_ref, s_ref, h, f"{order} d={d}")
    e_log = assert_log_density_close(logd, logp_ref, f"{order} d={d}")
    print(f"ordered samples d={d} {order}: score worst {worst:.3g} of allowance (rel frobenius {frob:.3g}), log err {e_log:.3g}",
          flush=True)


@pytest.mark.parametrize("d", [1, 16, 64])
def test_bitwise_deterministic(lib, d):
    P, torch = lib
    x, q, h = _mixture(3000, 500, d, 41)
    a = _gpu_pipeline(P, torch, x, q, h)
    b = _gpu_pipeline(P, torch, x, q, h)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_permutation_of_samples(lib):
    P, torch = lib
    x, q, h = _mixture(2500, 300, 16, 51)
    perm = np.random.default_rng(0).permutation(len(x))
    s1, _, _, l1 = _gpu_pipeline(P, torch, x, q, h)
    s2, _, _, l2 = _gpu_pipeline(P, torch, np.ascontiguousarray(x[perm]), q, h)
    assert_score_close(s2, s1[perm].astype(np.float64), "perm")
    assert np.max(np.abs(l1 - l2)) < 1e-4


def test_far_query_and_far_point(lib):
    # every phi underflows in fp32: documented behaviour is log density -inf, density 0, score 0
    P, torch = lib
    x, _, h = _mixture(500, 1, 16, 61)
    far = (x.mean(0, keepdims=True) + 1e3).astype(np.float32)
    xd, fd = torch.from_numpy(x).cuda(), torch.from_numpy(far).cuda()
    dens, logd = P.sdkde_eval(xd, fd, h, want="both")
    assert dens.item() == 0.0 and logd.item() == float("-inf")
    assert np.all(P.sdkde_score(xd, h, points=fd).cpu().numpy() == 0.0)

@pytest.mark.parametrize("flags", [0, 1, 16])
def test_weight_sums_below_the_normal_range_are_reported_as_underflow(lib, flags):
    """Three samples and queries up to 15 h away (found by a wider random sweep than the committed one): the GPU's
    exp2 flushes weights below 2^-126 to zero, so with all three samples ~13.1 h from a query part of the sum was
    lost and the log density came back finite but off by up to 0.56.  Now a sum that the flushed weights could
    change by more than 1e-3 (below 1000 n 2^-126) is the all-underflow case (log density -inf, density 0, score
    0), every finite result is within tolerance, and the max-shifted mode evaluates every query."""
    P, torch = lib
    n, m, d = 3, 1114, 12
    x, q, h = sdkde_inputs.gaussian_mixture(n, m, d, 3, 213145, diag_cov=True)
    h = float(h) * 1.5
    print(f"underflow band n={n} m={m} d={d} h={h:.4f} flags={flags}", flush=True)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    dens, logd = P.sdkde_eval(xd, qd, h, want="both", flags=flags)
    dens, logd = dens.cpu().numpy(), logd.cpu().numpy().astype(np.float64)
    sp = P.sdkde_score(xd, h, points=qd, flags=flags).cpu().numpy()
    ref = oracle.eval_log_density(x, q, h)
    s_ref = oracle.score(x, h, points=q)
    # log of the plain weight sum, and the least sum the library still trusts
    log_sum = ref + np.log(n) + d * np.log(h) + 0.5 * d * np.log(2.0 * np.pi)
    cut = np.log(1000.0 * n) - 126.0 * np.log(2.0)
    fin = np.isfinite(logd)
    if flags & 16:
        assert fin.all()
        assert np.max(np.abs(logd - ref)) <= TOL
        assert_score_close(sp, s_ref, "underflow band, shifted")
        return
    assert 0.5 < fin.mean() < 0.95, "the case must have queries on both sides of the cut"
    assert np.max(np.abs(logd[fin] - ref[fin])) <= TOL
    assert np.all(log_sum[fin] > cut - 0.01) and np.all(log_sum[~fin] < cut + 0.01)
    assert np.all(dens[~fin] == 0.0) and np.all(logd[~fin] == -np.inf)
    clear_in, clear_out = log_sum > cut + 0.01, log_sum < cut - 0.01
    assert np.all(sp[clear_out] == 0.0)
    assert_score_close(sp[clear_in], s_ref[clear_in], "underflow band, score at the queries")


def test_laplace_of_a_heavy_tailed_cloud_on_the_thin_path(lib):
    """2-D Student-t samples (3 degrees of freedom) reach 180 h from their centre; tail queries have Laplace terms that
    cancel a thousandfold, and the direct-difference path's own rounding of the squared distance shows there (found
    by the sweep over data shapes: 1.9 of the two-part allowance).  The derived allowance holds."""
    P, torch = lib
    g = np.random.default_rng(12130)
    x = g.standard_t(3, size=(9391, 2)).astype(np.float32)
    q = g.standard_t(3, size=(4805, 2)).astype(np.float32)
    h = float(sdkde_inputs.silverman_bandwidth(x))
    print(f"laplace heavy tails n={len(x)} m={len(q)} d=2 h={h:.4f}", flush=True)
    lap = P.sdkde_eval_laplace(torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda(), h).cpu().numpy()
    ref, mag = oracle.eval_laplace_density(x, q, h), oracle.eval_laplace_abs_density(x, q, h)
    kde = np.exp(oracle.eval_log_density(x, q, h))
    worst = assert_laplace_close(lap, ref, mag, "laplace heavy tails", exponent_error=gram_exponent_error(x, q, h), p_kde_ref=kde)
    print(f"laplace heavy tails: worst error {worst:.3g} of the allowance", flush=True)


@pytest.mark.parametrize("flags", [0, 1, 16])
def test_laplace_where_the_terms_cancel_a_thousandfold(lib, flags):
    """One 24-D Gaussian at the rule-of-thumb bandwidth (found by a wider random sweep than the committed one): the
    samples lie 7 - 12 h from their centre, the Laplace terms of a tail query cancel to 1e-3 of their magnitude,
    and what the fp32 Gram expansion loses in every exponent shows in the signed sum (1.4e-5 of the terms'
    magnitude, fp32 path).  The allowance derived from that arithmetic (parity.gram_exponent_error) holds."""
    P, torch = lib
    n, m, d = 11437, 1036, 24
    x, q, h = sdkde_inputs.gaussian_mixture(n, m, d, 1, 112423, diag_cov=False)
    print(f"laplace cancellation n={n} m={m} d={d} h={h:.4f} flags={flags}", flush=True)
    lap = P.sdkde_eval_laplace(torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda(), h, flags=flags).cpu().numpy()
    ref, mag = oracle.eval_laplace_density(x, q, h), oracle.eval_laplace_abs_density(x, q, h)
    kde = np.exp(oracle.eval_log_density(x, q, h))
    assert np.min(np.abs(ref[mag >= 1e-30]) / mag[mag >= 1e-30]) < 2e-3, "the case must have cancelling sums"
    bound = gram_exponent_error(x, q, h, low_precision_inputs=bool(flags & 15))
    worst = assert_laplace_close(lap, ref, mag, f"laplace cancellation flags={flags}", exponent_error=bound, p_kde_ref=kde)
    print(f"laplace cancellation flags={flags}: worst error {worst:.3g} of the allowance", flush=True)

@pytest.mark.parametrize("d,flags,h", [(32, 0, 0.8), (32, 1, 0.8), (16, 2, 0.45), (3, 0, 0.25)])
def test_scores_that_vanish_against_one_over_h(lib, d, flags, h):
    """Every sample has exact duplicates and no other neighbour within reach (found by a sweep over data shapes the
    mixtures do not have): the true score is ~1e-10 / h and below, and the paper's p D - T form of the numerator
    cannot resolve it in fp32.  What is lost is bounded in absolute terms (parity.score_resolution), and the thin
    path, which forms the differences directly, returns the zero."""
    P, torch = lib
    g = np.random.default_rng(343)
    if d > 3:
        base = g.standard_normal((50, d))
    else:           # 50 distinct points of a 5 x 5 x 5 lattice with spacing 5 (20 h apart)
        cells = g.permutation(125)[:50]
        base = 5.0 * np.stack([cells % 5, (cells // 5) % 5, cells // 25], axis=1).astype(np.float64)
    x = base[g.integers(0, 50, size=355)].astype(np.float32)
    print(f"vanishing score d={d} flags={flags} h={h}", flush=True)
    s = P.sdkde_score(torch.from_numpy(x).cuda(), h, flags=flags).cpu().numpy()
    s_ref = oracle.score(x, h)
    scale = np.linalg.norm(s_ref, axis=1).max() * h
    assert scale < 1e-6, f"the case must have a vanishing score field (largest |s| h = {scale:.2e})"
    err = np.linalg.norm(s.astype(np.float64) - s_ref, axis=1)
    if d <= 3:
        assert err.max() * h < 1e-12
    else:
        worst = float(np.max(err / score_resolution(x, x, h)))
        print(f"vanishing score d={d} flags={flags}: largest error {err.max() * h:.2e} / h, {worst:.3g} of the resolution", flush=True)
        assert worst <= 1.0


def test_argument_errors(lib):
    P, torch = lib
    x = torch.zeros((64, 16), device="cuda")
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_score(x, 0.0)
    assert e.value.status == 1
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_score(x, float("nan"))
    assert e.value.status == 1
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_score(x, 1.0, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 3
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_score(torch.zeros((8, 200), device="cuda"), 1.0)
    assert e.value.status == 2
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_eval(x, torch.zeros((4, 16), device="cuda"), -1.0)
    assert e.value.status == 1
    # empty query set is a no-op
    dens, _ = P.sdkde_eval(x, torch.zeros((0, 16), device="cuda"), 1.0)
    assert dens.numel() == 0
