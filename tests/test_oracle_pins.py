"""Pins for the CPU oracle: closed forms, quadrature, invariants, library special cases and
brute force, chosen so that a dropped term, a wrong sign/index or a wrong constant in the
oracle fails at least one of them.  Nothing here touches the GPU path."""
import math

import numpy as np
import pytest

import oracle
import sdkde_inputs

RNG = np.random.default_rng(1234)


def _rand(n, d, scale=1.0, rng=RNG):
    return rng.standard_normal((n, d)) * scale


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("d", [1, 2, 5, 16])
def test_single_sample_score_and_density(d):
    # n = 1: s(p) = -(p - x1)/h^2 for every p; p(q) = N(q; x1, h^2 I).
    x1 = _rand(1, d)
    p = _rand(7, d, 2.0)
    h = 0.83
    s = oracle.score(x1, h, points=p)
    np.testing.assert_allclose(s, -(p - x1) / h**2, rtol=1e-13, atol=1e-14)
    logp = oracle.eval_log_density(x1, p, h)
    want = -0.5 * np.sum((p - x1) ** 2, axis=1) / h**2 - d * math.log(h) - 0.5 * d * math.log(2 * math.pi)
    np.testing.assert_allclose(logp, want, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.eval_density(x1, p, h), np.exp(want), rtol=1e-12)


@pytest.mark.parametrize("d", [1, 3, 16])
def test_two_point_score_closed_form_and_exact_antisymmetry(d):
    x = _rand(2, d)
    h = 0.9
    phi = math.exp(-np.sum((x[0] - x[1]) ** 2) / (2 * h * h))
    s = oracle.score(x, h)
    want0 = (x[1] - x[0]) * phi / (h * h * (1 + phi))
    np.testing.assert_allclose(s[0], want0, rtol=1e-13)
    # exactly antisymmetric in IEEE arithmetic with direct differences
    assert np.array_equal(s[0], -s[1])


def test_identical_points_have_zero_score():
    x = np.tile(_rand(1, 4), (9, 1))
    s = oracle.score(x, 0.5)
    assert np.all(s == 0.0)
    np.testing.assert_array_equal(oracle.debias(x, s, 0.5), x)


def test_tiny_brute_force_by_hand():
    # n = 3, d = 2, every term written out.
    x = np.array([[0.0, 0.0], [1.0, 0.5], [-0.5, 2.0]])
    h = 0.75
    q = np.array([[0.25, 0.25]])

    def phi(a, b):
        return math.exp(-((a[0] - b[0]) ** 2 + (a[1] - b[1]) ** 2) / (2 * h * h))

    for i in range(3):
        den = sum(phi(x[i], x[j]) for j in range(3))
        num0 = sum(-(x[i][0] - x[j][0]) * phi(x[i], x[j]) for j in range(3))
        num1 = sum(-(x[i][1] - x[j][1]) * phi(x[i], x[j]) for j in range(3))
        s = oracle.score(x, h)[i]
        assert s[0] == pytest.approx(num0 / (h * h * den), rel=1e-13)
        assert s[1] == pytest.approx(num1 / (h * h * den), rel=1e-13)
    dens = sum(phi(q[0], x[j]) for j in range(3)) / (3 * h**2 * 2 * math.pi)
    assert oracle.eval_density(x, q, h)[0] == pytest.approx(dens, rel=1e-13)


def test_debias_is_x_plus_half_h2_score():
    x, s = _rand(11, 3), _rand(11, 3)
    h = 1.7
    np.testing.assert_allclose(oracle.debias(x, s, h), x + 0.5 * h * h * s, rtol=1e-15)
    # distinguishes h^2/2 from h/2 and h^2
    assert not np.allclose(oracle.debias(x, s, h), x + 0.5 * h * s)


# ---------------------------------------------------------------- quadrature (d = 1)

def test_1d_density_integrates_to_one_with_right_moments():
    x, _, h = sdkde_inputs.mixture_1d(400, 8, seed=3)
    x = x.astype(np.float64)
    s = oracle.score(x, h)
    x_sd = oracle.debias(x, s, h)
    lo, hi = x_sd.min() - 10 * h, x_sd.max() + 10 * h
    grid = np.linspace(lo, hi, 40001)
    p = oracle.eval_density(x_sd, grid.reshape(-1, 1), h)
    dx = grid[1] - grid[0]
    trap = lambda f: float(np.sum((f[1:] + f[:-1]) * 0.5) * dx)
    assert trap(p) == pytest.approx(1.0, abs=1e-10)
    assert trap(grid * p) == pytest.approx(float(x_sd.mean()), abs=1e-9)
    assert trap(grid**2 * p) == pytest.approx(float((x_sd**2).mean()) + h * h, abs=1e-8)


def test_2d_density_integrates_to_one():
    x = _rand(5, 2, 0.5)
    h = 0.4
    g = np.linspace(-5, 5, 501)
    xx, yy = np.meshgrid(g, g, indexing="ij")
    q = np.stack([xx.ravel(), yy.ravel()], axis=1)
    p = oracle.eval_density(x, q, h)
    assert float(p.sum() * (g[1] - g[0]) ** 2) == pytest.approx(1.0, abs=1e-8)


# ---------------------------------------------------------------- invariants

def make_cloud():
    x, q, h = sdkde_inputs.gaussian_mixture(300, 40, 5, components=3, seed=7)
    return x.astype(np.float64), q.astype(np.float64), h


@pytest.fixture(scope="module")
def cloud():
    return make_cloud()


def test_translation_invariance(cloud):
    x, q, h = cloud
    t = np.array([3.0, -1.0, 0.5, 10.0, -7.0])
    np.testing.assert_allclose(oracle.score(x + t, h), oracle.score(x, h), rtol=0, atol=1e-11)
    np.testing.assert_allclose(oracle.eval_log_density(x + t, q + t, h),
                               oracle.eval_log_density(x, q, h), rtol=0, atol=1e-11)


def test_sample_permutation_invariance(cloud):
    x, q, h = cloud
    perm = np.random.default_rng(0).permutation(len(x))
    np.testing.assert_allclose(oracle.score(x[perm], h), oracle.score(x, h)[perm], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.eval_log_density(x[perm], q, h),
                               oracle.eval_log_density(x, q, h), rtol=1e-13)


def test_rotation_equivariance(cloud):
    x, q, h = cloud
    rot, _ = np.linalg.qr(np.random.default_rng(5).standard_normal((5, 5)))
    np.testing.assert_allclose(oracle.score(x @ rot, h), oracle.score(x, h) @ rot, atol=1e-11)
    np.testing.assert_allclose(oracle.eval_log_density(x @ rot, q @ rot, h),
                               oracle.eval_log_density(x, q, h), atol=1e-11)


def test_scaling_equivariance(cloud):
    x, q, h = cloud
    a = 2.5
    np.testing.assert_allclose(oracle.score(a * x, a * h), oracle.score(x, h) / a, rtol=1e-11)
    np.testing.assert_allclose(oracle.eval_log_density(a * x, a * q, a * h),
                               oracle.eval_log_density(x, q, h) - x.shape[1] * math.log(a), atol=1e-11)


def test_momentum_identity(cloud):
    # sum_i D_i s(x_i) = 0 because (x_j - x_i) phi_ij is antisymmetric in (i, j).
    x, _, h = cloud
    n, d = x.shape
    dsum = oracle.eval_density(x, x, h) * n * h**d * (2 * math.pi) ** (d / 2)   # D_i
    s = oracle.score(x, h)
    tot = (dsum[:, None] * s).sum(axis=0)
    scale = np.abs(dsum[:, None] * s).sum(axis=0)
    assert np.all(np.abs(tot) <= 1e-12 * scale)
    assert np.all(dsum >= 1.0)         # self term contributes exactly 1


def test_mean_shift_identity(cloud):
    # x_sd = (x + T/D)/2 with T = Phi X: the shifted point is the midpoint of x and a convex
    # combination of the samples.
    x, _, h = cloud
    r2 = ((x[:, None, :] - x[None, :, :]) ** 2).sum(-1)
    phi = np.exp(-r2 / (2 * h * h))
    mean_shift = (phi @ x) / phi.sum(1, keepdims=True)
    x_sd = oracle.debias(x, oracle.score(x, h), h)
    np.testing.assert_allclose(x_sd, 0.5 * (x + mean_shift), rtol=1e-12, atol=1e-12)


def test_score_is_gradient_of_log_density(cloud):
    x, q, h = cloud
    s = oracle.score(x, h, points=q)
    eps = 1e-5 * h
    for k in range(x.shape[1]):
        e = np.zeros(x.shape[1])
        e[k] = eps
        fd = (oracle.eval_log_density(x, q + e, h) - oracle.eval_log_density(x, q - e, h)) / (2 * eps)
        np.testing.assert_allclose(s[:, k], fd, rtol=2e-6, atol=2e-7)


def test_bandwidth_limits(cloud):
    x, q, _ = cloud
    big = 1e4
    want = -(q - x.mean(0)) / big**2
    np.testing.assert_allclose(oracle.score(x, big, points=q), want, rtol=1e-5, atol=1e-5 * np.abs(want).max())
    s_small = oracle.score(x, 1e-3)        # neighbours vanish: only the self term is left
    assert np.max(np.abs(s_small)) < 1e-30


def test_far_query_does_not_underflow(cloud):
    x, _, h = cloud
    far = x.mean(0) + 500.0
    lp = oracle.eval_log_density(x, far[None, :], h)
    assert np.isfinite(lp[0]) and lp[0] < -1e4
    s = oracle.score(x, h, points=far[None, :])
    assert np.all(np.isfinite(s))


# ---------------------------------------------------------------- library special cases

def test_eval_matches_logsumexp_and_sklearn(cloud):
    from scipy.special import logsumexp
    x, q, h = cloud
    n, d = x.shape
    r2 = ((q[:, None, :] - x[None, :, :]) ** 2).sum(-1)
    want = logsumexp(-r2 / (2 * h * h), axis=1) - math.log(n) - d * math.log(h) - 0.5 * d * math.log(2 * math.pi)
    got = oracle.eval_log_density(x, q, h)
    np.testing.assert_allclose(got, want, rtol=1e-12)
    from sklearn.neighbors import KernelDensity
    kde = KernelDensity(kernel="gaussian", bandwidth=h, atol=0, rtol=0).fit(x)
    np.testing.assert_allclose(got, kde.score_samples(q), rtol=1e-10)


def test_gemm_form_agrees_with_direct_form():
    # The paper's regrouping: Gram-trick distances, T = Phi X, s = (T/D - x)/h^2.
    x, _, h = sdkde_inputs.gaussian_mixture(256, 1, 16, seed=2)
    x = x.astype(np.float64)
    nrm = (x * x).sum(1)
    r2 = nrm[:, None] + nrm[None, :] - 2.0 * (x @ x.T)
    phi = np.exp(-r2 / (2 * h * h))
    dsum = phi.sum(1, keepdims=True)
    s_gemm = ((phi @ x) / dsum - x) / (h * h)
    np.testing.assert_allclose(oracle.score(x, h), s_gemm, rtol=1e-9, atol=1e-10)


def test_laplace_corrected_matches_definition(cloud):
    # K_LC = K_h - (h^2/2) Laplacian K_h, checked against a finite-difference Laplacian of the
    # plain KDE (linear in the kernel) and against the closed-form factor for n = 1.
    x, q, h = cloud
    d = x.shape[1]
    x1 = x[:1]
    r2 = ((q - x1) ** 2).sum(1)
    k = np.exp(-r2 / (2 * h * h)) / ((2 * math.pi) ** (d / 2) * h**d)
    np.testing.assert_allclose(oracle.eval_laplace_density(x1, q, h), k * (1 + d / 2 - r2 / (2 * h * h)), rtol=1e-12)
    eps = 1e-3 * h
    lap = np.zeros(len(q))
    p0 = oracle.eval_density(x, q, h)
    for kk in range(d):
        e = np.zeros(d)
        e[kk] = eps
        lap += (oracle.eval_density(x, q + e, h) - 2 * p0 + oracle.eval_density(x, q - e, h)) / eps**2
    np.testing.assert_allclose(oracle.eval_laplace_density(x, q, h), p0 - 0.5 * h * h * lap, rtol=2e-5, atol=1e-12 * p0.max())


def test_laplace_abs_scale_bounds_signed_sum(cloud):
    x, q, h = cloud
    signed = oracle.eval_laplace_density(x, q, h)
    mag = oracle.eval_laplace_abs_density(x, q, h)
    assert np.all(mag >= np.abs(signed) * (1 - 1e-12))
    d = x.shape[1]
    r2 = ((q - x[:1]) ** 2).sum(1)
    k = np.exp(-r2 / (2 * h * h)) / ((2 * math.pi) ** (d / 2) * h**d)
    np.testing.assert_allclose(oracle.eval_laplace_abs_density(x[:1], q, h), k * np.abs(1 + d / 2 - r2 / (2 * h * h)), rtol=1e-12)


def test_laplace_integrates_to_one_1d():
    # the correction term -(h^2/2) Laplacian(K_h) integrates to zero, so p_LC keeps unit mass
    x, _, h = sdkde_inputs.mixture_1d(300, 4, seed=5)
    x = x.astype(np.float64)        # keep the grid arithmetic in double
    grid = np.linspace(x.min() - 12 * h, x.max() + 12 * h, 30001)
    p = oracle.eval_laplace_density(x, grid.reshape(-1, 1), h)
    dx = grid[1] - grid[0]
    assert float(np.sum((p[1:] + p[:-1]) * 0.5) * dx) == pytest.approx(1.0, abs=1e-9)
    assert p.min() < 0.0          # and it does go negative in the tails, as the paper notes


def test_gaussian_data_score_is_roughly_linear():
    rng = np.random.default_rng(11)
    sigma = 1.3
    x = sigma * rng.standard_normal((20000, 2))
    h = 1.0
    pts = np.array([[0.5, -0.3], [1.0, 1.0], [-0.8, 0.2]])
    s = oracle.score(x, h, points=pts)
    np.testing.assert_allclose(s, -pts / (sigma**2 + h * h), atol=0.03)


# ---------------------------------------------------------------- argument checking

def test_oracle_rejects_bad_arguments():
    x = _rand(4, 2)
    with pytest.raises(ValueError):
        oracle.score(x, 0.0)
    with pytest.raises(ValueError):
        oracle.score(x, float("nan"))
    with pytest.raises(ValueError):
        oracle.eval_density(x, _rand(3, 3), 1.0)


# ---------------------------------------------------------------- input recipe

def test_silverman_rule_reduces_to_1d_textbook_constant():
    x = RNG.standard_normal((1000, 1))
    h = sdkde_inputs.silverman_bandwidth(x)
    assert h == pytest.approx((4.0 / 3.0) ** 0.2 * x.std(ddof=1) * 1000 ** -0.2, rel=1e-12)
    assert (4.0 / 3.0) ** 0.2 == pytest.approx(1.06, abs=0.002)


def test_generators_are_seeded_and_shaped():
    a = sdkde_inputs.make("C1", seed=0, n=512, m=64)
    b = sdkde_inputs.make("C1", seed=0, n=512, m=64)
    c = sdkde_inputs.make("C1", seed=1, n=512, m=64)
    assert a[0].dtype == np.float32 and a[0].shape == (512, 16) and a[1].shape == (64, 16)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and a[2] == b[2]
    assert not np.array_equal(a[0], c[0])
    x, q, h = sdkde_inputs.make("C3", n=2048, m=100)
    assert x.shape == (2048, 1) and q[0, 0] == -5.0 and q[-1, 0] == 6.0
    x4, _, _ = sdkde_inputs.make("C4", n=4096, m=8)
    assert x4.shape == (4096, 64)
