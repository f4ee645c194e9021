"""Pins for the verification part of the oracle (CPU only).

Each test checks the oracle against something the paper or the mathematics
fixes independently of the oracle's own formula: library Gaussian densities,
the closed-form acceptance rate of App. D, exact preservation of the target
marginal (App. B), the reflection geometry of Lemmas 1-2, the 1-D special
case of Sec. 3.3, and the lambda properties stated after Eq. (acc_relax).
"""
import math
import os

import numpy as np
import pytest
from scipy import stats
from scipy.special import ndtr

from oracle import free_oracle as fo


def _case(d, seed, sep=1.0, sigma=0.3):
    rng = np.random.default_rng(seed)
    m = rng.standard_normal(d)
    dirn = rng.standard_normal(d)
    dirn /= np.linalg.norm(dirn)
    m_hat = m + sep * sigma * dirn
    x_hat = m_hat + sigma * rng.standard_normal(d)
    return m_hat, m, sigma, x_hat


# ---- likelihood ratio: Eq. (qp) against library log-densities ---------------
@pytest.mark.parametrize("d", [1, 4, 256])
def test_log_ratio_matches_library_gaussian_logpdf(d):
    for seed in range(5):
        m_hat, m, sigma, x_hat = _case(d, seed, sep=0.7)
        lq = stats.multivariate_normal(mean=m, cov=sigma ** 2).logpdf(x_hat)
        lp = stats.multivariate_normal(mean=m_hat, cov=sigma ** 2).logpdf(x_hat)
        assert fo.log_ratio(m_hat, m, sigma, x_hat) == pytest.approx(lq - lp, rel=1e-10, abs=1e-10)


def test_log_ratio_equals_squared_norm_form():
    m_hat, m, sigma, x_hat = _case(64, 3)
    direct = (np.sum((x_hat - m_hat) ** 2) - np.sum((x_hat - m) ** 2)) / (2 * sigma ** 2)
    assert fo.log_ratio(m_hat, m, sigma, x_hat) == pytest.approx(direct, rel=1e-11)


def test_accept_rule_is_the_density_ratio_test():
    """u <= min(1, q/p) with q, p from the library, on a grid of u."""
    for seed in range(20):
        m_hat, m, sigma, x_hat = _case(4, seed, sep=2.0)
        q = stats.multivariate_normal(mean=m, cov=sigma ** 2).pdf(x_hat)
        p = stats.multivariate_normal(mean=m_hat, cov=sigma ** 2).pdf(x_hat)
        for u in (0.0, 1e-6, 0.1, 0.3, 0.5, 0.7, 0.9, 0.999999):
            _, ok, _, _ = fo.verification(m_hat, m, sigma, x_hat, u)
            assert ok == (u <= min(1.0, q / p))


# ---- closed-form acceptance rate (App. D) and maximal coupling (App. B) -----
def _golden_rows(golden_dir):
    return [tuple(map(float, l.split())) for l in open(os.path.join(golden_dir, "acceptance_closed_form.txt"))
            if l.strip() and not l.startswith("#")]


def test_empirical_acceptance_matches_tabulated_closed_form(golden_dir):
    """Oracle acceptance frequency against the tabulated 2*Phi(-D/2) values."""
    rng = np.random.default_rng(42)
    n, d, sigma = 40_000, 3, 0.7
    for dist, val in _golden_rows(golden_dir):
        assert 2 * ndtr(-dist / 2) == pytest.approx(val, abs=5e-5)
        m = rng.standard_normal(d)
        dirn = rng.standard_normal(d)
        dirn /= np.linalg.norm(dirn)
        m_hat = m + dist * sigma * dirn
        xs = m_hat + sigma * rng.standard_normal((n, d))
        us = rng.random(n)
        acc = sum(fo.verification(m_hat, m, sigma, xs[i], us[i])[1] for i in range(n))
        se = math.sqrt(max(val * (1 - val), 1e-12) / n)
        assert abs(acc / n - val) < 4.5 * se + 5e-5


@pytest.mark.parametrize("d,sep", [(1, 1.0), (4, 0.5), (4, 2.0), (16, 1.0)])
def test_empirical_acceptance_matches_closed_form(d, sep):
    rng = np.random.default_rng(100 + d)
    n = 100_000
    sigma = 0.25
    m = rng.standard_normal(d)
    dirn = rng.standard_normal(d)
    dirn /= np.linalg.norm(dirn)
    m_hat = m + sep * sigma * dirn
    xs = m_hat + sigma * rng.standard_normal((n, d))
    us = rng.random(n)
    acc = 0
    moved = 0
    for i in range(n):
        x, ok, _, _ = fo.verification(m_hat, m, sigma, xs[i], us[i])
        acc += ok
        moved += not np.array_equal(x, xs[i])
    expect = 2 * ndtr(-sep / 2)               # E[a] = 2 Phi(-||m^-m||/(2 sigma))
    se = math.sqrt(expect * (1 - expect) / n)
    assert abs(acc / n - expect) < 4.5 * se
    # maximal coupling: P(x != x^) = TV(p, q) = 1 - E[a]
    assert moved == n - acc


def test_spec_verify_rate_matches_closed_form_with_realised_norms():
    """Per-draft decisions of the batched entry point: the mean of the
    closed-form rates at the realised ||m^-m||/sigma predicts the empirical rate."""
    rng = np.random.default_rng(7)
    n_traj, K, d = 4000, 3, 8
    sigma = rng.uniform(0.05, 0.2, (n_traj, K))
    m = rng.standard_normal((n_traj, K, d))
    m_hat = m + 0.4 * sigma[..., None] * rng.standard_normal((n_traj, K, d))
    x_hat = m_hat + sigma[..., None] * rng.standard_normal((n_traj, K, d))
    u = rng.random((n_traj, K))
    res = fo.spec_verify(m, m_hat, x_hat, sigma, u)
    dist = np.linalg.norm(m_hat - m, axis=-1) / sigma
    expect = (2 * ndtr(-dist / 2)).mean()
    n = n_traj * K
    assert abs(res["accept"].mean() - expect) < 4.5 * math.sqrt(expect * (1 - expect) / n)


# ---- the output has the target distribution (App. B, unbiasedness) ----------
def _run_many(d, sep, n, seed):
    rng = np.random.default_rng(seed)
    sigma = 0.5
    m = rng.standard_normal(d)
    dirn = rng.standard_normal(d)
    dirn /= np.linalg.norm(dirn)
    m_hat = m + sep * sigma * dirn
    xs = m_hat + sigma * rng.standard_normal((n, d))
    us = rng.random(n)
    out = np.empty((n, d))
    for i in range(n):
        out[i] = fo.verification(m_hat, m, sigma, xs[i], us[i])[0]
    return out, m, m_hat, sigma, dirn


def test_marginal_preserved_1d():
    out, m, m_hat, sigma, _ = _run_many(1, 1.5, 100_000, 11)
    assert stats.kstest((out[:, 0] - m[0]) / sigma, "norm").pvalue > 1e-3
    # and the proposal itself would fail the same test (the test has power)
    rng = np.random.default_rng(5)
    prop = m_hat[0] + sigma * rng.standard_normal(100_000)
    assert stats.kstest((prop - m[0]) / sigma, "norm").pvalue < 1e-6


def test_marginal_preserved_4d():
    out, m, m_hat, sigma, dirn = _run_many(4, 1.5, 100_000, 12)
    z = (out - m) / sigma
    for j in range(4):
        assert stats.kstest(z[:, j], "norm").pvalue > 1e-3
    assert stats.kstest(z @ dirn, "norm").pvalue > 1e-3
    assert stats.kstest((z ** 2).sum(axis=1), "chi2", args=(4,)).pvalue > 1e-3


# ---- reflection geometry (Lemmas 1-2; 1-D case of Sec. 3.3) ------------------
def test_reflection_1d_is_mirror_about_midpoint():
    for m_hat, m, x_hat in [(0.3, -0.2, 1.7), (-1.0, 2.0, 0.1), (5.0, 4.9, 5.2)]:
        x = fo.reflect(np.array([m_hat]), np.array([m]), np.array([x_hat]))
        assert x[0] == pytest.approx(2 * 0.5 * (m + m_hat) - x_hat, abs=1e-14)


@pytest.mark.parametrize("d", [2, 4, 257])
def test_reflection_invariants(d):
    m_hat, m, sigma, x_hat = _case(d, 21, sep=3.0)
    x = fo.reflect(m_hat, m, x_hat)
    e = (m_hat - m) / np.linalg.norm(m_hat - m)
    mid = 0.5 * (m + m_hat)
    # isometry / distance swap (Lemma 2)
    assert np.linalg.norm(x - m) == pytest.approx(np.linalg.norm(x_hat - m_hat), rel=1e-12)
    assert np.linalg.norm(x - m_hat) == pytest.approx(np.linalg.norm(x_hat - m), rel=1e-12)
    # mirror across the hyperplane through mid with normal e (Lemma 1)
    assert np.dot(x - mid, e) == pytest.approx(-np.dot(x_hat - mid, e), rel=1e-10)
    perp = lambda v: v - np.dot(v, e) * e
    np.testing.assert_allclose(perp(x - mid), perp(x_hat - mid), atol=1e-12)
    # density swap: p(x^) = q(S(x^))
    lp = stats.multivariate_normal(mean=m_hat, cov=sigma ** 2).logpdf(x_hat)
    lq = stats.multivariate_normal(mean=m, cov=sigma ** 2).logpdf(x)
    assert lp == pytest.approx(lq, rel=1e-10)
    # a reflection is an involution: mirroring x again across the same plane gives x^
    back = x - 2 * e * np.dot(x - mid, e)
    np.testing.assert_allclose(back, x_hat, atol=1e-12)


def test_householder_matrix_form():
    """x = m + (I - 2 e e^T)(x^ - m^) with the matrix built explicitly."""
    m_hat, m, _, x_hat = _case(6, 33, sep=2.0)
    e = ((m_hat - m) / np.linalg.norm(m_hat - m)).reshape(-1, 1)
    R = np.eye(6) - 2 * e @ e.T
    np.testing.assert_allclose(R.T @ R, np.eye(6), atol=1e-14)
    np.testing.assert_allclose(fo.reflect(m_hat, m, x_hat), m + R @ (x_hat - m_hat), atol=1e-13)


# ---- relaxed rule (Eq. acc_relax) -------------------------------------------
def test_lambda_one_is_strict_and_zero_accepts_all():
    rng = np.random.default_rng(2)
    for seed in range(50):
        m_hat, m, sigma, x_hat = _case(8, seed, sep=2.5)
        u = rng.random()
        strict = fo.verification(m_hat, m, sigma, x_hat, u)
        relaxed1 = fo.verification(m_hat, m, sigma, x_hat, u, lam=1.0)
        assert strict[1] == relaxed1[1] and np.array_equal(strict[0], relaxed1[0])
        assert fo.verification(m_hat, m, sigma, x_hat, u, lam=0.0)[1] is True


def test_relaxed_rule_matches_scaled_direction_formula():
    """acc_lambda = min(1, exp(v^T (x^ - mid)/sigma^2)), v = lambda (m - m^)."""
    rng = np.random.default_rng(3)
    for seed in range(200):
        m_hat, m, sigma, x_hat = _case(5, seed, sep=2.0)
        lam, u = rng.uniform(0, 1), rng.random()
        v = lam * (m - m_hat)
        a = min(1.0, math.exp(np.dot(v, x_hat - 0.5 * (m + m_hat)) / sigma ** 2))
        assert fo.verification(m_hat, m, sigma, x_hat, u, lam=lam)[1] == (u <= a)


def test_smaller_lambda_is_more_permissive():
    rng = np.random.default_rng(4)
    for seed in range(200):
        m_hat, m, sigma, x_hat = _case(5, seed, sep=3.0)
        u = rng.random()
        prev = False
        for lam in (1.0, 0.8, 0.5, 0.2, 0.0):       # accept set can only grow
            ok = fo.verification(m_hat, m, sigma, x_hat, u, lam=lam)[1]
            assert ok or not prev
            prev = ok


def test_relaxed_rejection_reflects_with_the_same_direction():
    m_hat, m, sigma, x_hat = _case(7, 9, sep=6.0)
    x1, ok1, _, _ = fo.verification(m_hat, m, sigma, x_hat, 0.999999, lam=1.0)
    x2, ok2, _, _ = fo.verification(m_hat, m, sigma, x_hat, 0.999999, lam=0.9)
    if not ok1 and not ok2:
        np.testing.assert_array_equal(x1, x2)


# ---- sequential scan and degenerate cases -----------------------------------
def test_n_accept_is_length_of_accepted_prefix():
    rng = np.random.default_rng(8)
    n_traj, K, d = 300, 6, 4
    sigma = np.full((n_traj, K), 0.3)
    m = rng.standard_normal((n_traj, K, d))
    m_hat = m + 0.3 * rng.standard_normal((n_traj, K, d))
    x_hat = m_hat + 0.3 * rng.standard_normal((n_traj, K, d))
    u = rng.random((n_traj, K))
    res = fo.spec_verify(m, m_hat, x_hat, sigma, u)
    seen = set()
    for n in range(n_traj):
        flags = [bool(fo.verification(m_hat[n, k], m[n, k], 0.3, x_hat[n, k], u[n, k])[1]) for k in range(K)]
        prefix = 0
        while prefix < K and flags[prefix]:
            prefix += 1
        assert res["n_accept"][n] == prefix
        assert list(res["accept"][n].astype(bool)) == flags
        seen.add(prefix)
        if prefix < K:
            np.testing.assert_array_equal(
                res["x_out"][n], fo.reflect(m_hat[n, prefix], m[n, prefix], x_hat[n, prefix]))
        else:
            assert not res["has_reflect"][n]
    assert len(seen) >= 4      # the case mix really covers several prefix lengths


def test_equal_means_always_accept_and_u_zero_accepts():
    m = np.arange(5.0)
    x, ok, l, _ = fo.verification(m, m, 0.1, m + 0.05, 1.0)
    assert ok and l == 0.0 and np.array_equal(x, m + 0.05)
    m_hat, mm, sigma, x_hat = _case(5, 1, sep=50.0)
    assert fo.verification(m_hat, mm, sigma, x_hat, 0.0)[1]
    assert not fo.verification(m_hat, mm, sigma, x_hat, 1e-30)[1]


def test_tie_flag_window():
    m_hat, m, sigma, x_hat = _case(5, 2, sep=1.0)
    l = fo.log_ratio(m_hat, m, sigma, x_hat)
    if l < 0:
        assert fo.verification(m_hat, m, sigma, x_hat, math.exp(l + 5e-5))[3]
        assert fo.verification(m_hat, m, sigma, x_hat, math.exp(l - 5e-5))[3]
        assert not fo.verification(m_hat, m, sigma, x_hat, math.exp(l - 1e-2))[3]


def test_stochasticity_family_shares_the_marginals_on_gaussian_data():
    """Eq. mean_var_gamma: for every stochasticity e the reverse process has the forward marginals.
    For data N(0, s0^2) the exact noise estimate is linear, eps(x) = x sqrt(1 - ab) / v with
    v = ab s0^2 + 1 - ab the marginal variance, so the variance recursion of the discrete chain is closed
    form: starting from v_T it must end near s0^2 for e = 0, 0.5, 1, 2 (first-order discretisation).
    A wrong (1 + e^2)/2 factor or sigma = e sqrt(beta) scaling misses s0^2 by far more."""
    T, s0 = 1000, 0.5
    beta = np.linspace(1e-4, 0.02, T)
    ab = np.cumprod(1 - beta)
    v_marg = ab * s0 ** 2 + 1 - ab
    for e in (0.0, 0.5, 1.0, 2.0):
        cx, ce, sg = fo.sde_coefficients(e, T)
        var = v_marg[-1]
        for i in range(T - 1, -1, -1):
            gain = cx[i] + ce[i] * np.sqrt(1 - ab[i]) / v_marg[i]       # x -> m is linear: m = gain x
            var = gain ** 2 * var + sg[i] ** 2
        assert abs(var - s0 ** 2) < 0.03 * s0 ** 2, (e, var)
    # the two factors matter: dropping (1 + e^2)/2 or the e in sigma breaks it
    cx, ce, sg = fo.sde_coefficients(2.0, T)
    var = v_marg[-1]
    for i in range(T - 1, -1, -1):
        var = (cx[i] + ce[i] / 2.5 * np.sqrt(1 - ab[i]) / v_marg[i]) ** 2 * var + sg[i] ** 2
    assert abs(var - s0 ** 2) > 0.5 * s0 ** 2
    # e = 1 is the DDPM update to first order in beta
    s = fo.ddpm_schedule()
    cx1, ce1, sg1 = fo.sde_coefficients(1.0, T)
    dcx, dce = fo.mean_coefficients(np.arange(T), s)
    assert np.max(np.abs(cx1 - dcx)) < 2e-4 and np.max(np.abs(ce1 / dce - 1)) < 0.011
