"""Pins of the verification with one variance per element (App. C: fixed-variance schedules richer than one
scalar per step; Sec. 3.3: draft and target must share the covariance): Alg. 2 in whitened coordinates."""
import math

import numpy as np
from scipy import stats
from scipy.special import ndtr

from oracle import free_oracle as fo


def _case(rng, d, sep=1.2):
    s = np.exp(0.5 * rng.standard_normal(d)) * 0.3
    m = rng.standard_normal(d)
    m_hat = m + sep * s * rng.standard_normal(d) / math.sqrt(d)
    x_hat = m_hat + s * rng.standard_normal(d)
    return m_hat, m, s, x_hat


def test_diag_log_ratio_matches_library_gaussian_logpdf():
    rng = np.random.default_rng(0)
    for d in (1, 3, 64):
        m_hat, m, s, x_hat = _case(rng, d)
        ref = (stats.multivariate_normal(m, np.diag(s * s)).logpdf(x_hat)
               - stats.multivariate_normal(m_hat, np.diag(s * s)).logpdf(x_hat))
        assert abs(fo.log_ratio_diag(m_hat, m, s, x_hat) - ref) < 1e-9 * max(1.0, abs(ref))


def test_diag_with_equal_variances_is_the_scalar_rule():
    rng = np.random.default_rng(1)
    for d in (2, 17):
        for _ in range(50):
            m_hat, m, _, x_hat = _case(rng, d)
            sigma, u, lam = 0.37, rng.random(), rng.choice([1.0, 0.6])
            a = fo.verification(m_hat, m, sigma, x_hat, u, lam)
            b = fo.verification_diag(m_hat, m, np.full(d, sigma), x_hat, u, lam)
            assert a[1] == b[1] and abs(a[2] - b[2]) < 1e-10 * max(1.0, abs(a[2]))
            assert np.allclose(a[0], b[0], rtol=1e-12, atol=1e-13)


def test_diag_is_the_scalar_rule_on_whitened_inputs():
    """Dividing every coordinate by its standard deviation turns the problem into the unit-variance one."""
    rng = np.random.default_rng(2)
    seen = set()
    for _ in range(200):
        m_hat, m, s, x_hat = _case(rng, 6)
        u = rng.random()
        x, ok, l, _ = fo.verification_diag(m_hat, m, s, x_hat, u)
        xw, okw, lw, _ = fo.verification(m_hat / s, m / s, 1.0, x_hat / s, u)
        assert ok == okw and abs(l - lw) < 1e-10 * max(1.0, abs(lw))
        assert np.allclose(x, xw * s, rtol=1e-12, atol=1e-13)
        seen.add(ok)
    assert seen == {True, False}


def test_diag_reflection_preserves_the_whitened_distances():
    rng = np.random.default_rng(3)
    m_hat, m, s, x_hat = _case(rng, 9)
    x = fo.reflect_diag(m_hat, m, s, x_hat)
    assert abs(np.linalg.norm((x - m) / s) - np.linalg.norm((x_hat - m_hat) / s)) < 1e-12
    assert abs(np.linalg.norm((x - m_hat) / s) - np.linalg.norm((x_hat - m) / s)) < 1e-12
    # the same reflection twice, roles swapped, returns the draft
    back = fo.reflect_diag(m, m_hat, s, x)
    assert np.allclose(back, x_hat, rtol=1e-12, atol=1e-13)


def test_diag_output_has_the_target_marginal_and_the_closed_form_rate():
    """Samples of N(m^, diag(s^2)) pushed through the rule are distributed as N(m, diag(s^2)) (App. B), and the
    acceptance rate is 2 Phi(-D/2) with D the distance of the means in whitened coordinates (App. D)."""
    rng = np.random.default_rng(4)
    d, n = 3, 60_000
    s = np.array([0.1, 0.45, 1.3])
    m = rng.standard_normal(d)
    m_hat = m + np.array([0.9, -0.7, 0.5]) * s
    xs = m_hat + s * rng.standard_normal((n, d))
    us = rng.random(n)
    out = np.empty((n, d))
    acc = 0
    for i in range(n):
        out[i], ok, _, _ = fo.verification_diag(m_hat, m, s, xs[i], us[i])
        acc += ok
    z = (out - m) / s
    for j in range(d):
        assert stats.kstest(z[:, j], "norm").pvalue > 1e-3
    assert stats.kstest((z ** 2).sum(axis=1), "chi2", args=(d,)).pvalue > 1e-3
    assert stats.kstest(((xs - m) / s)[:, 0], "norm").pvalue < 1e-6          # the proposal fails: the test has power
    dist = np.linalg.norm((m_hat - m) / s)
    p = 2 * ndtr(-dist / 2)
    assert abs(acc / n - p) < 4.5 * math.sqrt(p * (1 - p) / n)


def test_spec_verify_diag_prefix_and_scalar_agreement():
    rng = np.random.default_rng(5)
    n_traj, K, d = 12, 4, 10
    sigma = rng.uniform(0.05, 0.3, (n_traj, K))
    m = rng.standard_normal((n_traj, K, d))
    m_hat = m + 0.5 * sigma[..., None] * rng.standard_normal((n_traj, K, d))
    x_hat = m_hat + sigma[..., None] * rng.standard_normal((n_traj, K, d))
    u = rng.random((n_traj, K))
    a = fo.spec_verify(m, m_hat, x_hat, sigma, u)
    b = fo.spec_verify_diag(m, m_hat, x_hat, np.repeat(sigma[..., None], d, axis=2), u)
    assert np.array_equal(a["accept"], b["accept"]) and np.array_equal(a["n_accept"], b["n_accept"])
    assert np.allclose(a["log_ratio"], b["log_ratio"], rtol=1e-10) and np.allclose(a["x_out"], b["x_out"], rtol=1e-11)
    for n in range(n_traj):                              # n_accept is the length of the accepted prefix
        pre = 0
        while pre < K and b["accept"][n, pre]:
            pre += 1
        assert b["n_accept"][n] == pre
