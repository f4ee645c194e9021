"""Pins of the oracle's full sampler (Alg. 1): a perfect drafter reproduces plain sequential sampling,
the loop preserves the target's distribution on a model with a known answer, and the bookkeeping
(target calls, rounds, accepted drafts) adds up."""
import math

import numpy as np

from oracle import free_oracle as fo
from paper_2511_20390_amd import synth


def _linear_models(a, b, S):
    """Scalar toy chain: target transition N(a x, sigma^2), drafter N(b x, sigma^2); the feature is unused."""
    def target_means(states, i0):
        return [a * np.asarray(s) for s in states], [None if False else 0.0 for _ in states]

    def draft_mean(x, f, i):
        return b * np.asarray(x), 0.0
    return target_means, draft_mean


def test_perfect_drafter_is_sequential_sampling_and_all_drafts_pass():
    rng = np.random.default_rng(0)
    S, L, d = 23, 5, 3
    sigma = np.concatenate([rng.uniform(0.1, 0.5, S - 1), [0.0]])
    xi, u = rng.standard_normal((S, d)), rng.random(S)
    x0 = rng.standard_normal(d)
    tm, dm = _linear_models(0.9, 0.9, S)
    x, st = fo.speculative_loop(x0, S, S - 1, L, sigma, xi, u, None, tm, dm)
    ref = x0.copy()
    for i in range(S):
        ref = 0.9 * ref + sigma[i] * xi[i]
    assert np.allclose(x, ref, rtol=1e-13, atol=1e-13)
    # step 0 is a plain target step, then ceil(21 / 5) rounds, then the noise-free last step
    assert st["rounds"] == math.ceil((S - 2) / L) and st["target_calls"] == st["rounds"] + 2
    assert st["accepted"] == S - 2 == st["drafter_steps"] and st["n_accept"] == [5, 5, 5, 5, 1]


def test_every_step_is_taken_exactly_once_whatever_is_rejected():
    """With a poor drafter rejections occur; the states visited must still number S, each round must
    advance by n_accept + 1 (or K when all pass), and the counters must add up."""
    rng = np.random.default_rng(1)
    S, L = 40, 4
    sigma = np.concatenate([np.full(S - 1, 0.3), [0.0]])
    tm_calls = []
    a, b = 0.95, 0.6

    def tm(states, i0):
        tm_calls.append((i0, len(states)))
        return [a * np.asarray(s) for s in states], [0.0] * len(states)

    def dm(x, f, i):
        return b * np.asarray(x), 0.0
    x, st = fo.speculative_loop(np.array([2.0]), S, S - 1, L, sigma, rng.standard_normal((S, 1)), rng.random(S), None, tm, dm)
    assert st["target_calls"] == len(tm_calls) and 0 < st["accepted"] < st["drafter_steps"]
    # call 0 is the plain step at i = 0, then the rounds, then the plain noise-free step at i = S - 1
    assert tm_calls[0] == (0, 1) and tm_calls[-1] == (S - 1, 1) and len(tm_calls) == st["rounds"] + 2
    pos = 1
    for (i0, k), n in zip(tm_calls[1:-1], st["n_accept"]):
        assert i0 == pos and k == min(L, S - 1 - pos) and 0 <= n <= k
        pos += k if n == k else n + 1
    assert pos == S - 1


def test_loop_preserves_the_target_distribution_on_a_linear_gaussian_chain():
    """Target x_{i+1} ~ N(a x_i, s^2): x_S | x_0 is Gaussian with mean a^S x_0 and variance
    s^2 (1 - a^{2S}) / (1 - a^2), whatever the drafter proposes (App. B: the coupling is unbiased).
    A wrong acceptance rule, reflection, advance or feature hand-over shifts these moments."""
    a, b, s, S, L, n = 0.8, 0.5, 0.7, 12, 4, 20000
    rng = np.random.default_rng(2)
    tm, dm = _linear_models(a, b, S)
    sigma = np.full(S, s)
    out = np.empty(n)
    acc = 0
    for r in range(n):
        x, st = fo.speculative_loop(np.array([1.5]), S, S, L, sigma, rng.standard_normal((S, 1)), rng.random(S), None, tm, dm)
        out[r] = x[0]
        acc += st["accepted"]
    mean, var = a ** S * 1.5, s * s * (1 - a ** (2 * S)) / (1 - a * a)
    assert abs(out.mean() - mean) < 5 * math.sqrt(var / n)
    assert abs(out.var() - var) < 5 * var * math.sqrt(2.0 / n)
    # fourth moment of a Gaussian: kurtosis 3
    k = ((out - out.mean()) ** 4).mean() / out.var() ** 2
    assert abs(k - 3.0) < 0.15
    assert 0 < acc < n * (S - 1)                      # drafts were both accepted and rejected


def test_free_sample_with_a_target_copy_drafter_equals_the_sequential_dit_sampler():
    """The DiT-backed sampler with a drafter that reproduces the target: the result must be the plain
    ancestral chain x_{i+1} = m(x_i) + sigma_i xi_i run step by step with dit_forward (guidance on)."""
    cfg = synth.dit_config("tiny")
    w = synth.make_weights(cfg, seed=0, std=0.05)
    D = cfg["hidden"]
    wd = {"fuse_w": np.concatenate([np.eye(D), np.zeros((D, D))], axis=1), "fuse_b": np.zeros(D)}
    for l in range(cfg["depth"]):
        for k in ("ada_w", "ada_b", "qkv_w", "qkv_b", "proj_w", "proj_b", "fc1_w", "fc1_b", "fc2_w", "fc2_b"):
            wd[f"blk{l}.{k}"] = w[f"blk{l}.{k}"]
    for k in ("fin_ada_w", "fin_ada_b", "fin_w", "fin_b"):
        wd[k] = w[k]
    dcfg = dict(cfg, drafter_depth=cfg["depth"])
    sched = fo.ddpm_schedule()
    S, L, scale, y = 7, 3, 4.0, 3
    tmap = np.arange(S - 1, -1, -1) * 100 + 50                      # 650, 550, .., 50
    cx, ce = fo.mean_coefficients(tmap, sched)
    sigma = sched["sigma_clipped"][tmap].copy()
    sigma[-1] = 0.0
    rng = np.random.default_rng(3)
    d = synth.latent_dim(cfg)
    x0 = rng.standard_normal((cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]))
    xi, u = rng.standard_normal((S, d)), rng.random(S)
    x, st = fo.free_sample(wd, w, dcfg, x0, y, scale, tmap, cx, ce, sigma, S - 1, L, xi, u)
    ref = x0.copy()
    for i in range(S):
        m = fo.round_means(w, cfg, ref[None], tmap[i:i + 1], y, scale, cx[i:i + 1], ce[i:i + 1])[0]
        ref = m + sigma[i] * xi[i].reshape(m.shape)
    assert np.allclose(x, ref, rtol=1e-9, atol=1e-10)
    assert st["accepted"] == st["drafter_steps"] == S - 2 and st["n_accept"] == [3, 2]
