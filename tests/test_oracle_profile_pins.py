"""Pins of the relaxation-profile builder (Sec. 3.4): frozen-target drafting, the self-speculative run,
the monotone fit and its inversion."""
import itertools

import numpy as np

from oracle import free_oracle as fo
from paper_2511_20390_amd import synth


def test_monotone_fit_against_brute_force_and_library():
    rng = np.random.default_rng(0)
    # brute force on a tiny grid: the best non-decreasing sequence with values from the candidate set
    v = np.array([0.3, 0.1, 0.4, 0.35, 0.9])
    fit = fo.monotone_fit(v)
    cands = sorted(set(np.round(np.concatenate([v, [(0.3 + 0.1) / 2, (0.4 + 0.35) / 2]]), 6)))
    best, best_cost = None, 1e9
    for combo in itertools.combinations_with_replacement(cands, len(v)):
        cost = float(np.sum((np.array(combo) - v) ** 2))
        if cost < best_cost:
            best, best_cost = np.array(combo), cost
    assert np.allclose(fit, best, atol=1e-6)
    from sklearn.isotonic import IsotonicRegression
    for n in (7, 50, 200):
        v = np.cumsum(rng.standard_normal(n)) * 0.1 + np.linspace(0, 2, n)
        ref = IsotonicRegression(increasing=True).fit_transform(np.arange(n), v)
        assert np.allclose(fo.monotone_fit(v), ref, rtol=1e-10, atol=1e-12)
    # missing entries carry no weight
    v = np.array([np.nan, 1.0, np.nan, 0.5, 2.0, np.nan])
    assert np.allclose(fo.monotone_fit(v), [0.75, 0.75, 0.75, 0.75, 2.0, 2.0])


def test_profile_is_the_rescaled_inverse_of_the_fit():
    g = np.array([1.0, 2.0, 2.0, 4.0, 8.0])
    lam = fo.relaxation_profile_from_deltas(g)
    assert np.allclose(lam, [1.0, 0.5, 0.5, 0.25, 0.125])
    rng = np.random.default_rng(1)
    noisy = np.linspace(1, 5, 101) + 0.3 * rng.standard_normal(101)
    for window in (1, 9):
        lam = fo.relaxation_profile_from_deltas(noisy, window)
        assert lam[0] == 1.0 and np.all(lam > 0) and np.all(lam <= 1.0) and np.all(np.diff(lam) <= 1e-15)
    # smoothing keeps the ends and the monotonicity and removes the plateaus' corners
    lam9 = fo.relaxation_profile_from_deltas(noisy, 9)
    assert abs(lam9[-1] - fo.relaxation_profile_from_deltas(noisy, 1)[-1]) < 0.05


def test_frozen_drafts_closed_form():
    """With constant coefficients the recurrence x_{k+1} = a x_k + b e + s xi_k has the closed form
    a^k x_0 + b e (1 - a^k) / (1 - a) + s sum_j a^{k-1-j} xi_j."""
    rng = np.random.default_rng(2)
    K, d = 5, 12
    a, b, s = 1.02, -0.03, 0.2
    x0, e, xi = rng.standard_normal((1, 3, 4)), rng.standard_normal(d), rng.standard_normal((K, d))
    res = fo.frozen_draft_steps(x0, e, np.full(K, a), np.full(K, b), np.full(K, s), xi)
    for k in range(K + 1):
        ref = a ** k * x0.ravel() + b * e * (1 - a ** k) / (1 - a) + s * sum(a ** (k - 1 - j) * xi[j] for j in range(k))
        got = res["x_last"].ravel() if k == K else res["x_states"][k].ravel()
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-13)
    for k in range(K):
        assert np.allclose(res["m_draft"][k], a * res["x_states"][k].ravel() + b * e, rtol=1e-13)


def _run_case(w, cfg, cfg_scale=4.0, S=10, L=4, seed=3):
    sched = fo.ddpm_schedule()
    tmap = np.linspace(960, 30, S).round().astype(np.int32)
    cx, ce = fo.mean_coefficients(tmap, sched)
    sigma = sched["sigma_clipped"][tmap].copy()
    sigma[-1] = 0.0
    rng = np.random.default_rng(seed)
    d = synth.latent_dim(cfg)
    x0 = rng.standard_normal((cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]))
    return dict(x0=x0, y=2, cfg_scale=cfg_scale, tmap=tmap, coef_x=cx, coef_eps=ce, sigma=sigma, n_spec=S - 1, L=L,
                xi=rng.standard_normal((S, d)), u=rng.random(S))


def test_self_speculation_with_a_state_independent_noise_estimate_never_rejects():
    """If the network's noise estimate does not depend on the state or the timestep (zero output matrix: the
    estimate is the output bias), reusing it is exact: every deviation is 0 and every draft passes."""
    cfg = synth.dit_config("tiny")
    w = synth.make_weights(cfg, seed=0, std=0.05)
    w["fin_w"] = np.zeros_like(w["fin_w"])
    a = _run_case(w, cfg)
    x, st, delta, acc = fo.self_speculative_run(w, cfg, **a)
    checked = ~np.isnan(delta)
    assert checked.sum() == st["drafter_steps"] == st["accepted"] > 0
    assert np.all(delta[checked] < 1e-9) and np.all(acc[checked] == 1)
    assert np.isnan(delta[0]) and np.isnan(delta[-1]) and acc[0] == -1        # plain target steps are not checked


def test_self_speculation_records_deviation_and_outcome_per_checked_step():
    cfg = synth.dit_config("tiny")
    w = synth.make_weights(cfg, seed=1, std=0.3)          # a state-dependent network: deviations are non-zero
    a = _run_case(w, cfg, cfg_scale=1.0, S=12, L=3)
    x, st, delta, acc = fo.self_speculative_run(w, cfg, **a)
    checked = ~np.isnan(delta)
    assert np.array_equal(checked, acc >= 0)
    assert np.all(delta[checked] > 0)
    # every round checks n_accept + 1 drafts (n_accept when all passed)
    assert checked.sum() >= st["accepted"] and checked.sum() <= st["accepted"] + st["rounds"]
    lam = fo.relaxation_profile_from_deltas(delta, 3)
    assert lam.shape == (12,) and lam[0] == 1.0 and np.all(np.diff(lam) <= 1e-15)


def test_recorded_deviation_is_the_distance_between_the_two_noise_estimates():
    """Magnitude of eps_delta (Sec. 3.4: the deviation between the reused noise estimate and the target's own
    at the drafted state).  With one draft per round and u = 0 (every draft passes whatever the ratio) the chain
    is a plain recurrence that can be written down without the loop: e_i = eps_guided(x_i, t_i),
    x_1 = c_x x_0 + c_e e_0 + s xi_0, then x_{i+1} = c_x x_i + c_e e_{i-1} + s xi_i, and the deviation recorded
    at step i is || e_{i-1} - e_i ||_2, computed here from dit_forward on the visited states."""
    cfg = synth.dit_config("tiny")
    w = synth.make_weights(cfg, seed=4, std=0.3)
    for cfg_scale in (4.0, 1.0):
        a = _run_case(w, cfg, cfg_scale=cfg_scale, S=6, L=1, seed=8)
        a["u"] = np.zeros_like(a["u"])
        x, st, delta, acc = fo.self_speculative_run(w, cfg, **a)
        C, S = cfg["in_ch"], len(a["tmap"])

        def guided(xs, t):
            if cfg_scale > 1.0:
                out, _ = fo.dit_forward(w, cfg, np.stack([xs, xs]), np.array([t, t]), np.array([a["y"], cfg["num_classes"]]))
                return fo.cfg_combine(out[:1, :C], out[1:, :C], cfg_scale)[0]
            out, _ = fo.dit_forward(w, cfg, xs[None], np.array([t]), np.array([a["y"]]))
            return out[0, :C]

        xs = [np.asarray(a["x0"], np.float64)]
        es = []
        for i in range(S):
            es.append(guided(xs[i], a["tmap"][i]))
            used = es[i] if (i == 0 or i >= a["n_spec"]) else es[i - 1]      # plain target step / frozen draft
            xs.append(a["coef_x"][i] * xs[i] + a["coef_eps"][i] * used + a["sigma"][i] * a["xi"][i].reshape(xs[i].shape))
        assert st["rounds"] == S - 2 and st["accepted"] == S - 2
        for i in range(1, S - 1):
            want = np.linalg.norm((es[i - 1] - es[i]).ravel())
            assert want > 1e-6 and abs(delta[i] - want) <= 1e-9 * want, (i, delta[i], want)
        assert np.isnan(delta[0]) and np.isnan(delta[S - 1])
        assert np.allclose(x, xs[S], rtol=1e-10, atol=1e-12)
