"""The pins of the oracle have to be able to fail: each case below plants one plausible mistake into a function
of the oracle (on the CPU, by monkeypatching a replacement or an edited copy of its source: a dropped term, a
wrong sign, a swapped operand, a missing scale, a wrong index) and requires that at least one of the pin tests named next to it now fails.  A pin that still passes on
every mutant would pin nothing.  The unmodified oracle passes all of them (the pin modules themselves)."""
import inspect
import math

import numpy as np
import pytest

from oracle import free_oracle as fo

import test_oracle_diag_pins as diag_pins
import test_oracle_dit_pins as dit_pins
import test_oracle_drafter_pins as drafter_pins
import test_oracle_loop_pins as loop_pins
import test_oracle_profile_pins as profile_pins
import test_oracle_verify_pins as verify_pins

F64 = np.float64


def _flat(*arrays):
    return [np.asarray(a, F64).ravel() for a in arrays]


# ---- verification (Alg. 2, Eq. qp, Eq. acc_relax) ---------------------------------------------------------------
def _lr_no_midpoint(m_hat, m, sigma, x_hat):            # the -||m^ - m||^2 / 2 term dropped
    m_hat, m, x_hat = _flat(m_hat, m, x_hat)
    return float(np.dot(m - m_hat, x_hat - m_hat) / float(sigma) ** 2)


def _lr_wrong_sign(m_hat, m, sigma, x_hat):             # p / q instead of q / p
    m_hat, m, x_hat = _flat(m_hat, m, x_hat)
    return float(np.dot(m_hat - m, x_hat - 0.5 * (m + m_hat)) / float(sigma) ** 2)


def _lr_sigma_not_squared(m_hat, m, sigma, x_hat):
    m_hat, m, x_hat = _flat(m_hat, m, x_hat)
    return float(np.dot(m - m_hat, x_hat - 0.5 * (m + m_hat)) / float(sigma))


def _reflect_none(m_hat, m, x_hat):                     # translation only: the reflection forgotten
    return np.asarray(m, F64) + (np.asarray(x_hat, F64) - np.asarray(m_hat, F64))


def _reflect_unnormalised(m_hat, m, x_hat):             # e not divided by its norm
    m_hat, m, x_hat = (np.asarray(a, F64) for a in (m_hat, m, x_hat))
    e = (m_hat - m).ravel()
    r = (x_hat - m_hat).ravel()
    return (m.ravel() + r - 2.0 * e * float(np.dot(e, r))).reshape(m.shape)


def _reflect_about_draft_mean(m_hat, m, x_hat):         # result centred on m^ instead of m
    m_hat, m, x_hat = (np.asarray(a, F64) for a in (m_hat, m, x_hat))
    diff = (m_hat - m).ravel()
    e = diff / math.sqrt(float(np.dot(diff, diff)))
    r = (x_hat - m_hat).ravel()
    return (m_hat.ravel() + r - 2.0 * e * float(np.dot(e, r))).reshape(m.shape)


def _reflect_single_subtraction(m_hat, m, x_hat):       # projection (I - e e^T) instead of reflection
    m_hat, m, x_hat = (np.asarray(a, F64) for a in (m_hat, m, x_hat))
    diff = (m_hat - m).ravel()
    e = diff / math.sqrt(float(np.dot(diff, diff)))
    r = (x_hat - m_hat).ravel()
    return (m.ravel() + r - e * float(np.dot(e, r))).reshape(m.shape)


def _verification_accepts_by_ratio_only(m_hat, m, sigma, x_hat, u, lam=1.0):
    """Rejected drafts are resampled as the draft itself (no coupling step at all)."""
    x, ok, l, tie = _ORIGINAL["verification"](m_hat, m, sigma, x_hat, u, lam)
    return (np.asarray(x_hat, F64).copy(), ok, l, tie)


def _verification_relaxes_additively(m_hat, m, sigma, x_hat, u, lam=1.0):
    """Relaxed rule with lam added to the log-ratio instead of scaling it."""
    l = fo.log_ratio(m_hat, m, sigma, x_hat)
    if u <= 0.0:
        return np.asarray(x_hat, F64).copy(), True, l, False
    ok = math.log(u) <= min(0.0, l + (1.0 - float(lam)))
    return (np.asarray(x_hat, F64).copy() if ok else fo.reflect(m_hat, m, x_hat)), ok, l, False


_ORIGINAL = {"verification": fo.verification, "reflect": fo.reflect, "log_ratio": fo.log_ratio}

VERIFY_MUTANTS = [
    ("log_ratio", _lr_no_midpoint, [lambda: verify_pins.test_log_ratio_matches_library_gaussian_logpdf(4),
                                    verify_pins.test_log_ratio_equals_squared_norm_form]),
    ("log_ratio", _lr_wrong_sign, [lambda: verify_pins.test_log_ratio_matches_library_gaussian_logpdf(4),
                                   verify_pins.test_accept_rule_is_the_density_ratio_test]),
    ("log_ratio", _lr_sigma_not_squared, [lambda: verify_pins.test_log_ratio_matches_library_gaussian_logpdf(4),
                                          verify_pins.test_accept_rule_is_the_density_ratio_test]),
    ("reflect", _reflect_none, [verify_pins.test_reflection_1d_is_mirror_about_midpoint,
                                lambda: verify_pins.test_reflection_invariants(4),
                                verify_pins.test_householder_matrix_form]),
    ("reflect", _reflect_unnormalised, [lambda: verify_pins.test_reflection_invariants(4),
                                        verify_pins.test_householder_matrix_form]),
    ("reflect", _reflect_about_draft_mean, [verify_pins.test_reflection_1d_is_mirror_about_midpoint,
                                            lambda: verify_pins.test_reflection_invariants(4)]),
    ("reflect", _reflect_single_subtraction, [lambda: verify_pins.test_reflection_invariants(4),
                                              verify_pins.test_householder_matrix_form]),
    ("verification", _verification_accepts_by_ratio_only, [verify_pins.test_marginal_preserved_1d]),
    ("verification", _verification_relaxes_additively, [verify_pins.test_relaxed_rule_matches_scaled_direction_formula,
                                                        verify_pins.test_lambda_one_is_strict_and_zero_accepts_all]),
]


# ---- the DiT forward (Sec. 3.1 background; adaLN-Zero blocks) ------------------------------------------------------
def _gelu_erf(v):                                        # exact GELU where the tanh form is specified
    from scipy.special import erf
    return 0.5 * v * (1.0 + erf(v / math.sqrt(2.0)))


def _layer_norm_unbiased(v):                             # variance with n - 1
    mu = v.mean(axis=-1, keepdims=True)
    var = ((v - mu) ** 2).sum(axis=-1, keepdims=True) / (v.shape[-1] - 1)
    return (v - mu) / np.sqrt(var + fo.LN_EPS)


def _attention_unscaled(q, k, v):                        # 1 / sqrt(d_h) forgotten
    s = q @ k.T
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    return (p / p.sum(axis=-1, keepdims=True)) @ v


def _attention_softmax_over_queries(q, k, v):            # normalised over the wrong axis
    s = (q @ k.T) / math.sqrt(q.shape[-1])
    s = s - s.max(axis=0, keepdims=True)
    p = np.exp(s)
    return (p / p.sum(axis=0, keepdims=True)) @ v


def _silu_as_sigmoid(v):                                 # the factor v dropped
    return 1.0 / (1.0 + np.exp(-v))


def _timestep_embedding_sin_first(t, dim):               # [sin | cos] instead of [cos | sin]
    half = dim // 2
    w = np.exp(-math.log(fo.MAX_PERIOD) * np.arange(half, dtype=F64) / half)
    ang = np.asarray(t, F64).reshape(-1, 1) * w.reshape(1, -1)
    return np.concatenate([np.sin(ang), np.cos(ang)], axis=1)


def _patchify_channel_last(x, p):                        # patch flattened over (ph, pw, c) instead of (c, ph, pw)
    B, C, H, W = x.shape
    gh, gw = H // p, W // p
    v = x.reshape(B, C, gh, p, gw, p).transpose(0, 2, 4, 3, 5, 1)
    return v.reshape(B, gh * gw, C * p * p)


def _unpatchify_channel_first(tok, p, c_out, gh, gw):    # per-token order (c, ph, pw) instead of (ph, pw, c)
    B = tok.shape[0]
    v = tok.reshape(B, gh, gw, c_out, p, p).transpose(0, 3, 1, 4, 2, 5)
    return v.reshape(B, c_out, gh * p, gw * p)


def _eps_to_mean_plus(x, eps, i, sched):                 # the noise term added instead of removed
    cx, ce = fo.mean_coefficients(i, sched)
    return cx * np.asarray(x, F64) - ce * np.asarray(eps, F64)


def _cfg_combine_swapped(eps_cond, eps_null, scale):     # extrapolates from the conditional towards the null branch
    return eps_cond + scale * (eps_null - eps_cond)


_forward_pin = lambda: dit_pins.test_forward_matches_library_routine_implementation("tiny")

DIT_MUTANTS = [
    ("gelu_tanh", _gelu_erf, [_forward_pin]),
    ("layer_norm", _layer_norm_unbiased, [_forward_pin]),
    ("attention", _attention_unscaled, [_forward_pin]),
    ("attention", _attention_softmax_over_queries, [_forward_pin]),
    ("silu", _silu_as_sigmoid, [_forward_pin]),
    ("timestep_embedding", _timestep_embedding_sin_first, [dit_pins.test_timestep_embedding_properties, _forward_pin]),
    ("patchify", _patchify_channel_last, [dit_pins.test_patchify_unpatchify_layout, _forward_pin]),
    ("unpatchify", _unpatchify_channel_first, [dit_pins.test_patchify_unpatchify_layout, _forward_pin]),
    ("eps_to_mean", _eps_to_mean_plus, [dit_pins.test_eps_to_mean_is_posterior_mean_for_the_true_noise]),
    ("cfg_combine", _cfg_combine_swapped, [dit_pins.test_guidance_special_cases]),
]


# ---- per-element variance: mistakes planted into the whitened rule
def _reflect_diag_unwhitened_direction(m_hat, m, sigma_vec, x_hat):
    """The reflection direction taken in the original coordinates (the variances ignored)."""
    return _ORIGINAL["reflect"](m_hat, m, x_hat)


def _log_ratio_diag_mean_variance(m_hat, m, sigma_vec, x_hat):
    """One pooled variance instead of the per-element ones."""
    s = np.asarray(sigma_vec, F64).ravel()
    return _ORIGINAL["log_ratio"](m_hat, m, math.sqrt(float(np.mean(s * s))), x_hat)


DIAG_MUTANTS = [
    ("reflect_diag", _reflect_diag_unwhitened_direction,
     [diag_pins.test_diag_is_the_scalar_rule_on_whitened_inputs, diag_pins.test_diag_reflection_preserves_the_whitened_distances]),
    ("log_ratio_diag", _log_ratio_diag_mean_variance,
     [diag_pins.test_diag_log_ratio_matches_library_gaussian_logpdf, diag_pins.test_diag_is_the_scalar_rule_on_whitened_inputs]),
]


@pytest.mark.parametrize("name,mutant,pins", DIAG_MUTANTS, ids=[m.__name__.lstrip("_") for _, m, _ in DIAG_MUTANTS])
def test_planted_mistake_in_the_per_element_rule_is_caught(monkeypatch, name, mutant, pins):
    assert not _some_pin_fails(pins), "the pins must pass on the oracle as it stands"
    monkeypatch.setattr(fo, name, mutant)
    assert _some_pin_fails(pins), f"no pin noticed the mistake planted into {name}"


# ---- the loop of Alg. 1 and the relaxation profile (Sec. 3.4): mistakes planted into the source text ---------------
def _edited(func, old, new):
    """The oracle's own function with one piece of its source replaced, compiled in the oracle's namespace."""
    src = inspect.getsource(func)
    assert src.count(old) == 1, (func.__name__, old)
    scope = dict(vars(fo))
    exec(compile(src.replace(old, new), f"<{func.__name__} with a planted mistake>", "exec"), scope)
    return scope[func.__name__]


def _cumulative_maximum(v):                              # a monotone curve, but not the least-squares one
    v = np.asarray(v, F64)
    return np.maximum.accumulate(np.where(np.isnan(v), -np.inf, v))


SOURCE_MUTANTS = [
    # every draft of a round drawn with the first noise vector of the round
    ("same_noise_for_all_drafts", "speculative_loop",
     lambda: _edited(fo.speculative_loop, "states.append(m_hat[-1] + sigma[i + j] * xi[i + j].reshape(x.shape))",
                     "states.append(m_hat[-1] + sigma[i + j] * xi[i].reshape(x.shape))"),
     [loop_pins.test_perfect_drafter_is_sequential_sampling_and_all_drafts_pass]),
    # every draft checked against the target mean of the first packed state
    ("drafts_checked_against_first_mean", "speculative_loop",
     lambda: _edited(fo.speculative_loop, "np.asarray(means[j], F64).reshape(-1), sigma[i + j],",
                     "np.asarray(means[0], F64).reshape(-1), sigma[i + j],"),
     [loop_pins.test_perfect_drafter_is_sequential_sampling_and_all_drafts_pass]),
    # a rejected draft replaced by the draft itself: the reflected sample thrown away
    ("rejection_keeps_the_draft", "speculative_loop",
     lambda: _edited(fo.speculative_loop, "x = xr.reshape(x.shape)", "x = states[j + 1]"),
     [loop_pins.test_loop_preserves_the_target_distribution_on_a_linear_gaussian_chain]),
    # after a full round the sampler keeps the last but one draft
    ("full_round_keeps_the_wrong_state", "speculative_loop",
     lambda: _edited(fo.speculative_loop, "x, feat, i = states[K], feats[K - 1], i + K",
                     "x, feat, i = states[K - 1], feats[K - 1], i + K"),
     [loop_pins.test_perfect_drafter_is_sequential_sampling_and_all_drafts_pass,
      loop_pins.test_loop_preserves_the_target_distribution_on_a_linear_gaussian_chain]),
    # the fusion layer fed [feature | embedding] instead of [embedding | feature]
    ("fusion_inputs_swapped", "drafter_forward",
     lambda: _edited(fo.drafter_forward, "np.concatenate([emb[r], np.asarray(f_prev, F64)[r]], axis=1)",
                     "np.concatenate([np.asarray(f_prev, F64)[r], emb[r]], axis=1)"),
     [drafter_pins.test_embedding_passthrough_drafter_is_the_depth_limited_target,
      drafter_pins.test_feature_only_fusion_ignores_the_latent_and_batch_rows_are_independent]),
    # the propagated feature taken before the drafter's blocks instead of after them
    ("feature_taken_before_the_blocks", "drafter_forward",
     lambda: _edited(fo.drafter_forward, "        for l in range(ddepth):\n            z = dit_block(z, sc[r], wd, l, heads)\n        feat[r] = z\n",
                     "        feat[r] = z\n        for l in range(ddepth):\n            z = dit_block(z, sc[r], wd, l, heads)\n"),
     [drafter_pins.test_embedding_passthrough_drafter_is_the_depth_limited_target,
      drafter_pins.test_draft_chain_equals_its_step_by_step_composition,
      drafter_pins.test_a_drafter_that_reproduces_the_target_is_always_accepted]),
    # every drafting step reuses the feature of the reference state
    ("feature_not_propagated", "draft_steps",
     lambda: _edited(fo.draft_steps, "out, f = drafter_forward(", "out, _ = drafter_forward("),
     [drafter_pins.test_draft_chain_equals_its_step_by_step_composition]),
    # draft k + 1 drawn around the state instead of around the draft mean
    ("next_draft_around_the_state", "draft_steps",
     lambda: _edited(fo.draft_steps, "xs.append(m + float(sigma[k])", "xs.append(xk + float(sigma[k])"),
     [drafter_pins.test_zero_noise_drafts_sit_on_their_means,
      drafter_pins.test_draft_chain_equals_its_step_by_step_composition]),
    ("monotone_fit_is_a_running_maximum", "monotone_fit", lambda: _cumulative_maximum,
     [profile_pins.test_monotone_fit_against_brute_force_and_library]),
    ("profile_not_inverted", "relaxation_profile_from_deltas",
     lambda: _edited(fo.relaxation_profile_from_deltas, "return g[0] / g", "return g / g[-1]"),
     [profile_pins.test_profile_is_the_rescaled_inverse_of_the_fit]),
    ("frozen_drafts_advance_without_noise", "frozen_draft_steps",
     lambda: _edited(fo.frozen_draft_steps, "xs.append(m + float(sigma[k]) * np.asarray(xi, F64)[k].reshape(x.shape))",
                     "xs.append(m)"),
     [profile_pins.test_frozen_drafts_closed_form]),
    # the recorded deviation left in units of the mean: not divided by the coefficient of the noise estimate
    ("deviation_not_divided_by_coef_eps", "self_speculative_run",
     lambda: _edited(fo.self_speculative_run, " / abs(float(coef_eps[i]))", ""),
     [profile_pins.test_recorded_deviation_is_the_distance_between_the_two_noise_estimates]),
]


@pytest.mark.parametrize("label,name,make,pins", SOURCE_MUTANTS, ids=[m[0] for m in SOURCE_MUTANTS])
def test_planted_mistake_in_the_loop_or_profile_is_caught(monkeypatch, label, name, make, pins):
    assert not _some_pin_fails(pins), "the pins must pass on the oracle as it stands"
    monkeypatch.setattr(fo, name, make())
    assert _some_pin_fails(pins), f"no pin noticed: {label}"


def _some_pin_fails(pins):
    for pin in pins:
        try:
            pin()
        except AssertionError:
            return True
    return False


@pytest.mark.parametrize("name,mutant,pins", VERIFY_MUTANTS + DIT_MUTANTS,
                         ids=[m.__name__.lstrip("_") for _, m, _ in VERIFY_MUTANTS + DIT_MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant, pins):
    assert not _some_pin_fails(pins), "the pins must pass on the oracle as it stands"
    monkeypatch.setattr(fo, name, mutant)
    assert _some_pin_fails(pins), f"no pin noticed the mistake planted into {name}"
