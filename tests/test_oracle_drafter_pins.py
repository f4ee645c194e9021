"""Pins of the oracle's drafter and drafting loop (Sec. 3.2; Alg. 1, drafting loop) against facts
that do not depend on the drafter code itself."""
import numpy as np

from oracle import free_oracle as fo
from paper_2511_20390_amd import synth


def _target_as_drafter(cfg, w, depth):
    """Drafter weights under which the drafter IS the first `depth` target blocks: the fusion layer
    passes the embedding through ([I | 0], zero bias) and block / output weights are the target's."""
    D = cfg["hidden"]
    wd = {"fuse_w": np.concatenate([np.eye(D), np.zeros((D, D))], axis=1), "fuse_b": np.zeros(D)}
    for l in range(depth):
        for k in ("ada_w", "ada_b", "qkv_w", "qkv_b", "proj_w", "proj_b", "fc1_w", "fc1_b", "fc2_w", "fc2_b"):
            wd[f"blk{l}.{k}"] = w[f"blk{l}.{k}"]
    for k in ("fin_ada_w", "fin_ada_b", "fin_w", "fin_b"):
        wd[k] = w[k]
    return wd


def _case(name="tiny", B=3, seed=0):
    cfg = synth.dit_config(name)
    w = synth.make_weights(cfg, seed=seed, std=0.05)
    rng = np.random.default_rng(seed + 11)
    x = rng.standard_normal((B, cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]))
    f = rng.standard_normal((B, synth.n_tokens(cfg), cfg["hidden"]))
    t = rng.integers(0, 1000, B)
    y = rng.integers(0, cfg["num_classes"] + 1, B)
    return cfg, w, x, f, t, y


def test_embedding_passthrough_drafter_is_the_depth_limited_target():
    """Shared embedding + pass-through fusion + the target's own block and output weights: the drafter
    must reproduce the target truncated to that many blocks, whatever feature is propagated.
    (A swapped concatenation order, a missing positional table or a wrong conditioning fails this.)"""
    cfg, w, x, f, t, y = _case()
    for depth in (1, 2):
        wd = _target_as_drafter(cfg, w, depth)
        out, feat = fo.drafter_forward(wd, w, dict(cfg, drafter_depth=depth), x, f, t, y)
        ref_out, ref_feat = fo.dit_forward(w, dict(cfg, depth=depth), x, t, y)
        assert np.allclose(out, ref_out, rtol=1e-12, atol=1e-12)
        assert np.allclose(feat, ref_feat, rtol=1e-12, atol=1e-12)


def test_feature_only_fusion_ignores_the_latent_and_batch_rows_are_independent():
    cfg, w, x, f, t, y = _case(seed=1)
    wd = synth.make_drafter_weights(cfg, 1, seed=5, std=0.05)
    D = cfg["hidden"]
    wd = {k: v.astype(np.float64) for k, v in wd.items()}
    wd["fuse_w"][:, :D] = 0.0                                   # only the feature half is connected
    out1, feat1 = fo.drafter_forward(wd, w, cfg, x, f, t, y)
    out2, feat2 = fo.drafter_forward(wd, w, cfg, x[::-1] * 3.0 + 1.0, f, t, y)
    assert np.array_equal(out1, out2) and np.array_equal(feat1, feat2)
    # and a row of the batch does not see the others
    out3, feat3 = fo.drafter_forward(wd, w, cfg, x[1:2], f[1:2], t[1:2], y[1:2])
    assert np.allclose(out3[0], out1[1], rtol=1e-12, atol=1e-13) and np.allclose(feat3[0], feat1[1], rtol=1e-12, atol=1e-13)


def test_fusion_is_affine_in_the_feature():
    """z = W [e | f] + b: the pre-block activation is affine in f, so with identity blocks (zero
    modulation: adaLN-Zero) the predicted feature obeys f(a f1 + (1-a) f2) = a f(f1) + (1-a) f(f2)."""
    cfg, w, x, f, t, y = _case(seed=2)
    wd = {k: v.astype(np.float64) for k, v in synth.make_drafter_weights(cfg, 1, seed=6, std=0.05).items()}
    wd["blk0.ada_w"][:] = 0.0
    wd["blk0.ada_b"][:] = 0.0
    f2 = np.random.default_rng(9).standard_normal(f.shape)
    a = 0.3
    _, fa = fo.drafter_forward(wd, w, cfg, x, f, t, y)
    _, fb = fo.drafter_forward(wd, w, cfg, x, f2, t, y)
    _, fm = fo.drafter_forward(wd, w, cfg, x, a * f + (1 - a) * f2, t, y)
    assert np.allclose(fm, a * fa + (1 - a) * fb, rtol=1e-11, atol=1e-12)
    # and equals the fusion layer written out with plain matrix products
    D = cfg["hidden"]
    e = (fo.patchify(x, cfg["patch"]) @ w["patch_w"].astype(np.float64).T + w["patch_b"]
         + fo.pos_embed_2d(cfg["lat_h"] // cfg["patch"], cfg["lat_w"] // cfg["patch"], D))
    z = e @ wd["fuse_w"][:, :D].T + f @ wd["fuse_w"][:, D:].T + wd["fuse_b"]
    assert np.allclose(fa, z, rtol=1e-11, atol=1e-12)


def _draft_case(cfg_scale, K=4, seed=3):
    cfg = synth.dit_config("tiny")
    w = synth.make_weights(cfg, seed=seed, std=0.05)
    sched = fo.ddpm_schedule()
    di = synth.make_draft_inputs(cfg, K, seed, cfg_scale)
    cx, ce = fo.mean_coefficients(di["t"], sched)
    sigma = sched["sigma_clipped"][di["t"]]
    return cfg, w, sched, di, cx, ce, sigma


def test_draft_chain_equals_its_step_by_step_composition():
    """K drafting steps = K single drafter evaluations chained by hand (Alg. 1, drafting loop), with
    the mean from Eq. (ddpm_update) via eps_to_mean and guidance as in the target."""
    for cfg_scale in (1.0, 4.0):
        cfg, w, sched, di, cx, ce, sigma = _draft_case(cfg_scale)
        wd = synth.make_drafter_weights(cfg, 1, seed=7, std=0.05)
        res = fo.draft_steps(wd, w, cfg, di["x_a"], di["f_a"], di["t"], di["y"], cfg_scale, cx, ce, sigma, di["xi"])
        C = cfg["in_ch"]
        dup = 2 if cfg_scale > 1 else 1
        x = di["x_a"].astype(np.float64)
        f = di["f_a"].astype(np.float64)
        yy = np.array([di["y"], cfg["num_classes"]][:dup])
        for k in range(len(di["t"])):
            assert np.allclose(res["x_states"][k], x, rtol=0, atol=1e-13)
            out, f = fo.drafter_forward(wd, w, cfg, np.stack([x] * dup), f, np.full(dup, di["t"][k]), yy)
            eps = out[0, :C] if dup == 1 else out[1, :C] + cfg_scale * (out[0, :C] - out[1, :C])
            m = fo.eps_to_mean(x, eps, int(di["t"][k]), sched)
            assert np.allclose(res["m_draft"][k], m.reshape(-1), rtol=1e-10, atol=1e-12)
            x = m + sigma[k] * di["xi"][k].reshape(m.shape)
        assert np.allclose(res["x_last"], x, rtol=1e-10, atol=1e-12)
        assert np.allclose(res["f_last"], f, rtol=1e-10, atol=1e-12)


def test_zero_noise_drafts_sit_on_their_means():
    cfg, w, sched, di, cx, ce, sigma = _draft_case(1.0)
    wd = synth.make_drafter_weights(cfg, 1, seed=8, std=0.05)
    res = fo.draft_steps(wd, w, cfg, di["x_a"], di["f_a"], di["t"], di["y"], 1.0, cx, ce, sigma, np.zeros_like(di["xi"]))
    K = len(di["t"])
    for k in range(K - 1):
        assert np.allclose(res["x_states"][k + 1].reshape(-1), res["m_draft"][k], rtol=0, atol=1e-13)
    assert np.allclose(res["x_last"].reshape(-1), res["m_draft"][K - 1], rtol=0, atol=1e-13)


def test_a_drafter_that_reproduces_the_target_is_always_accepted():
    """If p = q the likelihood ratio is 1 (Alg. 2): every draft of the chain passes the verification of
    the same round for any u in (0, 1), and the log ratios vanish up to rounding."""
    for cfg_scale in (1.0, 4.0):
        cfg, w, sched, di, cx, ce, sigma = _draft_case(cfg_scale, K=3, seed=4)
        wd = _target_as_drafter(cfg, w, cfg["depth"])
        dcfg = dict(cfg, drafter_depth=cfg["depth"])
        res = fo.draft_steps(wd, w, dcfg, di["x_a"], di["f_a"], di["t"], di["y"], cfg_scale, cx, ce, sigma, di["xi"])
        u = np.full(3, 0.999999)
        out = fo.spec_round(w, cfg, res["x_states"], res["x_last"], res["m_draft"], di["t"], di["y"], cfg_scale,
                            cx, ce, sigma, u)
        assert int(out["n_accept"][0]) == 3
        assert np.all(np.abs(out["log_ratio"]) < 1e-6)
        assert not bool(out["has_reflect"][0])
