"""GPU parity of the drafter forward and of the drafting loop (Sec. 3.2; Alg. 1, drafting loop)
against the oracle, through the C ABI, and the chain drafting -> verification round."""
import numpy as np
import pytest

from oracle import free_oracle as fo
from paper_2511_20390_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

GAIN = 4.0      # output gain of the test drafter in the sampler test: drafts are accepted and rejected


def _models(name, mode, depth, seed=0, out_gain=1.0):
    from paper_2511_20390_amd import binding
    cfg = synth.dit_config(name)
    w = pu.weights_for(cfg, mode, seed=seed)
    wd = synth.make_drafter_weights(cfg, depth, seed=seed + 1, bf16_values=(mode == "bf16"))
    if out_gain != 1.0:       # a louder output projection: drafts far enough from the target to be rejected
        wd["fin_w"] = synth.bf16_round(wd["fin_w"] * np.float32(out_gain)) if mode == "bf16" else wd["fin_w"] * np.float32(out_gain)
    target = binding.FreeDit(cfg, w, mode)
    drafter = binding.FreeDrafter(target, wd, depth)
    return cfg, w, wd, target, drafter


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
@pytest.mark.parametrize("name,B,depth", [("tiny", 3, 1), ("small", 2, 1), ("small", 5, 2)])
def test_drafter_forward_parity(name, B, depth, mode):
    cfg, w, wd, target, drafter = _models(name, mode, depth)
    rng = np.random.default_rng(B + depth)
    x = rng.standard_normal((B, cfg["in_ch"], cfg["lat_h"], cfg["lat_w"])).astype(np.float32)
    f = rng.standard_normal((B, synth.n_tokens(cfg), cfg["hidden"])).astype(np.float32)
    t = rng.integers(0, 1000, B).astype(np.int32)
    y = rng.integers(0, cfg["num_classes"] + 1, B).astype(np.int32)
    eps, feat = drafter.drafter_forward(pu.to_dev(x), pu.to_dev(f), pu.to_dev(t), pu.to_dev(y))
    ref_eps, ref_feat = fo.drafter_forward(wd, w, dict(cfg, drafter_depth=depth), x, f, t, y)
    e1, e2 = pu.rel_l2(eps.cpu().numpy(), ref_eps), pu.rel_l2(feat.cpu().numpy(), ref_feat)
    print(f"{name}/{mode} B={B} depth={depth}: eps rel-L2 {e1:.3e}, feature rel-L2 {e2:.3e}")
    assert e1 <= pu.DIT_REL_L2[mode] and e2 <= pu.DIT_REL_L2[mode]
    drafter.close()
    target.close()


def _draft_inputs(cfg, K, seed, cfg_scale):
    sched = fo.ddpm_schedule()
    di = synth.make_draft_inputs(cfg, K, seed, cfg_scale)
    cx, ce = fo.mean_coefficients(di["t"], sched)
    sigma = sched["sigma_clipped"][di["t"]]
    return sched, di, cx, ce, sigma


def _run_draft(drafter, di, cfg_scale, cx, ce, sigma, want_feat=True):
    return drafter.draft_round(pu.to_dev(di["x_a"]), pu.to_dev(di["f_a"]), pu.to_dev(di["t"]), di["y"], cfg_scale,
                               pu.to_dev(cx.astype(np.float32)), pu.to_dev(ce.astype(np.float32)),
                               pu.to_dev(sigma.astype(np.float32)), pu.to_dev(di["xi"]), want_feat=want_feat)


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
# ("tiny", 9, 4.0, 1): 18 conditioning rows, more than one modulation pass holds - the per-step conditioning path
@pytest.mark.parametrize("name,K,cfg_scale,depth", [("tiny", 5, 4.0, 1), ("tiny", 1, 1.0, 1), ("small", 6, 4.0, 1),
                                                    ("small", 3, 1.0, 2), ("tiny", 9, 4.0, 1)])
def test_draft_round_parity(name, K, cfg_scale, depth, mode):
    """The whole autoregressive chain: errors compound over the K steps, so the last draft is the
    strictest check.  The oracle is fed the float32-rounded coefficients the library receives."""
    cfg, w, wd, target, drafter = _models(name, mode, depth, seed=2)
    sched, di, cx, ce, sigma = _draft_inputs(cfg, K, 5, cfg_scale)
    out = _run_draft(drafter, di, cfg_scale, cx, ce, sigma)
    ref = fo.draft_steps(wd, w, dict(cfg, drafter_depth=depth), di["x_a"], di["f_a"], di["t"], di["y"], cfg_scale,
                         cx.astype(np.float32), ce.astype(np.float32), sigma.astype(np.float32), di["xi"])
    d = synth.latent_dim(cfg)
    # the tolerance of the forward applies to the noise estimate; recover it from the mean: eps = (m - cx x) / ce
    xs_g = out["x_states"].cpu().numpy().reshape(K, d).astype(np.float64)
    m_g = out["m_draft"].cpu().numpy().astype(np.float64)
    for k in range(K):
        cxk, cek = np.float64(np.float32(cx[k])), np.float64(np.float32(ce[k]))
        eps_g = (m_g[k] - cxk * xs_g[k]) / cek
        eps_r = (ref["m_draft"][k] - cxk * ref["x_states"][k].reshape(-1)) / cek
        err = pu.rel_l2(eps_g, eps_r)
        print(f"{name}/{mode} K={K} step {k}: eps rel-L2 {err:.3e}")
        assert err <= pu.DIT_REL_L2[mode]               # the forward's tolerance, at every step of the chain
    tol = 1e-4 if mode == "fp32" else 2e-2
    assert pu.rel_l2(out["x_last"].cpu().numpy(), ref["x_last"].reshape(-1)) <= tol
    e_f = pu.rel_l2(out["f_last"].cpu().numpy(), ref["f_last"])
    print(f"{name}/{mode} K={K}: last feature rel-L2 {e_f:.3e}")
    assert e_f <= tol
    assert np.array_equal(out["x_states"][0].cpu().numpy(), di["x_a"])
    drafter.close()
    target.close()


def test_draft_then_verify_round_chain():
    """Drafting loop -> verification round on the GPU, against the same chain in the oracle: the outputs
    of draft_round are exactly the inputs of spec_round (Alg. 1)."""
    import torch
    mode, K, cfg_scale = "fp32", 4, 4.0
    cfg, w, wd, target, drafter = _models("tiny", mode, 1, seed=3)
    sched, di, cx, ce, sigma = _draft_inputs(cfg, K, 9, cfg_scale)
    # the target's own top-block feature of the previous state starts the chain
    rng = np.random.default_rng(4)
    x_prev = rng.standard_normal((1,) + di["x_a"].shape).astype(np.float32)
    tt = np.array([di["t"][0] + 1] * 2, np.int32) if di["t"][0] + 1 < 1000 else np.array([999, 999], np.int32)
    yy = np.array([di["y"], cfg["num_classes"]], np.int32)
    _, f_gpu = target.dit_forward_packed(pu.to_dev(np.repeat(x_prev, 2, 0)), pu.to_dev(tt), pu.to_dev(yy), want_feat=True)
    _, f_ref = fo.dit_forward(w, cfg, np.repeat(x_prev, 2, 0), tt, yy)
    di = dict(di, f_a=f_gpu.cpu().numpy())
    out = _run_draft(drafter, di, cfg_scale, cx, ce, sigma, want_feat=False)
    u = np.random.default_rng(5).random(K, dtype=np.float32)
    dev = lambda a: pu.to_dev(np.asarray(a, np.float32))
    res = target.spec_round(out["x_states"], out["x_last"], out["m_draft"], pu.to_dev(di["t"]), di["y"], cfg_scale,
                            dev(cx), dev(ce), dev(sigma), dev(u), None)
    torch.cuda.synchronize()
    ref_d = fo.draft_steps(wd, w, cfg, di["x_a"], f_ref, di["t"], di["y"], cfg_scale, cx.astype(np.float32),
                           ce.astype(np.float32), sigma.astype(np.float32), di["xi"])
    assert pu.rel_l2(out["m_draft"].cpu().numpy(), ref_d["m_draft"]) < 1e-4
    # verification is compared by composition on the GPU-produced chain (bit-exact decisions need identical inputs)
    ref_v = fo.spec_round(w, cfg, out["x_states"].cpu().numpy(), out["x_last"].cpu().numpy().reshape(di["x_a"].shape),
                          out["m_draft"].cpu().numpy(),
                          di["t"], di["y"], cfg_scale, cx.astype(np.float32), ce.astype(np.float32),
                          sigma.astype(np.float32), u)
    m_gpu = res["m_target"].cpu().numpy().astype(np.float64)
    assert pu.rel_l2(m_gpu, ref_v["m_target"]) < 1e-4
    xd = np.concatenate([out["x_states"].cpu().numpy()[1:].reshape(K - 1, -1), out["x_last"].cpu().numpy()[None]], 0)
    ref = fo.spec_verify(m_gpu[None], out["m_draft"].cpu().numpy()[None], xd[None], sigma.astype(np.float32)[None], u[None])
    pu.compare_verify(dict(accept=res["accept"], n_accept=res["n_accept"], log_ratio=res["log_ratio"],
                           x_out=res["x_out"]), ref, None, u, "draft -> verify chain")
    print("chain: accepted", int(res["n_accept"].item()), "of", K, "log ratios", res["log_ratio"].cpu().numpy())
    drafter.close()
    target.close()


@pytest.mark.parametrize("depth,K", [(1, 2), (2, 1)])
def test_drafter_xl2_512_bf16(depth, K):
    """DiT-XL/2 width at 1024 tokens with guidance (the shape bench.py times; two blocks in the sampler
    benchmark): one or two blocks on two samples are cheap enough for the oracle to check every output."""
    cfg, w, wd, target, drafter = _models("xl2_512", "bf16", depth)
    cfg = dict(cfg, drafter_depth=depth)
    cfg_scale = 4.0
    sched, di, cx, ce, sigma = _draft_inputs(cfg, K, 1, cfg_scale)
    out = _run_draft(drafter, di, cfg_scale, cx, ce, sigma)
    ref = fo.draft_steps(wd, w, cfg, di["x_a"], di["f_a"], di["t"], di["y"], cfg_scale, cx.astype(np.float32),
                         ce.astype(np.float32), sigma.astype(np.float32), di["xi"])
    d = synth.latent_dim(cfg)
    xs_g = out["x_states"].cpu().numpy().reshape(K, d).astype(np.float64)
    m_g = out["m_draft"].cpu().numpy().astype(np.float64)
    for k in range(K):
        cxk, cek = np.float64(np.float32(cx[k])), np.float64(np.float32(ce[k]))
        err = pu.rel_l2((m_g[k] - cxk * xs_g[k]) / cek, (ref["m_draft"][k] - cxk * ref["x_states"][k].reshape(-1)) / cek)
        print(f"xl2_512/bf16 drafter step {k}: eps rel-L2 {err:.3e}")
        assert err <= pu.DIT_REL_L2["bf16"]
    assert pu.rel_l2(out["f_last"].cpu().numpy(), ref["f_last"]) <= pu.DIT_REL_L2["bf16"]
    drafter.close()
    target.close()


@pytest.mark.parametrize("mode,cfg_scale,L", [("fp32", 4.0, 4), ("fp32", 1.0, 3), ("bf16", 4.0, 5)])
def test_free_sample_loop(mode, cfg_scale, L):
    """The whole sampler (Alg. 1) on the GPU against the oracle's loop: same noise, same uniforms.
    In fp32 mode the two chains take the same decisions (a flipped decision would need a log ratio
    within rounding of log u) and end in the same sample; in bf16 mode the means differ by 1e-3, so
    only the bookkeeping and the first round are compared."""
    import torch
    from paper_2511_20390_amd import binding
    cfg, w, wd, target, drafter = _models("tiny", mode, 1, seed=6, out_gain=GAIN)
    sched = fo.ddpm_schedule()
    S = 14
    tmap = (np.arange(S - 1, -1, -1) * 70 + 20).astype(np.int32)
    cx, ce = fo.mean_coefficients(tmap, sched)
    sigma = sched["sigma_clipped"][tmap].copy()
    sigma[-1] = 0.0
    rng = np.random.default_rng(12)
    d = synth.latent_dim(cfg)
    x0 = rng.standard_normal((cfg["in_ch"], cfg["lat_h"], cfg["lat_w"])).astype(np.float32)
    xi = rng.standard_normal((S, d)).astype(np.float32)
    u = rng.random(S).astype(np.float32)
    y = 4
    f32 = lambda a: pu.to_dev(np.asarray(a, np.float32))
    x_gpu, st, log = binding.free_sample(drafter, pu.to_dev(x0), y, cfg_scale, S - 1, L, pu.to_dev(tmap), f32(cx), f32(ce),
                                         f32(sigma), pu.to_dev(xi), pu.to_dev(u))
    x_ref, st_ref = fo.free_sample(wd, w, cfg, x0, y, cfg_scale, tmap, cx.astype(np.float32), ce.astype(np.float32),
                                   sigma.astype(np.float32), S - 1, L, xi, u)
    print(f"{mode} scale {cfg_scale} L={L}: gpu {st} log {log}; oracle {st_ref}")
    assert st["target_calls"] == st["rounds"] + 2 and st["drafter_steps"] >= st["accepted"]
    assert len(log) == st["rounds"] and sum(log) == st["accepted"]
    if mode == "fp32":
        assert log == st_ref["n_accept"]
        assert {k: st[k] for k in ("target_calls", "rounds", "accepted", "drafter_steps")} == \
               {k: st_ref[k] for k in ("target_calls", "rounds", "accepted", "drafter_steps")}
        assert pu.rel_l2(x_gpu.cpu().numpy(), x_ref) < 1e-4
        assert 0 < st["accepted"] < st["drafter_steps"], "the case should exercise both outcomes"
    else:
        # bf16 means differ from the oracle's by ~1e-3: a decision may legitimately differ, after which the
        # chains part; the first round starts from identical inputs and its outcome is compared
        assert abs(log[0] - st_ref["n_accept"][0]) <= 1
    drafter.close()
    target.close()


@pytest.mark.parametrize("cfg_scale,L", [(4.0, 4), (1.0, 6)])
def test_self_speculative_run_and_profile(cfg_scale, L):
    """The offline run of Sec. 3.4 on the GPU (frozen-target drafting) against the oracle: same outcomes,
    same recorded deviations, same final sample; then the profile built from them on both sides."""
    from paper_2511_20390_amd import binding
    cfg = synth.dit_config("tiny")
    w = synth.make_weights(cfg, seed=1, std=0.12)          # state-dependent enough for some rejections
    target = binding.FreeDit(cfg, w, "fp32")
    sched = fo.ddpm_schedule()
    S = 16
    tmap = np.linspace(960, 30, S).round().astype(np.int32)
    cx, ce = fo.mean_coefficients(tmap, sched)
    sigma = sched["sigma_clipped"][tmap].copy()
    sigma[-1] = 0.0
    rng = np.random.default_rng(21)
    d = synth.latent_dim(cfg)
    x0 = rng.standard_normal((cfg["in_ch"], cfg["lat_h"], cfg["lat_w"])).astype(np.float32)
    xi = rng.standard_normal((S, d)).astype(np.float32)
    u = rng.random(S).astype(np.float32)
    f32 = lambda a: pu.to_dev(np.asarray(a, np.float32))
    x_gpu, st, log, delta, acc = binding.free_self_speculative(target, pu.to_dev(x0), 3, cfg_scale, S - 1, L, pu.to_dev(tmap),
                                                               f32(cx), f32(ce), f32(sigma), pu.to_dev(xi), pu.to_dev(u))
    x_ref, st_ref, delta_ref, acc_ref = fo.self_speculative_run(w, cfg, x0, 3, cfg_scale, tmap, cx.astype(np.float32),
                                                                ce.astype(np.float32), sigma.astype(np.float32), S - 1, L, xi, u)
    print(f"scale {cfg_scale} L={L}: gpu {st} log {log}; oracle n_accept {st_ref['n_accept']}")
    print("eps_delta gpu", np.round(delta, 4), "\\n          ref", np.round(delta_ref, 4))
    assert log == st_ref["n_accept"] and np.array_equal(acc, acc_ref)
    chk = ~np.isnan(delta_ref)
    assert np.array_equal(np.isnan(delta), ~chk)
    assert np.allclose(delta[chk], delta_ref[chk], rtol=2e-3, atol=1e-5)
    assert pu.rel_l2(x_gpu.cpu().numpy(), x_ref) < 1e-4
    lam_gpu = binding.free_lambda_profile(delta, 3)
    lam_ref = fo.relaxation_profile_from_deltas(delta_ref, 3)
    assert np.allclose(lam_gpu, lam_ref, rtol=5e-3)
    target.close()


def test_free_sample_on_the_stochasticity_family():
    """The sampler with the transition coefficients of the reverse family with stochasticity 1.5
    (Eq. mean_var_gamma) instead of the DDPM posterior: coefficients are inputs, so this only has to agree
    with the oracle's loop on the same numbers; the larger sigma widens the acceptance region."""
    from paper_2511_20390_amd import binding
    cfg, w, wd, target, drafter = _models("tiny", "fp32", 1, seed=6, out_gain=GAIN)
    S, L, scale = 12, 4, 4.0
    tmap = np.linspace(950, 40, S).round().astype(np.int32)
    cx_all, ce_all, sg_all = binding.free_sde_schedule(1.5)
    ocx, oce, osg = fo.sde_coefficients(1.5)
    assert np.allclose(cx_all, ocx) and np.allclose(sg_all, osg)
    cx, ce, sigma = cx_all[tmap], ce_all[tmap], sg_all[tmap].copy()
    sigma[-1] = 0.0
    rng = np.random.default_rng(31)
    d = synth.latent_dim(cfg)
    x0 = rng.standard_normal((cfg["in_ch"], cfg["lat_h"], cfg["lat_w"])).astype(np.float32)
    xi, u = rng.standard_normal((S, d)).astype(np.float32), rng.random(S).astype(np.float32)
    f32 = lambda a: pu.to_dev(np.asarray(a, np.float32))
    x_gpu, st, log = binding.free_sample(drafter, pu.to_dev(x0), 1, scale, S - 1, L, pu.to_dev(tmap), f32(cx), f32(ce),
                                         f32(sigma), pu.to_dev(xi), pu.to_dev(u))
    x_ref, st_ref = fo.free_sample(wd, w, cfg, x0, 1, scale, tmap, cx.astype(np.float32), ce.astype(np.float32),
                                   sigma.astype(np.float32), S - 1, L, xi, u)
    print("stochasticity 1.5:", st, log)
    assert log == st_ref["n_accept"] and pu.rel_l2(x_gpu.cpu().numpy(), x_ref) < 1e-4
    drafter.close()
    target.close()
