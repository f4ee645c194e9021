"""Pins for the schedule / eps->mean and the DiT-forward parts of the oracle (CPU only).

The schedule is pinned to the Gaussian-conditioning identities of the DDPM
forward process (textbook, independent of the oracle's formula).  The DiT
forward has no published activations; it is pinned by invariants (adaLN-Zero
identity, permutation/packing invariance, guidance special cases, the
shift-invariance of sinusoidal inner products) and by agreement with a second
implementation assembled from PyTorch CPU library routines.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import free_oracle as fo
from paper_2511_20390_amd import synth


# ---- schedule and eps -> mean (Eq. ddpm_update, App. C) ----------------------
def test_schedule_basic_values():
    s = fo.ddpm_schedule()
    assert s["beta"][0] == pytest.approx(1e-4) and s["beta"][-1] == pytest.approx(0.02)
    assert s["alphabar"][-1] == pytest.approx(4.0358e-5, rel=1e-3)      # 1e-4 -> 0.02 linear, T = 1000
    assert s["sigma"][0] == 0.0 and s["sigma_clipped"][0] == s["sigma"][1] > 0
    assert np.all(np.diff(s["alphabar"]) < 0)


def test_posterior_variance_is_gaussian_conditioning():
    """betatilde_i = Var(x_{i-1} | x_i, x_0) for the forward chain
    x_{i-1} = sqrt(ab_{i-1}) x0 + sqrt(1-ab_{i-1}) e1, x_i = sqrt(a_i) x_{i-1} + sqrt(b_i) e2."""
    s = fo.ddpm_schedule()
    for i in (1, 2, 10, 500, 999):
        var_prev = 1 - s["alphabar"][i - 1]
        cov = math.sqrt(s["alpha"][i]) * var_prev
        var_cur = s["alpha"][i] * var_prev + s["beta"][i]
        assert var_cur == pytest.approx(1 - s["alphabar"][i], rel=1e-12)
        assert s["beta_tilde"][i] == pytest.approx(var_prev - cov ** 2 / var_cur, rel=1e-9)


def test_eps_to_mean_is_posterior_mean_for_the_true_noise():
    """With eps the noise that produced x_i from x_0, the transition mean equals
    the posterior mean of q(x_{i-1} | x_i, x_0) (DDPM, posterior of the forward chain)."""
    s = fo.ddpm_schedule()
    rng = np.random.default_rng(0)
    x0, eps = rng.standard_normal(16), rng.standard_normal(16)
    for i in (1, 7, 400, 999):
        ab, abp, a, b = s["alphabar"][i], s["alphabar"][i - 1], s["alpha"][i], s["beta"][i]
        xi = math.sqrt(ab) * x0 + math.sqrt(1 - ab) * eps
        post = math.sqrt(abp) * b / (1 - ab) * x0 + math.sqrt(a) * (1 - abp) / (1 - ab) * xi
        np.testing.assert_allclose(fo.eps_to_mean(xi, eps, i, s), post, rtol=1e-10, atol=1e-12)
        cx, ce = fo.mean_coefficients(i, s)
        np.testing.assert_allclose(cx * xi + ce * eps, post, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(fo.eps_to_mean(xi, 0 * eps, 5, s), xi / math.sqrt(s["alpha"][5]))


# ---- embeddings ---------------------------------------------------------------
def test_timestep_embedding_properties():
    e = fo.timestep_embedding(np.array([0, 3, 10, 999]), 256)
    assert e.shape == (4, 256)
    np.testing.assert_allclose(e[0], np.r_[np.ones(128), np.zeros(128)])     # cos first, then sin
    # first frequency is 1: cos(t), sin(t); last is 10000^(-127/128)
    assert e[1, 0] == pytest.approx(math.cos(3.0)) and e[1, 128] == pytest.approx(math.sin(3.0))
    assert e[2, 127] == pytest.approx(math.cos(10.0 * 10000 ** (-127 / 128)))
    # <e(t), e(t')> depends on t - t' only
    f = fo.timestep_embedding(np.array([100, 103, 500, 503]), 256)
    assert f[0] @ f[1] == pytest.approx(f[2] @ f[3], rel=1e-9)


def test_pos_embed_properties():
    gh, gw, D = 5, 7, 32
    pe = fo.pos_embed_2d(gh, gw, D).reshape(gh, gw, D)
    np.testing.assert_allclose(pe[0, 0], np.r_[np.zeros(8), np.ones(8), np.zeros(8), np.ones(8)])
    assert pe[2, 3, 0] == pytest.approx(math.sin(3.0))       # first quarter: column index
    assert pe[2, 3, 16] == pytest.approx(math.sin(2.0))      # third quarter: row index
    assert pe[2, 3, 15] == pytest.approx(math.cos(3.0 / 10000 ** (7 / 8)))
    # inner products are shift invariant
    assert pe[1, 2] @ pe[3, 5] == pytest.approx(pe[2, 3] @ pe[4, 6], rel=1e-9)
    assert np.allclose((pe ** 2).sum(-1), D / 2)


def test_patchify_unpatchify_layout():
    B, C, H, W, p = 2, 3, 4, 6, 2
    x = np.arange(B * C * H * W, dtype=float).reshape(B, C, H, W)
    tok = fo.patchify(x, p)
    assert tok.shape == (B, 6, C * p * p)
    # token (i=1, j=2), element (c=2, ph=1, pw=0)
    assert tok[1, 1 * 3 + 2, 2 * 4 + 1 * 2 + 0] == x[1, 2, 1 * 2 + 1, 2 * 2 + 0]
    # unpatchify uses (ph, pw, c) per token
    t2 = np.arange(B * 6 * p * p * C, dtype=float).reshape(B, 6, p * p * C)
    img = fo.unpatchify(t2, p, C, 2, 3)
    assert img[1, 2, 1 * 2 + 1, 2 * 2 + 0] == t2[1, 1 * 3 + 2, (1 * 2 + 0) * C + 2]
    # library cross-check: unfold gives (c, ph, pw) patches in row-major patch order
    ref = TF.unfold(torch.from_numpy(x), kernel_size=p, stride=p).transpose(1, 2).numpy()
    np.testing.assert_array_equal(tok, ref)
    ref_img = TF.fold(torch.from_numpy(t2.reshape(B, 6, p, p, C).transpose(0, 1, 4, 2, 3).reshape(B, 6, -1))
                      .transpose(1, 2), output_size=(H, W), kernel_size=p, stride=p).numpy()
    np.testing.assert_array_equal(img, ref_img)


# ---- DiT forward: second implementation from PyTorch library routines ---------
def _torch_dit(w, cfg, x, t, y):
    tw = {k: torch.from_numpy(np.asarray(v, np.float64)) for k, v in w.items()}
    x = torch.from_numpy(np.asarray(x, np.float64))
    B, C, H, W = x.shape
    p, D, heads = cfg["patch"], cfg["hidden"], cfg["heads"]
    gh, gw = H // p, W // p
    half = cfg["t_freq_dim"] // 2
    freqs = torch.exp(-math.log(10000.0) * torch.arange(half, dtype=torch.float64) / half)
    ang = torch.tensor(t, dtype=torch.float64)[:, None] * freqs[None]
    temb = torch.cat([torch.cos(ang), torch.sin(ang)], dim=1)
    c = TF.linear(TF.silu(TF.linear(temb, tw["t_w1"], tw["t_b1"])), tw["t_w2"], tw["t_b2"])
    c = c + TF.embedding(torch.tensor(y, dtype=torch.long), tw["y_table"])
    sc = TF.silu(c)
    # patch embedding as a strided convolution
    tok = TF.conv2d(x, tw["patch_w"].reshape(D, C, p, p), tw["patch_b"], stride=p).flatten(2).transpose(1, 2)
    q4 = D // 4
    om = 1.0 / 10000.0 ** (torch.arange(q4, dtype=torch.float64) / q4)
    jj = torch.arange(gw, dtype=torch.float64).repeat(gh)
    ii = torch.arange(gh, dtype=torch.float64).repeat_interleave(gw)
    pos = torch.cat([torch.sin(jj[:, None] * om), torch.cos(jj[:, None] * om),
                     torch.sin(ii[:, None] * om), torch.cos(ii[:, None] * om)], dim=1)
    h = tok + pos
    for l in range(cfg["depth"]):
        mod = TF.linear(sc, tw[f"blk{l}.ada_w"], tw[f"blk{l}.ada_b"])
        sh1, sc1, g1, sh2, sc2, g2 = mod.chunk(6, dim=1)
        hn = TF.layer_norm(h, (D,), eps=1e-6) * (1 + sc1[:, None]) + sh1[:, None]
        qkv = TF.linear(hn, tw[f"blk{l}.qkv_w"], tw[f"blk{l}.qkv_b"]).reshape(B, -1, 3, heads, D // heads)
        q, k, v = qkv.permute(2, 0, 3, 1, 4)
        a = TF.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(B, -1, D)
        h = h + g1[:, None] * TF.linear(a, tw[f"blk{l}.proj_w"], tw[f"blk{l}.proj_b"])
        hn = TF.layer_norm(h, (D,), eps=1e-6) * (1 + sc2[:, None]) + sh2[:, None]
        mid = TF.gelu(TF.linear(hn, tw[f"blk{l}.fc1_w"], tw[f"blk{l}.fc1_b"]), approximate="tanh")
        h = h + g2[:, None] * TF.linear(mid, tw[f"blk{l}.fc2_w"], tw[f"blk{l}.fc2_b"])
    feat = h
    sh, scl = TF.linear(sc, tw["fin_ada_w"], tw["fin_ada_b"]).chunk(2, dim=1)
    o = TF.linear(TF.layer_norm(h, (D,), eps=1e-6) * (1 + scl[:, None]) + sh[:, None], tw["fin_w"], tw["fin_b"])
    c_out = 2 * C
    o = o.reshape(B, gh, gw, p, p, c_out)
    img = torch.einsum("bhwpqc->bchpwq", o).reshape(B, c_out, H, W)
    return img.numpy(), feat.numpy()


@pytest.mark.parametrize("name", ["tiny", "small"])
def test_forward_matches_library_routine_implementation(name):
    cfg = synth.dit_config(name)
    w = synth.make_weights(cfg, seed=1)
    rng = np.random.default_rng(1)
    B = 3
    x = rng.standard_normal((B, cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]))
    t = [999, 17, 0]
    y = [3, cfg["num_classes"], 0]
    out, feat = fo.dit_forward(w, cfg, x, t, y)
    ref_out, ref_feat = _torch_dit(w, cfg, x, t, y)
    np.testing.assert_allclose(out, ref_out, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(feat, ref_feat, rtol=1e-9, atol=1e-11)
    assert out.std() > 1e-3                 # non-trivial output


# ---- DiT forward: invariants ----------------------------------------------------
def _setup(name="tiny", seed=0, **kw):
    cfg = synth.dit_config(name)
    w = synth.make_weights(cfg, seed=seed, **kw)
    rng = np.random.default_rng(seed + 50)
    x = rng.standard_normal((4, cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]))
    t = np.array([900, 500, 20, 3])
    y = np.array([1, 7, 2, cfg["num_classes"]])
    return cfg, w, x, t, y


def test_adaln_zero_makes_every_block_the_identity():
    cfg, w, x, t, y = _setup(zero_adaln=True)
    out, feat = fo.dit_forward(w, cfg, x, t, y)
    cfg0 = dict(cfg, depth=0)
    out0, feat0 = fo.dit_forward(w, cfg0, x, t, y)
    np.testing.assert_array_equal(feat, feat0)         # blocks changed nothing
    np.testing.assert_array_equal(out, out0)
    # with zero modulation the output cannot depend on timestep or label
    out_b, _ = fo.dit_forward(w, cfg, x, t[::-1].copy(), y[::-1].copy())
    np.testing.assert_array_equal(out, out_b)
    # ... while with non-zero modulation the blocks do act
    cfg, w, x, t, y = _setup()
    assert np.abs(fo.dit_forward(w, cfg, x, t, y)[1] - fo.dit_forward(w, dict(cfg, depth=0), x, t, y)[1]).max() > 1e-3


def test_gate_only_zero_is_identity_too():
    """Zeroing just the two gate thirds of the modulation is enough."""
    cfg, w, x, t, y = _setup()
    D = cfg["hidden"]
    for l in range(cfg["depth"]):
        for g in (2, 5):
            w[f"blk{l}.ada_w"][g * D:(g + 1) * D] = 0
            w[f"blk{l}.ada_b"][g * D:(g + 1) * D] = 0
    np.testing.assert_array_equal(fo.dit_forward(w, cfg, x, t, y)[1],
                                  fo.dit_forward(w, dict(cfg, depth=0), x, t, y)[1])


def test_pack_permutation_and_packing_invariance():
    cfg, w, x, t, y = _setup()
    out, feat = fo.dit_forward(w, cfg, x, t, y)
    perm = np.array([2, 0, 3, 1])
    outp, featp = fo.dit_forward(w, cfg, x[perm], t[perm], y[perm])
    np.testing.assert_allclose(outp, out[perm], rtol=1e-12, atol=1e-14)
    for b in range(4):
        o1, f1 = fo.dit_forward(w, cfg, x[b:b + 1], t[b:b + 1], y[b:b + 1])
        np.testing.assert_allclose(o1[0], out[b], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(f1[0], feat[b], rtol=1e-12, atol=1e-14)
    sub, _ = fo.dit_forward(w, cfg, x, t, y, samples=[3, 1])
    np.testing.assert_allclose(sub, out[[3, 1]], rtol=1e-12, atol=1e-14)


def test_timestep_and_label_matter():
    cfg, w, x, t, y = _setup()
    base = fo.dit_forward(w, cfg, x[:1], t[:1], y[:1])[0]
    assert np.abs(fo.dit_forward(w, cfg, x[:1], t[:1] - 1, y[:1])[0] - base).max() > 1e-6
    assert np.abs(fo.dit_forward(w, cfg, x[:1], t[:1], y[:1] + 1)[0] - base).max() > 1e-6


def test_guidance_special_cases():
    rng = np.random.default_rng(0)
    ec, en = rng.standard_normal((2, 3, 4, 8, 8))
    np.testing.assert_allclose(fo.cfg_combine(ec, en, 1.0), ec, atol=1e-15)
    np.testing.assert_allclose(fo.cfg_combine(ec, ec, 4.0), ec, atol=1e-15)
    np.testing.assert_allclose(fo.cfg_combine(ec, en, 4.0), 4 * ec - 3 * en, atol=1e-14)


def test_round_means_and_spec_round_composition():
    """spec_round = packed forward (+guidance) -> eps->mean -> verification loop."""
    cfg = synth.dit_config("tiny")
    w = synth.make_weights(cfg, seed=0)
    s = fo.ddpm_schedule()
    K = 6
    ri = synth.make_round_inputs(cfg, K, 0, s["sigma_clipped"], 0.05)
    cx, ce = fo.mean_coefficients(ri["t"], s)
    # label == null label: guidance has no effect whatever the scale
    m_a = fo.round_means(w, cfg, ri["x_states"], ri["t"], cfg["num_classes"], 4.0, cx, ce)
    m_b = fo.round_means(w, cfg, ri["x_states"], ri["t"], cfg["num_classes"], 1.0, cx, ce)
    np.testing.assert_allclose(m_a, m_b, rtol=1e-12, atol=1e-13)
    # composition, with draft means calibrated around the target so outcomes are mixed
    m = fo.round_means(w, cfg, ri["x_states"], ri["t"], ri["y"], 4.0, cx, ce).reshape(K, -1)
    d = m.shape[1]
    rng = np.random.default_rng(5)
    sig = ri["sigma"].astype(np.float64)
    m_draft = m + (1.349 / math.sqrt(d)) * sig[:, None] * rng.standard_normal((K, d))
    x_d = m_draft + sig[:, None] * rng.standard_normal((K, d))
    x_states = np.concatenate([ri["x_states"][:1].reshape(1, -1), x_d[:K - 1]], 0).reshape(ri["x_states"].shape)
    res = fo.spec_round(w, cfg, x_states, x_d[K - 1].reshape(ri["x_last"].shape), m_draft, ri["t"], ri["y"],
                        4.0, cx, ce, ri["sigma"], ri["u"])
    m2 = fo.round_means(w, cfg, x_states, ri["t"], ri["y"], 4.0, cx, ce).reshape(K, -1)
    ref = fo.spec_verify(m2[None], m_draft[None], x_d[None], sig[None], ri["u"][None])
    assert res["n_accept"][0] == ref["n_accept"][0]
    np.testing.assert_array_equal(res["accept"], ref["accept"])
    np.testing.assert_array_equal(res["x_out"], ref["x_out"])
    for k in range(K):      # eps -> mean through the schedule function
        out, _ = fo.dit_forward(w, cfg, np.stack([x_states[k]] * 2), [ri["t"][k]] * 2, [ri["y"], cfg["num_classes"]])
        eps = fo.cfg_combine(out[0, :4], out[1, :4], 4.0)
        np.testing.assert_allclose(res["m_target"][k], fo.eps_to_mean(x_states[k], eps, ri["t"][k], s).ravel(),
                                   rtol=1e-10, atol=1e-12)
