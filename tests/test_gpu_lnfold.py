"""GPU parity of the LayerNorm that is folded into the GEMMs around it (bf16 mode): the three pieces against the
oracle's definitions (layer_norm, modulation, linear, gelu_tanh composed in fp64), then the packed forward and a
whole round with the folded path forced on and off."""
import math

import numpy as np
import pytest

from oracle import free_oracle as fo
from paper_2511_20390_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

OP_TOL, ROW_TOL = 6e-3, 2e-2          # the bf16 operator bounds of test_gpu_dit


def _bf(a):
    return synth.bf16_round(np.asarray(a, np.float32)).astype(np.float64)


def _bf16_dev(a):
    import torch
    return pu.to_dev(np.asarray(a, np.float32), torch.bfloat16)


@pytest.mark.parametrize("B,D,F,depth", [(3, 128, 256, 2), (12, 1152, 4608, 2), (16, 384, 1536, 1), (5, 256, 512, 3)])
def test_fold_vectors(B, D, F, depth):
    """c1 = (1 + scale) W^T, c0 = shift W^T + b for both folded layers of every block."""
    from paper_2511_20390_amd import binding
    rng = np.random.default_rng(B * D + depth)
    mod = (0.5 * rng.standard_normal((B, 6 * depth * D + 2 * D))).astype(np.float32)
    wq = [(rng.standard_normal((3 * D, D)) / math.sqrt(D)).astype(np.float32) for _ in range(depth)]
    bq = [rng.standard_normal(3 * D).astype(np.float32) for _ in range(depth)]
    w1 = [(rng.standard_normal((F, D)) / math.sqrt(D)).astype(np.float32) for _ in range(depth)]
    b1 = [rng.standard_normal(F).astype(np.float32) for _ in range(depth)]
    fold = binding.op_ln_fold_vectors(pu.to_dev(mod), D, F, [_bf16_dev(w) for w in wq], [pu.to_dev(b) for b in bq],
                                      [_bf16_dev(w) for w in w1], [pu.to_dev(b) for b in b1]).cpu().numpy().astype(np.float64)
    rows = depth * (3 * D + F)
    assert fold.shape == (B, 2 * rows)
    m64 = mod.astype(np.float64)
    for l in range(depth):
        for which, (W, b, n) in enumerate(((wq[l], bq[l], 3 * D), (w1[l], b1[l], F))):
            shift = m64[:, l * 6 * D + (3 if which else 0) * D:][:, :D]
            scale = m64[:, l * 6 * D + (4 if which else 1) * D:][:, :D]
            r0 = l * (3 * D + F) + (3 * D if which else 0)
            c1 = (1.0 + scale) @ _bf(W).T
            c0 = shift @ _bf(W).T + b
            # against the vectors as the kernel uses them (rounded to bf16): fp32 accumulation only
            c1r = _bf(1.0 + scale.astype(np.float32)) @ _bf(W).T
            c0r = _bf(shift) @ _bf(W).T + b
            assert pu.rel_l2(fold[:, r0:r0 + n], c1r) < 2e-5, (l, which)
            assert pu.rel_l2(fold[:, rows + r0:rows + r0 + n], c0r) < 2e-5, (l, which)
            # against the exact vectors: one bf16 rounding per term
            assert pu.rel_l2(fold[:, r0:r0 + n], c1) < 4e-3 and pu.rel_l2(fold[:, rows + r0:rows + r0 + n], c0) < 4e-3


@pytest.mark.parametrize("M,N,K,rows", [(256, 128, 64, 32), (1000, 1152, 1152, 200), (2048, 1152, 4608, 1024),
                                        (12288, 1152, 1152, 1024), (6144, 1152, 4608, 1024), (777, 384, 128, 111)])
def test_residual_update_that_prepares_the_next_layer_norm(M, N, K, rows):
    """resid += gate (A W^T + b); z = bf16(resid_new (1 + scale_next)); per row and 128-column slot the sums of
    resid_new and resid_new^2."""
    import torch
    from paper_2511_20390_amd import binding
    rng = np.random.default_rng(M + N + K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) / math.sqrt(K)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    nb = (M + rows - 1) // rows
    mod = rng.standard_normal((nb, 3 * N)).astype(np.float32)         # [gate | scale_next | unused]: one row stride
    resid = (rng.standard_normal((M, N)) * 2 + 0.7).astype(np.float32)
    dres, dmod = pu.to_dev(resid), pu.to_dev(mod)
    z, stats = binding.op_linear_resid_prep(_bf16_dev(A), _bf16_dev(W), pu.to_dev(bias), dres, dmod[:, :N],
                                            dmod[:, N:2 * N], rows)
    torch.cuda.synchronize()
    smp = np.arange(M) // rows
    want = resid + mod[smp, :N].astype(np.float64) * (_bf(A) @ _bf(W).T + bias)
    got = dres.cpu().numpy().astype(np.float64)
    assert pu.rel_l2(got, want) < 2e-5 and pu.row_rel_l2(got, want, N) < 1e-4
    # z from the residual the GPU really wrote (its own fp32 values), rounded once to bf16
    z_want = got.astype(np.float32) * (1.0 + mod[smp, N:2 * N])
    zg = z.float().cpu().numpy().astype(np.float64)
    assert np.max(np.abs(zg - z_want) / (np.abs(z_want) + 1e-30)) < 2.0 ** -8 + 1e-6     # one bf16 rounding (+ fp32 product)
    st = stats.cpu().numpy().astype(np.float64)
    assert st.shape == (M, N // 128, 2)
    g3 = got.reshape(M, N // 128, 128)
    assert np.allclose(st[:, :, 0], g3.sum(-1), rtol=1e-5, atol=1e-3)
    assert np.allclose(st[:, :, 1], (g3 * g3).sum(-1), rtol=1e-5, atol=1e-3)


@pytest.mark.parametrize("gelu", [False, True])
@pytest.mark.parametrize("M,N,K,rows,mean", [(256, 256, 128, 32, 0.0), (1024, 3456, 1152, 256, 0.5),
                                             (12288, 3456, 1152, 1024, 0.3), (12288, 4608, 1152, 1024, 0.0),
                                             (6144, 4608, 1152, 1024, 1.0), (1000, 392, 384, 96, 0.2)])
def test_linear_after_a_folded_layer_norm(M, N, K, rows, mean, gelu):
    """act((LN(x) (1 + scale) + shift) W^T + b) from z = bf16(x (1 + scale)), the row sums and the fold vectors,
    against the oracle's layer_norm / linear / gelu_tanh on the same x."""
    from paper_2511_20390_amd import binding
    rng = np.random.default_rng(M + N + K + int(gelu))
    x = (rng.standard_normal((M, K)) * (1 + 2 * rng.random((M, 1))) + mean * (1 + rng.random((M, 1)))).astype(np.float32)
    nb = (M + rows - 1) // rows
    shift = (0.3 * rng.standard_normal((nb, K))).astype(np.float32)
    scale = (0.3 * rng.standard_normal((nb, K))).astype(np.float32)
    W = (rng.standard_normal((N, K)) / math.sqrt(K)).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32)
    smp = np.arange(M) // rows
    x64 = x.astype(np.float64)
    ref = fo.linear(fo.layer_norm(x64) * (1.0 + scale[smp]) + shift[smp], _bf(W), b)
    if gelu:
        ref = fo.gelu_tanh(ref)
    # inputs of the folded form, prepared in fp64 / fp32 on the host (the GPU's own producers have their tests above)
    z = x * (1.0 + scale[smp])
    x3 = x64.reshape(M, K // 128, 128)
    stats = np.stack([x3.sum(-1), (x3 * x3).sum(-1)], axis=-1).astype(np.float32)
    c = np.concatenate([(1.0 + scale.astype(np.float64)) @ _bf(W).T, shift.astype(np.float64) @ _bf(W).T + b], axis=1)
    dc = pu.to_dev(c.astype(np.float32))
    out = binding.op_linear_ln(_bf16_dev(z), _bf16_dev(W), pu.to_dev(stats), dc[:, :N], dc[:, N:], rows, gelu)
    out = out.float().cpu().numpy()
    assert pu.rel_l2(out, ref) < OP_TOL and pu.row_rel_l2(out, ref, N) < ROW_TOL


def _model_case(over, B, seed, zero_mean_shift=0.0):
    from paper_2511_20390_amd import binding
    cfg = synth.dit_config("small", **over)
    # weights four times the usual spread: with small modulation gates the blocks would hardly move the residual
    # stream and the comparison would say little about what happens inside them
    w = pu.weights_for(cfg, "bf16", seed, std=0.08)
    rng = np.random.default_rng(seed + 11)
    x = (rng.standard_normal((B, cfg["in_ch"], cfg["lat_h"], cfg["lat_w"])) + zero_mean_shift).astype(np.float32)
    t = rng.integers(0, 1000, B).astype(np.int32)
    y = rng.integers(0, cfg["num_classes"] + 1, B).astype(np.int32)
    return cfg, w, x, t, y, binding.FreeDit(cfg, w, "bf16")


@pytest.mark.parametrize("over,B", [
    (dict(hidden=256, heads=4, mlp_hidden=1024, depth=3, lat_h=16, lat_w=16), 5),       # 64 tokens per sample
    (dict(hidden=384, heads=6, mlp_hidden=1536, depth=2, lat_h=24, lat_w=16), 3),       # 96 tokens: blocks of 32 rows
    (dict(hidden=128, heads=2, mlp_hidden=256, depth=4, lat_h=32, lat_w=32), 2),        # 256 tokens
    (dict(hidden=256, heads=4, mlp_hidden=512, depth=1, lat_h=16, lat_w=16), 7)])       # a single block
def test_forward_with_the_layer_norms_folded_against_the_oracle(over, B):
    """The packed forward with the folded path forced (shapes far below the size from which it is the default),
    against the oracle to the DiT tolerance, and against the separate LayerNorm kernel."""
    from paper_2511_20390_amd import binding
    cfg, w, x, t, y, model = _model_case(over, B, seed=3)
    dx, dt, dy = pu.to_dev(x), pu.to_dev(t), pu.to_dev(y)
    assert not model.ln_fold_active(B)                          # small batch: the separate kernel by default
    e_off, f_off = model.dit_forward_packed(dx, dt, dy, want_feat=True)
    e_off, f_off = e_off.cpu().numpy(), f_off.cpu().numpy()
    model.set_ln_fold(binding.LN_FOLD_REQUIRE)
    assert model.ln_fold_active(B)
    e_on, f_on = model.dit_forward_packed(dx, dt, dy, want_feat=True)
    e_on, f_on = e_on.cpu().numpy(), f_on.cpu().numpy()
    ref, ref_feat = fo.dit_forward(w, cfg, x, t, y)
    for name, e, f in (("separate", e_off, f_off), ("folded", e_on, f_on)):
        e1, e2 = pu.rel_l2(e, ref), pu.rel_l2(f, ref_feat)
        print(f"{name}: eps rel-L2 {e1:.3e}, top-feature rel-L2 {e2:.3e}")
        assert e1 <= pu.DIT_REL_L2["bf16"] and e2 <= pu.DIT_REL_L2["bf16"]
        p = cfg["patch"]
        assert pu.row_rel_l2(pu.token_rows(e, p), pu.token_rows(ref, p), e.shape[1] * p * p) <= pu.ROW_REL_L2["bf16"]
        assert pu.row_rel_l2(f, ref_feat, cfg["hidden"]) <= pu.ROW_REL_L2["bf16"]
    assert not np.array_equal(f_on, f_off)                      # the two paths really differ in rounding
    model.set_ln_fold(binding.LN_FOLD_OFF)
    e_again, _ = model.dit_forward_packed(dx, dt, dy, want_feat=True)
    assert np.array_equal(e_again.cpu().numpy(), e_off)
    model.close()


def test_requiring_the_folded_path_on_a_model_it_does_not_cover_is_an_error():
    from paper_2511_20390_amd import binding
    cfg, w, x, t, y, model = _model_case(dict(hidden=192, heads=3, mlp_hidden=384, depth=1, lat_h=8, lat_w=8), 2, seed=1)
    with pytest.raises(binding.FreeError):                      # hidden % 128 != 0
        model.set_ln_fold(binding.LN_FOLD_REQUIRE)
    assert not model.ln_fold_active(64)
    model.close()
    cfg, w, x, t, y, model = _model_case(dict(hidden=128, heads=2, mlp_hidden=256, depth=1, lat_h=10, lat_w=14), 2, seed=1)
    with pytest.raises(binding.FreeError):                      # 35 tokens per sample: not a multiple of 32
        model.set_ln_fold(binding.LN_FOLD_REQUIRE)
    model.close()


def test_folded_forward_is_the_default_at_the_headline_shape_and_both_schedules_agree():
    """DiT-XL/2 at 512^2, 12 packed states: the folded path is taken without being asked for, and the one- and the
    two-stream schedule give identical bits (the fold vectors are computed on a third stream in both)."""
    import torch
    from paper_2511_20390_amd import binding
    cfg = synth.dit_config("xl2_512")
    w = pu.weights_for(cfg, "bf16", 0)
    model = binding.FreeDit(cfg, w, "bf16")
    B = 12
    assert model.ln_fold_active(B) and not model.ln_fold_active(2)
    rng = np.random.default_rng(5)
    x = pu.to_dev(rng.standard_normal((B, cfg["in_ch"], cfg["lat_h"], cfg["lat_w"])).astype(np.float32))
    t = pu.to_dev(rng.integers(0, 1000, B).astype(np.int32))
    y = pu.to_dev(rng.integers(0, cfg["num_classes"] + 1, B).astype(np.int32))
    outs = []
    for n in (1, 2, 3, 1):
        model.set_streams(n)
        outs.append(model.dit_forward_packed(x, t, y).clone())
    torch.cuda.synchronize()
    assert all(torch.equal(outs[0], o) for o in outs[1:])
    model.set_ln_fold(binding.LN_FOLD_OFF)
    model.set_streams(1)
    off = model.dit_forward_packed(x, t, y)
    d = pu.rel_l2(outs[0].cpu().numpy(), off.cpu().numpy())
    print(f"folded vs separate at the headline shape: rel-L2 {d:.3e}")
    assert 0.0 < d < pu.DIT_REL_L2["bf16"]
    model.close()
