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
            # activations enter as a bf16 high part plus a bf16 remainder: about 2^-16 relative per element
            assert pu.rel_l2(fold[:, r0:r0 + n], c1) < 2e-5, (l, which)
            assert pu.rel_l2(fold[:, rows + r0:rows + r0 + n], c0) < 2e-5, (l, which)


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
