"""GPU parity of the DiT operators, the packed forward and a whole round against the
oracle (through the C ABI)."""
import math

import numpy as np
import pytest

from oracle import free_oracle as fo
from paper_2511_20390_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

OP_TOL = {"fp32": 2e-5, "bf16": 6e-3}


def _tdtype(mode):
    import torch
    return torch.float32 if mode == "fp32" else torch.bfloat16


def _vals(a, mode):
    """Values the GPU really sees (bf16-rounded in bf16 mode), as float64."""
    return (synth.bf16_round(a) if mode == "bf16" else np.asarray(a, np.float32)).astype(np.float64)


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
@pytest.mark.parametrize("M,N,K", [(96, 192, 64), (576, 432, 144), (300, 1152, 1152), (1536, 3456, 1152),
                                   (257, 136, 328), (1024, 1152, 4608)])
def test_op_linear(mode, M, N, K):
    import torch
    from paper_2511_20390_amd import binding
    rng = np.random.default_rng(M + N + K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) / math.sqrt(K)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    Av, Wv = _vals(A, mode), _vals(W, mode)
    ref = Av @ Wv.T + bias
    dA, dW, db = pu.to_dev(A, _tdtype(mode)), pu.to_dev(W, _tdtype(mode)), pu.to_dev(bias)
    out = binding.op_linear(dA, dW, db, mode, binding.EPI_BIAS)
    assert pu.rel_l2(out.float().cpu().numpy(), ref) < OP_TOL[mode]
    out = binding.op_linear(dA, dW, db, mode, binding.EPI_BIAS_GELU)
    assert pu.rel_l2(out.float().cpu().numpy(), fo.gelu_tanh(ref)) < OP_TOL[mode]
    rows = 48 if M % 48 == 0 else M
    nb = M // rows
    gate = rng.standard_normal((nb, 3 * N)).astype(np.float32)
    resid = rng.standard_normal((M, N)).astype(np.float32)
    dres = pu.to_dev(resid)
    dgate = pu.to_dev(gate)
    binding.op_linear(dA, dW, db, mode, binding.EPI_GATE_RESID, resid=dres, gate=dgate[:, N:2 * N],
                      rows_per_sample=rows)
    torch.cuda.synchronize()
    ref2 = resid + np.repeat(gate[:, N:2 * N], rows, axis=0) * ref
    assert pu.rel_l2(dres.cpu().numpy(), ref2) < OP_TOL[mode]


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
@pytest.mark.parametrize("B,N,heads,dh", [(2, 16, 4, 16), (3, 96, 2, 72), (2, 256, 3, 72), (1, 1024, 2, 72),
                                          (2, 200, 2, 64), (1, 77, 1, 128)])
def test_op_attention(mode, B, N, heads, dh):
    from paper_2511_20390_amd import binding
    rng = np.random.default_rng(B * N + dh)
    D = heads * dh
    qkv = (rng.standard_normal((B * N, 3 * D)) * 1.5).astype(np.float32)
    v = _vals(qkv, mode).reshape(B, N, 3, heads, dh)
    ref = np.empty((B, N, heads, dh))
    for b in range(B):
        for h in range(heads):
            ref[b, :, h] = fo.attention(v[b, :, 0, h], v[b, :, 1, h], v[b, :, 2, h])
    out = binding.op_attention(pu.to_dev(qkv, _tdtype(mode)), B, N, heads, dh, mode)
    assert pu.rel_l2(out.float().cpu().numpy(), ref.reshape(B * N, D)) < OP_TOL[mode]


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
@pytest.mark.parametrize("M,D,rows", [(96, 64, 16), (576, 144, 96), (1030, 1152, 515)])
def test_op_ln_modulate(mode, M, D, rows):
    from paper_2511_20390_amd import binding
    rng = np.random.default_rng(M + D)
    x = (rng.standard_normal((M, D)) * 2 + 0.5).astype(np.float32)
    mod = rng.standard_normal((M // rows, 2 * D)).astype(np.float32)
    ref = fo.layer_norm(x.astype(np.float64)) * (1 + np.repeat(mod[:, D:], rows, 0)) + np.repeat(mod[:, :D], rows, 0)
    dmod = pu.to_dev(mod)
    out = binding.op_ln_modulate(pu.to_dev(x), dmod[:, :D], dmod[:, D:], rows, mode)
    assert pu.rel_l2(out.float().cpu().numpy(), ref) < (2e-6 if mode == "fp32" else 4e-3)


def _forward_case(name, mode, B, seed, **wkw):
    from paper_2511_20390_amd import binding
    cfg = synth.dit_config(name)
    w = pu.weights_for(cfg, mode, seed, **wkw)
    rng = np.random.default_rng(seed + 7)
    x = rng.standard_normal((B, cfg["in_ch"], cfg["lat_h"], cfg["lat_w"])).astype(np.float32)
    t = rng.integers(0, 1000, B).astype(np.int32)
    t[0] = 999
    y = rng.integers(0, cfg["num_classes"] + 1, B).astype(np.int32)
    y[-1] = cfg["num_classes"]
    model = binding.FreeDit(cfg, w, mode)
    eps, feat = model.dit_forward_packed(pu.to_dev(x), pu.to_dev(t), pu.to_dev(y), want_feat=True)
    return cfg, w, x, t, y, eps.cpu().numpy(), feat.cpu().numpy(), model


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
@pytest.mark.parametrize("name,B", [("tiny", 6), ("small", 6), ("small", 1)])
def test_forward_parity(name, B, mode):
    cfg, w, x, t, y, eps, feat, model = _forward_case(name, mode, B, seed=1)
    ref, ref_feat = fo.dit_forward(w, cfg, x, t, y)
    e1, e2 = pu.rel_l2(eps, ref), pu.rel_l2(feat, ref_feat)
    print(f"{name}/{mode} B={B}: eps rel-L2 {e1:.3e}, top-feature rel-L2 {e2:.3e}")
    assert e1 <= pu.DIT_REL_L2[mode] and e2 <= pu.DIT_REL_L2[mode]
    model.close()


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
def test_forward_adaln_zero_blocks_are_identity(mode):
    """With zero modulation the GPU blocks must leave the token stream untouched:
    the top feature equals the depth-0 oracle embedding exactly up to fp32 rounding."""
    cfg, w, x, t, y, eps, feat, model = _forward_case("tiny", mode, 3, seed=2, zero_adaln=True)
    _, ref_feat = fo.dit_forward(w, dict(cfg, depth=0), x, t, y)
    assert pu.rel_l2(feat, ref_feat) < 1e-6
    model.close()


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
def test_forward_packing_invariance(mode):
    """A state gives the same output alone (B = 1) as inside the pack."""
    from paper_2511_20390_amd import binding
    cfg, w, x, t, y, eps, feat, model = _forward_case("small", mode, 4, seed=3)
    for b in (0, 3):
        e1 = model.dit_forward_packed(pu.to_dev(x[b:b + 1]), pu.to_dev(t[b:b + 1]), pu.to_dev(y[b:b + 1]))
        assert pu.rel_l2(e1.cpu().numpy()[0], eps[b]) < (1e-6 if mode == "fp32" else 1e-2)
    model.close()


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
@pytest.mark.parametrize("name,cfg_scale", [("tiny", 4.0), ("tiny", 1.0), ("small", 4.0)])
def test_round_parity(name, cfg_scale, mode):
    st = pu.run_round_parity(name, mode=mode, K=6, cfg_scale=cfg_scale, seed=11, verbose=True)
    assert st["ties"] == 0 or st["ties"] < 6


def test_round_k1_and_relaxed():
    pu.run_round_parity("tiny", mode="fp32", K=1, cfg_scale=4.0, seed=5, verbose=True)
    pu.run_round_parity("tiny", mode="fp32", K=3, cfg_scale=1.5, seed=6, verbose=True)
