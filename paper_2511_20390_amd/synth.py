"""Seeded synthetic inputs shared by the oracle-side tests and the HIP path.

This module only draws random numbers and lays them out; it contains none of
the method's arithmetic (no schedule, no embedding, no network, no acceptance
rule).  Quantities the method derives (the sigma table of the diffusion
schedule) are passed in by the caller.  Everything is generated on the host
with NumPy's PCG64 from an explicit seed, so both sides see identical bytes.

Workload shapes follow the class-conditional DiT-XL/2 setting of the paper's
experiments (Sec. 4: ImageNet 256^2 / 512^2 latents, 1000 denoising steps,
guidance scale 4.0 in the high-uncertainty setting); the values are synthetic
stand-ins for the ImageNet latents, pretrained weights and trained drafter the
paper uses.
"""
from __future__ import annotations

import numpy as np

CONFIGS = {
    # latent 4x8x8, 16 tokens: the oracle finishes in well under a second
    "tiny": dict(in_ch=4, lat_h=8, lat_w=8, patch=2, hidden=64, depth=2, heads=4,
                 mlp_hidden=256, num_classes=10, learn_sigma=1, t_freq_dim=256),
    # a few tiles and ragged tails for every kernel, still seconds on the CPU
    "small": dict(in_ch=4, lat_h=16, lat_w=24, patch=2, hidden=144, depth=3, heads=2,
                  mlp_hidden=320, num_classes=10, learn_sigma=1, t_freq_dim=256),
    "xl2_256": dict(in_ch=4, lat_h=32, lat_w=32, patch=2, hidden=1152, depth=28, heads=16,
                    mlp_hidden=4608, num_classes=1000, learn_sigma=1, t_freq_dim=256),
    "xl2_512": dict(in_ch=4, lat_h=64, lat_w=64, patch=2, hidden=1152, depth=28, heads=16,
                    mlp_hidden=4608, num_classes=1000, learn_sigma=1, t_freq_dim=256),
}

# names of the large matrices that are stored as bf16 buffers in bf16 mode
BIG_MATRIX_SUFFIXES = ("ada_w", "qkv_w", "proj_w", "fc1_w", "fc2_w", "fin_ada_w", "fin_w", "fuse_w")


def dit_config(name: str, **over) -> dict:
    cfg = dict(CONFIGS[name])
    cfg.update(over)
    return cfg


def n_tokens(cfg: dict) -> int:
    return (cfg["lat_h"] // cfg["patch"]) * (cfg["lat_w"] // cfg["patch"])


def latent_dim(cfg: dict) -> int:
    return cfg["in_ch"] * cfg["lat_h"] * cfg["lat_w"]


def weight_spec(cfg: dict):
    """Ordered (name, shape) list; this order is the order of the pointer array
    handed to the library.  Matrices are [out, in] row-major."""
    D, F = cfg["hidden"], cfg["mlp_hidden"]
    pp = cfg["patch"] ** 2
    c_out = cfg["in_ch"] * (2 if cfg["learn_sigma"] else 1)
    spec = [("patch_w", (D, cfg["in_ch"] * pp)), ("patch_b", (D,)),
            ("t_w1", (D, cfg["t_freq_dim"])), ("t_b1", (D,)),
            ("t_w2", (D, D)), ("t_b2", (D,)),
            ("y_table", (cfg["num_classes"] + 1, D))]
    for l in range(cfg["depth"]):
        spec += [(f"blk{l}.ada_w", (6 * D, D)), (f"blk{l}.ada_b", (6 * D,)),
                 (f"blk{l}.qkv_w", (3 * D, D)), (f"blk{l}.qkv_b", (3 * D,)),
                 (f"blk{l}.proj_w", (D, D)), (f"blk{l}.proj_b", (D,)),
                 (f"blk{l}.fc1_w", (F, D)), (f"blk{l}.fc1_b", (F,)),
                 (f"blk{l}.fc2_w", (D, F)), (f"blk{l}.fc2_b", (D,))]
    spec += [("fin_ada_w", (2 * D, D)), ("fin_ada_b", (2 * D,)),
             ("fin_w", (pp * c_out, D)), ("fin_b", (pp * c_out,))]
    return spec


def drafter_weight_spec(cfg: dict, drafter_depth: int = 1):
    """Ordered (name, shape) list of the drafter's own weights (it shares the
    embedding layers with the target): fusion layer on [embedding | feature],
    `drafter_depth` blocks of the target's form, output projection of the form
    of the target's final layer.  About 32 M parameters at DiT-XL/2 width."""
    D, F = cfg["hidden"], cfg["mlp_hidden"]
    pp = cfg["patch"] ** 2
    c_out = cfg["in_ch"] * (2 if cfg["learn_sigma"] else 1)
    spec = [("fuse_w", (D, 2 * D)), ("fuse_b", (D,))]
    for l in range(drafter_depth):
        spec += [(f"blk{l}.ada_w", (6 * D, D)), (f"blk{l}.ada_b", (6 * D,)),
                 (f"blk{l}.qkv_w", (3 * D, D)), (f"blk{l}.qkv_b", (3 * D,)),
                 (f"blk{l}.proj_w", (D, D)), (f"blk{l}.proj_b", (D,)),
                 (f"blk{l}.fc1_w", (F, D)), (f"blk{l}.fc1_b", (F,)),
                 (f"blk{l}.fc2_w", (D, F)), (f"blk{l}.fc2_b", (D,))]
    spec += [("fin_ada_w", (2 * D, D)), ("fin_ada_b", (2 * D,)),
             ("fin_w", (pp * c_out, D)), ("fin_b", (pp * c_out,))]
    return spec


def make_drafter_weights(cfg: dict, drafter_depth: int = 1, seed: int = 1, std: float = 0.02,
                         bf16_values: bool = False) -> dict:
    """Random-init drafter weights ~ N(0, std^2) (a stand-in for the trained drafter)."""
    rng = np.random.default_rng(seed)
    w = {}
    for name, shape in drafter_weight_spec(cfg, drafter_depth):
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        w[name] = bf16_round(a) if bf16_values else a
    return w


def make_draft_inputs(cfg: dict, K: int, seed: int, cfg_scale: float, t0: int | None = None, T: int = 1000) -> dict:
    """Inputs of one drafting loop: reference state ~ N(0, I), a top-block feature per guidance
    branch ~ N(0, 1) (stand-in for the target's), consecutive timesteps, a label, standard normal draws."""
    rng = np.random.default_rng(seed)
    C, H, W = cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]
    dup = 2 if cfg_scale > 1.0 else 1
    x_a = rng.standard_normal((C, H, W), dtype=np.float32)
    f_a = rng.standard_normal((dup, n_tokens(cfg), cfg["hidden"]), dtype=np.float32)
    if t0 is None:
        t0 = int(rng.integers(K - 1, T))
    t = (t0 - np.arange(K)).astype(np.int32)
    y = int(rng.integers(0, cfg["num_classes"]))
    xi = rng.standard_normal((K, C * H * W), dtype=np.float32)
    return dict(x_a=x_a, f_a=f_a, t=t, y=y, xi=xi)


def is_big_matrix(name: str) -> bool:
    return name.endswith(BIG_MATRIX_SUFFIXES)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    rounded = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def make_weights(cfg: dict, seed: int = 0, std: float = 0.02, bf16_values: bool = False,
                 zero_adaln: bool = False) -> dict:
    """Random-init weights: every tensor (matrices, biases, embedding table,
    adaLN modulation) ~ N(0, std^2), fp32.  bf16_values rounds every value to a
    bf16-representable one (the buffers stay fp32 here).  zero_adaln sets the
    modulation matrices and biases of every block and of the final layer to
    zero (the adaLN-Zero initial state)."""
    rng = np.random.default_rng(seed)
    w = {}
    for name, shape in weight_spec(cfg):
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if zero_adaln and ("ada_w" in name or "ada_b" in name):
            a = np.zeros(shape, np.float32)
        if bf16_values:
            a = bf16_round(a)
        w[name] = a
    return w


def relaxation_profile(t: np.ndarray, T: int = 1000) -> np.ndarray:
    """Synthetic relaxation profile lambda_t in [0.25, 1]: with s the denoising
    progress (0 at t = T-1, 1 at t = 0) and g(s) = 1 + 3 s^2 a smooth increasing
    stand-in for the measured discrepancy curve, lambda = g(0) / g(s)."""
    s = 1.0 - np.asarray(t, np.float64) / (T - 1)
    return (1.0 / (1.0 + 3.0 * s * s)).astype(np.float32)


def make_round_inputs(cfg: dict, K: int, seed: int, sigma_table: np.ndarray,
                      draft_noise: float = 0.1, t0: int | None = None, T: int = 1000) -> dict:
    """One verification round: input state ~ N(0, I), K drafts = input +
    N(0, draft_noise^2) (K-1 of them are packed with the input, the last one is
    only verified), consecutive timesteps t0, t0-1, ..., t0-K+1 with t0 uniform
    in [K-1, T-1], a uniform class label, seeded uniforms, and draft means
    m^_k = x^_{k+1} - sigma_k z_k so that each draft is a sample of its proposal."""
    rng = np.random.default_rng(seed)
    C, H, W = cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]
    x_in = rng.standard_normal((C, H, W), dtype=np.float32)
    drafts = x_in[None] + np.float32(draft_noise) * rng.standard_normal((K, C, H, W), dtype=np.float32)
    if t0 is None:
        t0 = int(rng.integers(K - 1, T))
    t = (t0 - np.arange(K)).astype(np.int32)
    y = int(rng.integers(0, cfg["num_classes"]))
    u = rng.random(K, dtype=np.float32)
    sigma = np.asarray(sigma_table, np.float64)[t].astype(np.float32)
    z = rng.standard_normal((K, C, H, W), dtype=np.float32)
    m_draft = drafts - sigma.reshape(K, 1, 1, 1) * z
    x_states = np.concatenate([x_in[None], drafts[:K - 1]], axis=0)
    return dict(x_states=np.ascontiguousarray(x_states), x_last=np.ascontiguousarray(drafts[K - 1]),
                m_draft=np.ascontiguousarray(m_draft.reshape(K, -1)), t=t, y=y, u=u, sigma=sigma,
                lam=relaxation_profile(t, T))


def make_verify_inputs_diag(n_traj: int, K: int, d: int, delta: float, seed: int, sigma_table: np.ndarray,
                            spread: float = 0.4, T: int = 1000) -> dict:
    """Verification workload with one standard deviation per element: the step's sigma times a log-normal
    factor exp(spread * N(0, 1)) per element; draft means = target means + delta * sigma_elem * N(0, I);
    drafts = draft means + sigma_elem * N(0, I)."""
    rng = np.random.default_rng(seed)
    t = rng.integers(0, T, size=(n_traj, K))
    sigma = np.asarray(sigma_table, np.float64)[t].astype(np.float32)
    sigma_elem = (sigma[..., None] * np.exp(np.float32(spread) * rng.standard_normal((n_traj, K, d), dtype=np.float32)))
    sigma_elem = np.ascontiguousarray(sigma_elem.astype(np.float32))
    m_target = rng.standard_normal((n_traj, K, d), dtype=np.float32)
    m_draft = m_target + np.float32(delta) * sigma_elem * rng.standard_normal((n_traj, K, d), dtype=np.float32)
    x_draft = m_draft + sigma_elem * rng.standard_normal((n_traj, K, d), dtype=np.float32)
    u = rng.random((n_traj, K), dtype=np.float32)
    return dict(m_target=m_target, m_draft=np.ascontiguousarray(m_draft), x_draft=np.ascontiguousarray(x_draft),
                sigma_elem=sigma_elem, u=u, lam=relaxation_profile(t, T), t=t.astype(np.int32))


def make_verify_inputs(n_traj: int, K: int, d: int, delta: float, seed: int,
                       sigma_table: np.ndarray, T: int = 1000) -> dict:
    """Stand-alone verification workload: target means ~ N(0, I); sigma from the
    supplied table at uniformly drawn timesteps; draft means = target means +
    delta * sigma * N(0, I); drafts = draft means + sigma * N(0, I); seeded
    uniforms; lambda from the synthetic relaxation profile."""
    rng = np.random.default_rng(seed)
    t = rng.integers(0, T, size=(n_traj, K))
    sigma = np.asarray(sigma_table, np.float64)[t].astype(np.float32)
    m_target = rng.standard_normal((n_traj, K, d), dtype=np.float32)
    g = rng.standard_normal((n_traj, K, d), dtype=np.float32)
    m_draft = m_target + np.float32(delta) * sigma[..., None] * g
    z = rng.standard_normal((n_traj, K, d), dtype=np.float32)
    x_draft = m_draft + sigma[..., None] * z
    u = rng.random((n_traj, K), dtype=np.float32)
    return dict(m_target=m_target, m_draft=np.ascontiguousarray(m_draft),
                x_draft=np.ascontiguousarray(x_draft), sigma=sigma, u=u,
                lam=relaxation_profile(t, T), t=t.astype(np.int32))
