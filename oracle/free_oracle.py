"""Plain fp64 CPU oracle for FREE's parallel verification pass.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
cpu-baseline leg of the benchmark.  The product path never imports it and it
imports nothing from the product package.  NumPy only; every floating-point
quantity is float64.  No blocking, fusion or reordering: each function is the
definition written out so it can be checked against the paper by eye.

What it follows
---------------
* Verification of one draft: Alg. 2 (accept with probability
  min(1, q(x^)/p(x^)), reflect on rejection), with the likelihood ratio in the
  form of Eq. (qp) and the relaxed rule of Eq. (acc_relax).
* Sequential check of the K drafts of a round, stopping at the first
  rejection: Alg. 1, inner verification loop; Sec. 3.3.
* Noise prediction -> transition mean with the fixed posterior variance:
  Eq. (ddpm_update), App. C.
* The packed target forward: the paper only cites the class-conditional DiT;
  the architecture below (patchify, sinusoidal timestep + label embedding,
  adaLN-Zero blocks, final adaLN layer, unpatchify) is the public DiT design
  restated as formulas.  Conventions the paper does not fix are listed in the
  module-level constants and in the function docstrings.

Pins (see tests): closed-form acceptance rate of App. D, preservation of the
target marginal (App. B, unbiasedness), reflection invariants (Lemmas 1-2),
lambda=1 reduction and monotonicity (Sec. 3.4), the DDPM posterior identities
for the schedule, adaLN-Zero identity blocks, permutation/packing invariance,
and agreement with an independent implementation built from library routines.
The DiT forward has no published activations to compare against: beyond those
invariants and the library-routine cross-check it is "parity unpinned".

* Verification with one variance per element (App. C names fixed-variance
  schedules richer than one scalar per step; Sec. 3.3 only requires that draft
  and target share the covariance): Alg. 2 in whitened coordinates.  Pins: the
  scalar case, library log-densities with a diagonal covariance, equivalence
  with the scalar routine on whitened inputs, preservation of the target
  marginal and the closed-form acceptance rate at the whitened distance.

* The drafter and the drafting loop (Sec. 3.2, "Feature-Level Autoregressive
  Drafting"; Alg. 1, inner drafting loop): shared embedding -> FC layer fusing
  the embedding output with the propagated top-block feature -> DiT block(s)
  -> output projection -> noise estimate -> transition mean -> sample.  Pins:
  a drafter whose fusion passes the embedding through and whose block and
  output weights are the target's reproduces the (depth-limited) target, such
  a drafter is always accepted by the verification, the feature-only fusion
  ignores the latent, and the drafted chain equals its step-by-step
  composition.  Like the DiT forward it is otherwise "parity unpinned".
* The whole sampler (Alg. 1): plain target step, drafting, one packed target
  evaluation per round, sequential verification, advance.  Pins: with a drafter
  equal to the target it is plain sequential ancestral sampling (checked on a
  scalar chain and on the DiT), on a linear-Gaussian chain the distribution of
  the result has the target's closed-form mean, variance and kurtosis whatever
  the drafter proposes, and every step is taken exactly once.
* The relaxation profile (Sec. 3.4): self-speculative run with frozen-target
  drafting recording the noise-estimate deviation per checked step, monotone
  least-squares fit (pool adjacent violators), smoothing, inverse rescaled to
  (0, 1].  Pins: the fit against brute force and a library isotonic regression,
  the closed form of the frozen recurrence, exactness of frozen drafting for a
  state-independent network, monotonicity and range of the profile.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64

LN_EPS = 1e-6            # LayerNorm epsilon (no affine parameters, biased variance)
MAX_PERIOD = 10000.0     # base of both sinusoidal embeddings
TIE_WINDOW = 1e-4        # |lambda*l - log u| below this is flagged as a tie


# ----------------------------------------------------------------------------
# Diffusion schedule and eps -> mean  (Eq. ddpm_update; App. C)
# ----------------------------------------------------------------------------
def ddpm_schedule(T: int = 1000, beta_start: float = 1e-4, beta_end: float = 0.02) -> dict:
    """Linear-beta DDPM schedule, 0-indexed (index i is network timestep i).

    beta_i linear from beta_start to beta_end; alpha = 1 - beta;
    alphabar_i = prod_{j<=i} alpha_j with alphabar_{-1} = 1;
    posterior variance betatilde_i = beta_i (1 - alphabar_{i-1}) / (1 - alphabar_i);
    sigma_i = sqrt(betatilde_i) (App. C: the fixed variance is the posterior one).
    `sigma_clipped` replaces index 0 (where betatilde = 0) by index 1 so that a
    verification step never divides by zero.
    """
    i = np.arange(T, dtype=F64)
    beta = beta_start + (beta_end - beta_start) * i / (T - 1)
    alpha = 1.0 - beta
    alphabar = np.cumprod(alpha)
    alphabar_prev = np.concatenate([[1.0], alphabar[:-1]])
    beta_tilde = beta * (1.0 - alphabar_prev) / (1.0 - alphabar)
    sigma = np.sqrt(beta_tilde)
    sigma_clipped = sigma.copy()
    sigma_clipped[0] = sigma[1]
    return dict(T=T, beta=beta, alpha=alpha, alphabar=alphabar, alphabar_prev=alphabar_prev,
                beta_tilde=beta_tilde, sigma=sigma, sigma_clipped=sigma_clipped)


def sde_coefficients(stochasticity: float, T: int = 1000, beta_start: float = 1e-4, beta_end: float = 0.02):
    """One Euler step of the reverse family with stochasticity parameter e (Eq. mean_var_gamma) for the
    variance-preserving diffusion of the linear-beta schedule: forward drift f(x) = -beta x / 2, g^2 = beta,
    score s = -eps / sqrt(1 - alphabar).  m = x + [beta x / 2 + (1 + e^2)/2 beta s], sigma^2 = e^2 beta,
    i.e. m = coef_x x + coef_eps eps.  Returns (coef_x, coef_eps, sigma), each [T]."""
    beta = np.linspace(beta_start, beta_end, T, dtype=F64)
    alphabar = np.cumprod(1.0 - beta)
    e2 = float(stochasticity) ** 2
    return 1.0 + 0.5 * beta, -0.5 * (1.0 + e2) * beta / np.sqrt(1.0 - alphabar), float(stochasticity) * np.sqrt(beta)


def eps_to_mean(x: np.ndarray, eps: np.ndarray, i: int, sched: dict) -> np.ndarray:
    """Transition mean of Eq. (ddpm_update) without the noise term:
    m = (x - (1 - alpha_i) / sqrt(1 - alphabar_i) * eps) / sqrt(alpha_i)."""
    x = np.asarray(x, F64)
    eps = np.asarray(eps, F64)
    a = sched["alpha"][i]
    ab = sched["alphabar"][i]
    return (x - (1.0 - a) / math.sqrt(1.0 - ab) * eps) / math.sqrt(a)


def mean_coefficients(i, sched: dict):
    """(coef_x, coef_eps) with m = coef_x * x + coef_eps * eps, same formula."""
    a = sched["alpha"][i]
    ab = sched["alphabar"][i]
    return 1.0 / np.sqrt(a), -(1.0 - a) / (np.sqrt(1.0 - ab) * np.sqrt(a))


# ----------------------------------------------------------------------------
# Verification (Alg. 2, Eq. qp, Eq. acc_relax)
# ----------------------------------------------------------------------------
def log_ratio(m_hat, m, sigma: float, x_hat) -> float:
    """log of N(x^; m, s^2 I) / N(x^; m^, s^2 I) in the form of Eq. (qp):
    (m - m^)^T (x^ - mid) / s^2 with mid = (m + m^)/2."""
    m_hat = np.asarray(m_hat, F64).ravel()
    m = np.asarray(m, F64).ravel()
    x_hat = np.asarray(x_hat, F64).ravel()
    mid = 0.5 * (m + m_hat)
    return float(np.dot(m - m_hat, x_hat - mid) / (float(sigma) ** 2))


def reflect(m_hat, m, x_hat) -> np.ndarray:
    """Rejection branch of Alg. 2: e = (m^ - m)/||m^ - m||,
    x = m + (I - 2 e e^T)(x^ - m^)."""
    m_hat = np.asarray(m_hat, F64)
    m = np.asarray(m, F64)
    x_hat = np.asarray(x_hat, F64)
    diff = (m_hat - m).ravel()
    e = diff / math.sqrt(float(np.dot(diff, diff)))
    r = (x_hat - m_hat).ravel()
    out = m.ravel() + r - 2.0 * e * float(np.dot(e, r))
    return out.reshape(m.shape)


def verification(m_hat, m, sigma: float, x_hat, u: float, lam: float = 1.0):
    """Alg. 2 with the relaxed rule of Eq. (acc_relax); lam = 1 is the strict rule.

    Returns (x, accepted, l, tie) where l is the unscaled log-ratio of Eq. (qp).
    The test u <= min(1, exp(lam*l)) is taken in the log domain,
    log u <= min(0, lam*l), which is the same decision (log is monotone) and
    cannot overflow; u = 0 always accepts.  If m^ == m the ratio is one, the
    draft is accepted whatever u is and the (undefined) direction e is never
    formed.  `tie` flags decisions within TIE_WINDOW of the threshold.
    """
    m_hat = np.asarray(m_hat, F64)
    m = np.asarray(m, F64)
    x_hat = np.asarray(x_hat, F64)
    diff = (m_hat - m).ravel()
    s2 = float(np.dot(diff, diff))
    l = log_ratio(m_hat, m, sigma, x_hat)
    if s2 == 0.0:
        return x_hat.copy(), True, l, False
    thr = min(0.0, float(lam) * l)
    if u <= 0.0:
        return x_hat.copy(), True, l, False
    logu = math.log(u)
    accepted = logu <= thr
    tie = abs(float(lam) * l - logu) < TIE_WINDOW
    if accepted:
        return x_hat.copy(), True, l, tie
    return reflect(m_hat, m, x_hat), False, l, tie


def spec_verify(m_target, m_draft, x_draft, sigma, u, lam=None) -> dict:
    """The K drafts of each trajectory checked in order (Alg. 1, verification loop).

    m_target, m_draft, x_draft: [n_traj, K, d]; sigma, u, lam: [n_traj, K]
    (lam None => strict rule everywhere).  For every (trajectory, draft) the
    log-ratio and the stand-alone decision are recorded; n_accept is the number
    of drafts accepted before the first rejection, and x_out holds the
    reflected sample of that first rejected draft (zeros where nothing was
    rejected: has_reflect marks the rows that were written).
    """
    m_target = np.asarray(m_target, F64)
    m_draft = np.asarray(m_draft, F64)
    x_draft = np.asarray(x_draft, F64)
    n_traj, K, d = m_target.shape
    sigma = np.asarray(sigma, F64).reshape(n_traj, K)
    u = np.asarray(u, F64).reshape(n_traj, K)
    lam = np.ones((n_traj, K), F64) if lam is None else np.asarray(lam, F64).reshape(n_traj, K)
    lr = np.zeros((n_traj, K), F64)
    acc = np.zeros((n_traj, K), np.uint8)
    tie = np.zeros((n_traj, K), bool)
    n_accept = np.zeros(n_traj, np.int32)
    x_out = np.zeros((n_traj, d), F64)
    has_reflect = np.zeros(n_traj, bool)
    for n in range(n_traj):
        first_reject = K
        for k in range(K):
            x, ok, l, tk = verification(m_draft[n, k], m_target[n, k], sigma[n, k],
                                        x_draft[n, k], u[n, k], lam[n, k])
            lr[n, k] = l
            acc[n, k] = 1 if ok else 0
            tie[n, k] = tk
            if not ok and first_reject == K:
                first_reject = k
                x_out[n] = x
                has_reflect[n] = True
        n_accept[n] = first_reject
    return dict(log_ratio=lr, accept=acc, n_accept=n_accept, x_out=x_out,
                has_reflect=has_reflect, tie=tie)


# ----------------------------------------------------------------------------
# Verification with one variance per element (App. C: fixed-variance schedules richer than a scalar per
# step; Sec. 3.3 only needs draft and target to share the covariance).  Both transitions are
# N(mean, diag(s^2)) with the same vector s: in the whitened coordinates z = (x - c) / s they are isotropic
# with unit variance, so Alg. 2 applies there unchanged and the result is mapped back.
# ----------------------------------------------------------------------------
def log_ratio_diag(m_hat, m, sigma_vec, x_hat) -> float:
    """log of N(x^; m, diag(s^2)) / N(x^; m^, diag(s^2)) = sum_i (m_i - m^_i)(x^_i - mid_i) / s_i^2
    (Eq. qp with the per-element variance inside the sum)."""
    m_hat = np.asarray(m_hat, F64).ravel()
    m = np.asarray(m, F64).ravel()
    x_hat = np.asarray(x_hat, F64).ravel()
    s = np.asarray(sigma_vec, F64).ravel()
    mid = 0.5 * (m + m_hat)
    return float(np.sum((m - m_hat) * (x_hat - mid) / (s * s)))


def reflect_diag(m_hat, m, sigma_vec, x_hat) -> np.ndarray:
    """Rejection branch of Alg. 2 in the whitened coordinates: e = ((m^ - m)/s) / ||(m^ - m)/s||,
    x = m + s * (I - 2 e e^T) ((x^ - m^)/s)."""
    m_hat = np.asarray(m_hat, F64)
    m = np.asarray(m, F64)
    x_hat = np.asarray(x_hat, F64)
    s = np.asarray(sigma_vec, F64).ravel()
    dw = (m_hat - m).ravel() / s
    e = dw / math.sqrt(float(np.dot(dw, dw)))
    z = (x_hat - m_hat).ravel() / s
    out = m.ravel() + s * (z - 2.0 * e * float(np.dot(e, z)))
    return out.reshape(m.shape)


def verification_diag(m_hat, m, sigma_vec, x_hat, u: float, lam: float = 1.0):
    """Alg. 2 (with the relaxed rule of Eq. acc_relax) for transitions that share a diagonal covariance.
    Same conventions as `verification`: decision in the log domain, u = 0 and m^ == m accept."""
    m_hat = np.asarray(m_hat, F64)
    m = np.asarray(m, F64)
    x_hat = np.asarray(x_hat, F64)
    l = log_ratio_diag(m_hat, m, sigma_vec, x_hat)
    if not np.any(m_hat != m) or u <= 0.0:
        return x_hat.copy(), True, l, False
    logu = math.log(u)
    accepted = logu <= min(0.0, float(lam) * l)
    tie = abs(float(lam) * l - logu) < TIE_WINDOW
    if accepted:
        return x_hat.copy(), True, l, tie
    return reflect_diag(m_hat, m, sigma_vec, x_hat), False, l, tie


def spec_verify_diag(m_target, m_draft, x_draft, sigma_elem, u, lam=None) -> dict:
    """spec_verify with sigma_elem [n_traj, K, d]: one standard deviation per element of every draft."""
    m_target = np.asarray(m_target, F64)
    n_traj, K, d = m_target.shape
    m_draft = np.asarray(m_draft, F64)
    x_draft = np.asarray(x_draft, F64)
    sigma_elem = np.asarray(sigma_elem, F64).reshape(n_traj, K, d)
    u = np.asarray(u, F64).reshape(n_traj, K)
    lam = np.ones((n_traj, K), F64) if lam is None else np.asarray(lam, F64).reshape(n_traj, K)
    lr = np.zeros((n_traj, K), F64)
    acc = np.zeros((n_traj, K), np.uint8)
    tie = np.zeros((n_traj, K), bool)
    n_accept = np.full(n_traj, K, np.int32)
    x_out = np.zeros((n_traj, d), F64)
    has_reflect = np.zeros(n_traj, bool)
    for n in range(n_traj):
        for k in range(K):
            x, ok, l, tk = verification_diag(m_draft[n, k], m_target[n, k], sigma_elem[n, k], x_draft[n, k],
                                             u[n, k], lam[n, k])
            lr[n, k], acc[n, k], tie[n, k] = l, 1 if ok else 0, tk
            if not ok and not has_reflect[n]:
                n_accept[n] = k
                x_out[n] = x
                has_reflect[n] = True
    return dict(log_ratio=lr, accept=acc, n_accept=n_accept, x_out=x_out, has_reflect=has_reflect, tie=tie)


# ----------------------------------------------------------------------------
# DiT forward (public DiT architecture restated; the paper only cites it)
# ----------------------------------------------------------------------------
def silu(v):
    return v / (1.0 + np.exp(-v))


def gelu_tanh(v):
    """tanh form of GELU: 0.5 v (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3)))."""
    return 0.5 * v * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))


def layer_norm(v):
    """LayerNorm over the last axis, no affine, biased variance, eps = LN_EPS."""
    mu = v.mean(axis=-1, keepdims=True)
    var = ((v - mu) ** 2).mean(axis=-1, keepdims=True)
    return (v - mu) / np.sqrt(var + LN_EPS)


def linear(v, w, b):
    """y = v W^T + b with W stored [out, in]."""
    return v @ np.asarray(w, F64).T + np.asarray(b, F64)


def timestep_embedding(t, dim: int) -> np.ndarray:
    """[cos(t w_j) | sin(t w_j)], w_j = MAX_PERIOD^(-j/(dim/2)), j < dim/2."""
    half = dim // 2
    w = np.exp(-math.log(MAX_PERIOD) * np.arange(half, dtype=F64) / half)
    ang = np.asarray(t, F64).reshape(-1, 1) * w.reshape(1, -1)
    return np.concatenate([np.cos(ang), np.sin(ang)], axis=1)


def pos_embed_2d(gh: int, gw: int, dim: int) -> np.ndarray:
    """Fixed 2-D sin-cos table [gh*gw, dim] for token (i, j), row-major:
    [sin(j w) | cos(j w) | sin(i w) | cos(i w)], w_k = MAX_PERIOD^(-k/(dim/4))."""
    q = dim // 4
    w = 1.0 / MAX_PERIOD ** (np.arange(q, dtype=F64) / q)
    ii, jj = np.meshgrid(np.arange(gh, dtype=F64), np.arange(gw, dtype=F64), indexing="ij")
    aj = jj.reshape(-1, 1) * w
    ai = ii.reshape(-1, 1) * w
    return np.concatenate([np.sin(aj), np.cos(aj), np.sin(ai), np.cos(ai)], axis=1)


def patchify(x, p: int) -> np.ndarray:
    """[B, C, H, W] -> [B, (H/p)(W/p), C p p]; tokens row-major over the patch
    grid, each patch flattened over (c, ph, pw)."""
    B, C, H, W = x.shape
    gh, gw = H // p, W // p
    v = x.reshape(B, C, gh, p, gw, p)
    v = v.transpose(0, 2, 4, 1, 3, 5)          # B, gh, gw, C, ph, pw
    return v.reshape(B, gh * gw, C * p * p)


def unpatchify(tok, p: int, c_out: int, gh: int, gw: int) -> np.ndarray:
    """[B, gh gw, p p c_out] with per-token order (ph, pw, c) -> [B, c_out, gh p, gw p]."""
    B = tok.shape[0]
    v = tok.reshape(B, gh, gw, p, p, c_out)
    v = v.transpose(0, 5, 1, 3, 2, 4)          # B, c, gh, ph, gw, pw
    return v.reshape(B, c_out, gh * p, gw * p)


def conditioning(w: dict, cfg: dict, t, y) -> np.ndarray:
    """c = MLP(timestep_embedding(t)) + label_table[y]; returns c (before SiLU)."""
    temb = timestep_embedding(t, cfg["t_freq_dim"])
    h = silu(linear(temb, w["t_w1"], w["t_b1"]))
    h = linear(h, w["t_w2"], w["t_b2"])
    return h + np.asarray(w["y_table"], F64)[np.asarray(y, np.int64)]


def attention(q, k, v) -> np.ndarray:
    """softmax(q k^T / sqrt(d_h)) v for one head; q, k, v: [N, d_h]."""
    s = (q @ k.T) / math.sqrt(q.shape[-1])
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return p @ v


def self_attention(xn, wqkv, bqkv, wproj, bproj, heads: int) -> np.ndarray:
    """Multi-head self-attention of one sample, xn: [N, D].  QKV rows are
    ordered [q | k | v], each split into `heads` consecutive groups of d_h."""
    N, D = xn.shape
    dh = D // heads
    qkv = linear(xn, wqkv, bqkv)
    q, k, v = qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:]
    out = np.empty((N, D), F64)
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        out[:, sl] = attention(q[:, sl], k[:, sl], v[:, sl])
    return linear(out, wproj, bproj)


def dit_block(xb, sc, w: dict, l: int, heads: int) -> np.ndarray:
    """One adaLN-Zero block on one sample: xb [N, D], sc = SiLU(c) [D]."""
    D = xb.shape[1]
    mod = linear(sc, w[f"blk{l}.ada_w"], w[f"blk{l}.ada_b"])
    sh1, sc1, g1, sh2, sc2, g2 = (mod[i * D:(i + 1) * D] for i in range(6))
    a = self_attention(layer_norm(xb) * (1.0 + sc1) + sh1,
                       w[f"blk{l}.qkv_w"], w[f"blk{l}.qkv_b"],
                       w[f"blk{l}.proj_w"], w[f"blk{l}.proj_b"], heads)
    xb = xb + g1 * a
    hmid = gelu_tanh(linear(layer_norm(xb) * (1.0 + sc2) + sh2,
                            w[f"blk{l}.fc1_w"], w[f"blk{l}.fc1_b"]))
    xb = xb + g2 * linear(hmid, w[f"blk{l}.fc2_w"], w[f"blk{l}.fc2_b"])
    return xb


def dit_forward(w: dict, cfg: dict, x, t, y, samples=None):
    """Forward of the packed batch: every state has its own timestep and label.

    x: [B, C, H, W]; t, y: [B].  Returns (out [B, 2C, H, W], top_feat [B, N, D]):
    `out` holds the noise prediction in channels [0, C) and the (unused, App. C)
    learned-variance channels in [C, 2C); `top_feat` is the output of the last
    block (the paper's feature f).  `samples` restricts the work to a subset of
    the batch rows (each row is independent of the others).
    """
    x = np.asarray(x, F64)
    B, C, H, W = x.shape
    p, D, depth, heads = cfg["patch"], cfg["hidden"], cfg["depth"], cfg["heads"]
    gh, gw = H // p, W // p
    rows = list(range(B)) if samples is None else list(samples)
    t = np.asarray(t)
    y = np.asarray(y)
    c = conditioning(w, cfg, t[rows], y[rows])
    sc = silu(c)
    tok = linear(patchify(x[rows], p), w["patch_w"], w["patch_b"]) + pos_embed_2d(gh, gw, D)
    c_out = 2 * C if cfg.get("learn_sigma", 1) else C
    out_tok = np.empty((len(rows), gh * gw, p * p * c_out), F64)
    feat = np.empty((len(rows), gh * gw, D), F64)
    for r in range(len(rows)):
        xb = tok[r]
        for l in range(depth):
            xb = dit_block(xb, sc[r], w, l, heads)
        feat[r] = xb
        mod = linear(sc[r], w["fin_ada_w"], w["fin_ada_b"])
        sh, scl = mod[:D], mod[D:]
        out_tok[r] = linear(layer_norm(xb) * (1.0 + scl) + sh, w["fin_w"], w["fin_b"])
    return unpatchify(out_tok, p, c_out, gh, gw), feat


def cfg_combine(eps_cond, eps_null, scale: float) -> np.ndarray:
    """Classifier-free guidance: eps = eps_null + s (eps_cond - eps_null)."""
    eps_cond = np.asarray(eps_cond, F64)
    eps_null = np.asarray(eps_null, F64)
    return eps_null + float(scale) * (eps_cond - eps_null)


def round_means(w: dict, cfg: dict, x_states, t, y: int, cfg_scale: float, coef_x, coef_eps):
    """Target means of one round: packed forward on the K states (twice the
    batch, second half with the null label, when cfg_scale > 1), guidance on
    the noise channels, then m_k = coef_x[k] x_k + coef_eps[k] eps_k."""
    x_states = np.asarray(x_states, F64)
    K, C = x_states.shape[0], x_states.shape[1]
    t = np.asarray(t)
    if cfg_scale > 1.0:
        xx = np.concatenate([x_states, x_states], axis=0)
        tt = np.concatenate([t, t])
        yy = np.concatenate([np.full(K, y), np.full(K, cfg["num_classes"])])
        out, _ = dit_forward(w, cfg, xx, tt, yy)
        eps = cfg_combine(out[:K, :C], out[K:, :C], cfg_scale)
    else:
        out, _ = dit_forward(w, cfg, x_states, t, np.full(K, y))
        eps = out[:, :C]
    cx = np.asarray(coef_x, F64).reshape(K, 1, 1, 1)
    ce = np.asarray(coef_eps, F64).reshape(K, 1, 1, 1)
    return cx * x_states + ce * eps


def spec_round(w: dict, cfg: dict, x_states, x_last, m_draft, t, y: int, cfg_scale: float,
               coef_x, coef_eps, sigma, u, lam=None) -> dict:
    """One verification round (Alg. 1: packed target forward + verification loop).

    x_states [K, C, H, W] = (x_a, x^_{a+1}, ..., x^_{a+K-1}) are run through the
    target; draft k+1 (x_states[k+1], and x_last for k = K-1) is verified against
    (m_draft[k], m_k, sigma[k])."""
    x_states = np.asarray(x_states, F64)
    K = x_states.shape[0]
    m = round_means(w, cfg, x_states, t, y, cfg_scale, coef_x, coef_eps)
    xd = np.concatenate([x_states[1:], np.asarray(x_last, F64)[None]], axis=0)
    res = spec_verify(m.reshape(1, K, -1), np.asarray(m_draft, F64).reshape(1, K, -1),
                      xd.reshape(1, K, -1), np.asarray(sigma).reshape(1, K),
                      np.asarray(u).reshape(1, K),
                      None if lam is None else np.asarray(lam).reshape(1, K))
    res["m_target"] = m.reshape(K, -1)
    return res


# ----------------------------------------------------------------------------
# Drafter and autoregressive drafting (Sec. 3.2; Alg. 1, drafting loop)
# ----------------------------------------------------------------------------
def drafter_forward(wd: dict, w: dict, cfg: dict, x, f_prev, t, y):
    """One evaluation of the drafter p(. | x^_{t-1}, f_{t-1}) (Sec. 3.2).

    The drafter reuses the target's embedding layers (patch embedding with the
    positional table, timestep and label embedding: weights `w`), fuses the
    embedded latent with the propagated feature by one fully connected layer on
    their concatenation [embedding | feature] (`wd["fuse_w"]` is [D, 2D]), runs
    its own DiT block(s) (`wd["blk{l}.*"]`, `cfg["drafter_depth"]` of them, one
    in the paper's main setting) and a small output projection of the same form
    as the target's final layer (`wd["fin_*"]`).

    x [B, C, H, W], f_prev [B, N, D], t, y [B].  Returns (out [B, c_out, H, W],
    f [B, N, D]): the noise estimate sits in channels [0, C) of `out`, `f` (the
    output of the last drafter block) is the predicted next top-block feature.
    """
    x = np.asarray(x, F64)
    B, C, H, W = x.shape
    p, D, heads = cfg["patch"], cfg["hidden"], cfg["heads"]
    ddepth = cfg.get("drafter_depth", 1)
    gh, gw = H // p, W // p
    sc = silu(conditioning(w, cfg, np.asarray(t), np.asarray(y)))
    emb = linear(patchify(x, p), w["patch_w"], w["patch_b"]) + pos_embed_2d(gh, gw, D)
    c_out = 2 * C if cfg.get("learn_sigma", 1) else C
    out_tok = np.empty((B, gh * gw, p * p * c_out), F64)
    feat = np.empty((B, gh * gw, D), F64)
    for r in range(B):
        z = linear(np.concatenate([emb[r], np.asarray(f_prev, F64)[r]], axis=1), wd["fuse_w"], wd["fuse_b"])
        for l in range(ddepth):
            z = dit_block(z, sc[r], wd, l, heads)
        feat[r] = z
        mod = linear(sc[r], wd["fin_ada_w"], wd["fin_ada_b"])
        out_tok[r] = linear(layer_norm(z) * (1.0 + mod[D:]) + mod[:D], wd["fin_w"], wd["fin_b"])
    return unpatchify(out_tok, p, c_out, gh, gw), feat


def draft_steps(wd: dict, w: dict, cfg: dict, x_a, f_a, t, y: int, cfg_scale: float,
                coef_x, coef_eps, sigma, xi) -> dict:
    """The drafting loop of Alg. 1 for one trajectory.

    Starting from the reference state x_a and the target's top-block feature
    f_a, step k = 0..K-1 evaluates the drafter on (x^_k, f_{k-1}) at timestep
    t[k] (x^_0 = x_a, f_{-1} = f_a), turns its noise estimate into the draft
    mean m^_k = coef_x[k] x^_k + coef_eps[k] eps^_k and draws the next draft
    x^_{k+1} = m^_k + sigma[k] xi[k] (xi: the standard normal draws, an input).
    With guidance (cfg_scale > 1) the drafter runs on the label and on the null
    label, each branch carrying its own feature (f_a is [2, N, D]: label branch
    first), and the two noise estimates are combined as in the target.

    Returns x_states [K, C, H, W] = (x_a, x^_1 .. x^_{K-1}), x_last = x^_K,
    m_draft [K, d] and the final feature(s): exactly the inputs of spec_round.
    """
    x_a = np.asarray(x_a, F64)
    C = x_a.shape[0]
    K = len(t)
    dup = 2 if cfg_scale > 1.0 else 1
    f = np.asarray(f_a, F64).reshape((dup,) + np.asarray(f_a).shape[-2:])
    yy = np.array([y, cfg["num_classes"]][:dup])
    xs = [x_a]
    m_draft = []
    for k in range(K):
        xk = xs[-1]
        out, f = drafter_forward(wd, w, cfg, np.repeat(xk[None], dup, axis=0), f, np.full(dup, t[k]), yy)
        eps = cfg_combine(out[0, :C], out[1, :C], cfg_scale) if dup == 2 else out[0, :C]
        m = float(coef_x[k]) * xk + float(coef_eps[k]) * eps
        m_draft.append(m.reshape(-1))
        xs.append(m + float(sigma[k]) * np.asarray(xi, F64)[k].reshape(m.shape))
    return dict(x_states=np.stack(xs[:K]), x_last=xs[K], m_draft=np.stack(m_draft), f_last=f)


# ----------------------------------------------------------------------------
# The whole sampler (Alg. 1): target step, drafting, packed verification, advance
# ----------------------------------------------------------------------------
def speculative_loop(x0, S: int, n_spec: int, L: int, sigma, xi, u, lam, target_means, draft_mean, on_verify=None):
    """Alg. 1 around two callables, so that the control flow can be checked on models with a known answer.

    Steps are indexed i = 0..S-1: step i takes the state x_i and produces x_{i+1}; x_S is returned.
      target_means(states, i0) -> (means, feats): the target's transition means of `states` (a list of
          latents sitting at steps i0, i0+1, ...) and one opaque feature per state;
      draft_mean(x, feat, i)   -> (mean, feat'): the drafter on (x, feature of the previous evaluation).
    Reading of Alg. 1 used here (the listing's `a <- k` would re-draw an already verified state):
      * a plain target step x_{i+1} = m_i + sigma_i xi_i is taken when no feature exists yet (i = 0) and for
        the steps i >= n_spec that cannot be speculated (sigma = 0: the last, noise-free step);
      * otherwise one round drafts K = min(L, n_spec - i) steps from (x_i, feature), draft j being
        x^_{i+j+1} = m^_{i+j} + sigma_{i+j} xi_{i+j}, runs ONE packed target evaluation on
        (x_i, x^_{i+1}, .., x^_{i+K-1}) and verifies draft j against (m^_{i+j}, m_{i+j}, sigma_{i+j}, u_{i+j});
      * with n drafts accepted the sampler advances to x_{i+n} = x^_{i+n} if n = K, else to the reflected
        x_{i+n+1}; the feature handed to the next round is the target's feature of the packed state that
        produced the transition just taken (index K-1, or n).  Every round therefore costs one target call.
    `on_verify(i, m_hat, m, accepted)` is called for every draft that is checked (step index i).
    Returns (x_S, stats) with stats = dict(target_calls, rounds, accepted, drafter_steps, n_accept=[...]).
    """
    x = np.asarray(x0, F64)
    d = x.size
    sigma = np.asarray(sigma, F64)
    xi = np.asarray(xi, F64).reshape(S, d)
    u = np.asarray(u, F64)
    lam = np.ones(S, F64) if lam is None else np.asarray(lam, F64)
    stats = dict(target_calls=0, rounds=0, accepted=0, drafter_steps=0, n_accept=[])
    feat = None
    i = 0
    while i < S:
        if feat is None or i >= n_spec:
            means, feats = target_means([x], i)
            stats["target_calls"] += 1
            x = np.asarray(means[0], F64) + sigma[i] * xi[i].reshape(x.shape)
            feat = feats[0]
            i += 1
            continue
        K = min(L, n_spec - i)
        states, m_hat, f = [x], [], feat
        for j in range(K):
            m, f = draft_mean(states[-1], f, i + j)
            m_hat.append(np.asarray(m, F64))
            states.append(m_hat[-1] + sigma[i + j] * xi[i + j].reshape(x.shape))
        stats["drafter_steps"] += K
        means, feats = target_means(states[:K], i)
        stats["target_calls"] += 1
        stats["rounds"] += 1
        n = K
        for j in range(K):
            xr, ok, _, _ = verification(m_hat[j].reshape(-1), np.asarray(means[j], F64).reshape(-1), sigma[i + j],
                                        states[j + 1].reshape(-1), u[i + j], lam[i + j])
            if on_verify is not None:
                on_verify(i + j, m_hat[j], np.asarray(means[j], F64), bool(ok))
            if not ok:
                n = j
                x = xr.reshape(x.shape)
                break
        stats["accepted"] += n
        stats["n_accept"].append(n)
        if n == K:
            x, feat, i = states[K], feats[K - 1], i + K
        else:
            feat, i = feats[n], i + n + 1
    return x, stats


def free_sample(wd: dict, w: dict, cfg: dict, x0, y: int, cfg_scale: float, tmap, coef_x, coef_eps, sigma,
                n_spec: int, L: int, xi, u, lam=None):
    """Alg. 1 with the DiT target and the feature-level drafter: `tmap[i]` is the network timestep of
    step i, (coef_x, coef_eps, sigma)[i] its transition coefficients (Eq. ddpm_update)."""
    C = np.asarray(x0).shape[0]
    dup = 2 if cfg_scale > 1.0 else 1
    yy = np.array([y, cfg["num_classes"]][:dup])

    def guided(out, K):
        return cfg_combine(out[:K, :C], out[K:, :C], cfg_scale) if dup == 2 else out[:, :C]

    def target_means(states, i0):
        K = len(states)
        xs = np.stack(states)
        t = np.asarray([tmap[i0 + j] for j in range(K)])
        out, feat = dit_forward(w, cfg, np.concatenate([xs] * dup), np.concatenate([t] * dup), np.repeat(yy, K))
        eps = guided(out, K)
        means = [float(coef_x[i0 + j]) * xs[j] + float(coef_eps[i0 + j]) * eps[j] for j in range(K)]
        feats = [np.stack([feat[b * K + j] for b in range(dup)]) for j in range(K)]
        return means, feats

    def draft_mean(x, f, i):
        out, f2 = drafter_forward(wd, w, cfg, np.stack([x] * dup), f, np.full(dup, tmap[i]), yy)
        eps = guided(out, 1)[0]
        return float(coef_x[i]) * np.asarray(x, F64) + float(coef_eps[i]) * eps, f2

    S = len(tmap)
    return speculative_loop(x0, S, n_spec, L, sigma, xi, u, lam, target_means, draft_mean)


# ----------------------------------------------------------------------------
# Relaxation profile (Sec. 3.4): offline self-speculative run, monotone fit, inverse rescaled to [0, 1]
# ----------------------------------------------------------------------------
def frozen_draft_steps(x_a, eps_frozen, coef_x, coef_eps, sigma, xi) -> dict:
    """Frozen-target drafting (Sec. 2: several future steps approximated by reusing a single noise estimate
    of the target): m^_k = coef_x[k] x^_k + coef_eps[k] eps_frozen, x^_{k+1} = m^_k + sigma[k] xi[k]."""
    x = np.asarray(x_a, F64)
    e = np.asarray(eps_frozen, F64).reshape(x.shape)
    K = len(sigma)
    xs, ms = [x], []
    for k in range(K):
        m = float(coef_x[k]) * xs[-1] + float(coef_eps[k]) * e
        ms.append(m.reshape(-1))
        xs.append(m + float(sigma[k]) * np.asarray(xi, F64)[k].reshape(x.shape))
    return dict(x_states=np.stack(xs[:K]), x_last=xs[K], m_draft=np.stack(ms))


def self_speculative_run(w: dict, cfg: dict, x0, y: int, cfg_scale: float, tmap, coef_x, coef_eps, sigma,
                         n_spec: int, L: int, xi, u, lam=None):
    """The offline run of Sec. 3.4: the target DiT both proposes (frozen-target drafting: the guided noise
    estimate of its latest evaluation is reused for the next K steps) and verifies (Alg. 2).  For every
    checked draft at step i it records eps_delta[i] = || eps_pred - eps_ref ||_2 (the reused estimate
    against the target's own at that state) and whether the draft passed; steps that were never checked
    (plain target steps, drafts after a rejection) hold NaN / -1.
    Returns (x_S, stats, eps_delta [S], accepted [S])."""
    C = np.asarray(x0).shape[0]
    S = len(tmap)
    dup = 2 if cfg_scale > 1.0 else 1
    yy = np.array([y, cfg["num_classes"]][:dup])
    eps_delta = np.full(S, np.nan)
    accepted = np.full(S, -1, np.int8)

    def target_means(states, i0):
        K = len(states)
        xs = np.stack(states)
        t = np.asarray([tmap[i0 + j] for j in range(K)])
        out, _ = dit_forward(w, cfg, np.concatenate([xs] * dup), np.concatenate([t] * dup), np.repeat(yy, K))
        eps = cfg_combine(out[:K, :C], out[K:, :C], cfg_scale) if dup == 2 else out[:, :C]
        means = [float(coef_x[i0 + j]) * xs[j] + float(coef_eps[i0 + j]) * eps[j] for j in range(K)]
        return means, [eps[j] for j in range(K)]          # the "feature" handed on is the noise estimate

    def draft_mean(x, eps_frozen, i):
        return float(coef_x[i]) * np.asarray(x, F64) + float(coef_eps[i]) * eps_frozen, eps_frozen

    def on_verify(i, m_hat, m, ok):
        eps_delta[i] = np.linalg.norm((m_hat - m).ravel()) / abs(float(coef_eps[i]))
        accepted[i] = 1 if ok else 0

    x, stats = speculative_loop(x0, S, n_spec, L, sigma, xi, u, lam, target_means, draft_mean, on_verify)
    return x, stats, eps_delta, accepted


def monotone_fit(v) -> np.ndarray:
    """Least-squares non-decreasing fit of a sequence (pool adjacent violators); NaN entries carry no weight
    and take the value of the fit at their position."""
    v = np.asarray(v, F64)
    ok = ~np.isnan(v)
    if not ok.any():
        raise ValueError("no measured value")
    blocks = []                                   # [sum, weight, length]
    for val, has in zip(v, ok):
        blocks.append([val if has else 0.0, 1.0 if has else 0.0, 1])
        while len(blocks) > 1:
            a, b = blocks[-2], blocks[-1]
            if a[1] == 0.0 or b[1] == 0.0 or a[0] / a[1] > b[0] / b[1]:
                blocks[-2:] = [[a[0] + b[0], a[1] + b[1], a[2] + b[2]]]
            else:
                break
    out = np.concatenate([np.full(n, s_ / w_) for s_, w_, n in blocks])
    return out


def relaxation_profile_from_deltas(eps_delta, window: int = 1) -> np.ndarray:
    """lambda_i from the measured deviations (Sec. 3.4): a monotonically increasing curve g fitted to
    eps_delta over the denoising steps (isotonic least squares, then a centred moving average of odd width
    `window` with the ends held, which keeps it monotone and makes it smooth), inverted and rescaled to
    (0, 1]: lambda_i = g_0 / g_i, so the rule is strict (lambda = 1) where the uncertainty is lowest and
    relaxes as it grows."""
    g = monotone_fit(eps_delta)
    if window > 1:
        if window % 2 == 0:
            raise ValueError("window must be odd")
        h = window // 2
        gp = np.concatenate([np.full(h, g[0]), g, np.full(h, g[-1])])
        g = np.convolve(gp, np.full(window, 1.0 / window), mode="valid")
    g = np.maximum(g, 1e-300)
    return g[0] / g
