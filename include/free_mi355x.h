/*
 * free_mi355x.h - C ABI of the MI355X (gfx950) implementation of FREE's
 * parallel verification pass: the packed target forward of Alg. 1 ("compute
 * means ... in parallel") followed by the sequential verification loop of
 * Alg. 1 with the per-draft test of Alg. 2.
 *
 * Conventions
 * -----------
 *  - Every entry point returns an int32_t status (FREE_OK or a negative
 *    FREE_ERR_*).  Nothing throws, aborts or prints.
 *  - Unless a parameter is marked [host], tensor pointers are DEVICE pointers
 *    owned by the caller.  The hot-path calls (dit_forward_packed,
 *    spec_verify, spec_round) never allocate or free: scratch memory comes
 *    from a caller-provided device workspace whose size is given by the
 *    *_workspace_bytes functions.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Hot-path calls only enqueue work and return: none of them waits for the
 *    device, times itself or reads device memory on the host.  Outputs are valid
 *    after the caller synchronises the stream.  Calls that share a workspace
 *    must be ordered on one stream.
 *  - Argument checks are host-side (null pointers, shapes).  Values that live
 *    in device memory (timesteps, labels, sigma, u, lambda) are NOT range
 *    checked: a timestep is any int, a label must lie in [0, num_classes]
 *    (num_classes = the null label), sigma must be > 0, u in [0, 1],
 *    lambda in [0, 1]; violating that is the caller's error.
 *  - Latents are [B, C, H, W] fp32, contiguous (the paper's x in R^d with
 *    d = C*H*W).  Per-draft scalars are [n_traj, K] fp32.
 */
#ifndef FREE_MI355X_H
#define FREE_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FREE_OK              0
#define FREE_ERR_NULL       -1   /* a required pointer is NULL */
#define FREE_ERR_SHAPE      -2   /* inconsistent or unsupported sizes */
#define FREE_ERR_RANGE      -3   /* a host-side scalar is out of range */
#define FREE_ERR_DTYPE      -4   /* unknown compute mode */
#define FREE_ERR_WORKSPACE  -5   /* workspace missing, misaligned or too small */
#define FREE_ERR_HIP        -6   /* HIP runtime error; see free_last_hip_error */
#define FREE_ERR_LIMIT      -7   /* problem larger than a fixed built-in limit */

#define FREE_FP32 0   /* fp32 weights and activations, fp32 accumulation */
#define FREE_BF16 1   /* bf16 large matrices and activations, fp32 accumulation,
                         fp32 residual stream, statistics and softmax */

#define FREE_MAX_DRAFTS 256   /* largest K accepted by spec_verify / spec_round */

/* Class-conditional DiT geometry.  The paper uses DiT-XL/2 (Sec. 4): in_ch 4,
 * patch 2, hidden 1152, depth 28, heads 16, mlp_hidden 4608, 1000 classes,
 * learn_sigma 1 (8 output channels; the variance half is ignored, App. C).
 * Constraints: lat_h, lat_w multiples of patch; hidden a multiple of heads,
 * of 8 and of 4 (2-D sin-cos table); mlp_hidden a multiple of 8; t_freq_dim
 * even; in FREE_BF16 mode hidden/heads must be a multiple of 8 and <= 128. */
typedef struct free_dit_config {
    int32_t in_ch, lat_h, lat_w, patch, hidden, depth, heads, mlp_hidden;
    int32_t num_classes, learn_sigma, t_freq_dim, mode;
} free_dit_config;

typedef struct free_dit_s* free_dit_t;   /* opaque model handle */

/* ---- utilities (host only, no GPU needed) -------------------------------- */

const char* free_version(void);
const char* free_status_string(int32_t status);
/* hipError_t of the last failing HIP call seen by this thread (0 = none). */
int32_t free_last_hip_error(void);

/* Linear-beta DDPM schedule and the coefficients of the one-step update
 * (Eq. ddpm_update, App. C), 0-indexed by network timestep i in [0, T):
 *   coef_x[i]   = 1 / sqrt(alpha_i)
 *   coef_eps[i] = -(1 - alpha_i) / (sqrt(1 - alphabar_i) * sqrt(alpha_i))
 *   sigma[i]    = sqrt(betatilde_i), betatilde_i the posterior variance;
 *                 index 0 (where betatilde = 0) takes the value of index 1.
 * so that the transition mean is m = coef_x * x + coef_eps * eps.
 * All three outputs are [host] arrays of T doubles; any may be NULL. */
int32_t free_ddpm_schedule(int32_t T, double beta_start, double beta_end,
                           double* coef_x, double* coef_eps, double* sigma);

/* Opt-in range check of device-resident inputs of spec_verify / spec_round / the samplers (the hot-path
 * calls do not look at device values: that would force a synchronisation).  t: [device] n_t timesteps,
 * each must lie in [0, T); sigma, u, lambda: [device] n values each; sigma must be positive and finite
 * (Alg. 2 divides by sigma^2), u and lambda in [0, 1] (Alg. 2; Eq. acc_relax); NaN fails.  Any pointer
 * may be NULL (that check is skipped).  Blocking: enqueues one kernel on `stream`, waits, and allocates and
 * frees four bytes of device memory.  violations (nullable, [host]): bit 0 t, bit 1 sigma, bit 2 u,
 * bit 3 lambda.  Returns FREE_OK, FREE_ERR_RANGE if any value is out of range, FREE_ERR_SHAPE for negative
 * counts or T < 1, FREE_ERR_HIP. */
int32_t free_validate_inputs(const int32_t* t, int64_t n_t, int32_t T, const float* sigma, const float* u,
                             const float* lambda, int64_t n, uint32_t* violations, void* stream);

/* The family of reverse processes with a stochasticity parameter e >= 0 (App. on the
 * stochasticity hyperparameter, Eq. mean_var_gamma): one Euler step of
 *   dY = [ -f(Y) + (1 + e^2)/2 g^2 s(Y) ] dt + e g dW
 * for the variance-preserving diffusion behind the linear-beta schedule (f(x) = -beta x / 2,
 * g^2 = beta, one step = one of the T discrete betas, score s = -eps / sqrt(1 - alphabar)):
 *   coef_x[i]   = 1 + beta_i / 2
 *   coef_eps[i] = -(1 + e^2)/2 * beta_i / sqrt(1 - alphabar_i)
 *   sigma[i]    = e * sqrt(beta_i)
 * e = 1 is the reverse SDE (the DDPM update to first order in beta), e = 0 the probability-flow
 * ODE (sigma = 0: such steps cannot be speculated).  [host] arrays of T doubles; any may be NULL. */
int32_t free_sde_schedule(int32_t T, double beta_start, double beta_end, double stochasticity,
                          double* coef_x, double* coef_eps, double* sigma);

/* Number of weight pointers free_dit_create expects: 7 + 10*depth + 4. */
int32_t free_weight_count(const free_dit_config* cfg);

/* ---- model handle ---------------------------------------------------------
 * weight_ptrs: [host] array of n_ptrs DEVICE pointers, borrowed (the caller
 * keeps them alive and unchanged until free_dit_destroy), in this order, all
 * matrices [out, in] row-major:
 *   patch_w [hidden, in_ch*patch^2] (flattened over c, ph, pw), patch_b,
 *   t_w1 [hidden, t_freq_dim], t_b1, t_w2 [hidden, hidden], t_b2,
 *   y_table [num_classes+1, hidden] (last row = null label),
 *   then per block: ada_w [6*hidden, hidden] (rows: shift1, scale1, gate1,
 *   shift2, scale2, gate2), ada_b, qkv_w [3*hidden, hidden] (rows: q | k | v,
 *   each head-major), qkv_b, proj_w, proj_b, fc1_w [mlp_hidden, hidden],
 *   fc1_b, fc2_w [hidden, mlp_hidden], fc2_b,
 *   then fin_ada_w [2*hidden, hidden] (shift, scale), fin_ada_b,
 *   fin_w [patch^2*c_out, hidden] (rows ordered ph, pw, c), fin_b.
 * Element types: in FREE_BF16 mode ada_w, qkv_w, proj_w, fc1_w, fc2_w,
 * fin_ada_w and fin_w are bf16; everything else, and everything in FREE_FP32
 * mode, is fp32.  All pointers must be 16-byte aligned.
 * free_dit_create is not a hot-path call: it allocates a small device table
 * (positional embedding, pointer table) that free_dit_destroy releases. */
int32_t free_dit_create(const free_dit_config* cfg, const void* const* weight_ptrs,
                        int32_t n_ptrs, free_dit_t* out);
int32_t free_dit_destroy(free_dit_t h);

/* Device workspace (bytes, 256-byte aligned) for a forward on B packed states;
 * also sufficient for spec_round with the same B.  0 on a bad configuration. */
size_t free_workspace_bytes(const free_dit_config* cfg, int32_t B);

/* ---- schedule of the packed forward (Alg. 1: the K states of a round are
 *      independent samples of one batch) -------------------------------------
 * One stream (the default): the kernels of a forward run in sequence on the
 * caller's stream.  Several streams: when every part keeps at least 2048 token rows,
 * the handle can cut the batch in two halves or three thirds and run their
 * transformer blocks concurrently on side streams owned by the handle; the
 * work is forked from and joined back into the caller's stream by events, so
 * stream-ordered semantics towards the caller are unchanged.  All schedules give bit-identical results; which one is
 * faster differs by a few per cent between machines of one type.
 *   free_dit_set_streams(h, n): n = 1, 2 or 3 forces that schedule for every batch
 *     size (a batch too small for n parts takes the next smaller schedule); n = 0
 *     (the initial state) uses, per batch size, what free_dit_tune measured, and
 *     one stream where nothing was measured.
 *   free_dit_tune(h, x, t, y, B, eps_out, workspace, ws_bytes, stream): NOT a
 *     hot-path call - it enqueues up to 36 forwards of B samples (runs of four, the
 *     schedules the batch allows in turn), WAITS for them on the host, adds up the
 *     last two runs of each schedule and remembers the fastest split schedule for
 *     this batch size if it was more than 0.5 % faster than one stream (up to 8
 *     batch sizes per handle; the oldest entry is replaced).  eps_out holds a valid forward
 *     afterwards.  Batches too small to split return at once.
 *   free_dit_stream_choice(h, B): the schedule (1, 2 or 3) a forward on B packed
 *     samples would take now.
 * Settings belong to the handle; calls on one handle must not race. */
int32_t free_dit_set_streams(free_dit_t h, int32_t n);
int32_t free_dit_tune(free_dit_t h, const float* x, const int32_t* t, const int32_t* y, int32_t B,
                      float* eps_out, void* workspace, size_t ws_bytes, void* stream);
int32_t free_dit_stream_choice(free_dit_t h, int32_t B);

/* ---- LayerNorm folded into the neighbouring GEMMs (bf16 mode) --------------
 * The adaLN-Zero block of the packed forward (Alg. 1; the DiT the paper samples
 * from, Sec. 4) normalises the residual stream twice per block:
 * LN(x) (1 + scale) + shift, followed by a linear layer with weights W, bias b.
 * With z = x (1 + scale), row mean mu and r = 1 / sqrt(var + eps) this equals
 *     r (z W^T) - r mu c1 + c0,  c1 = (1 + scale) W^T,  c0 = shift W^T + b
 * (c1, c0 per packed sample).  In the folded form the GEMM that updates the
 * residual stream (attention out-projection, MLP second layer) also writes z in
 * bf16 and per-row partial sums of x and x^2, one launch computes c1 and c0 of
 * every block from the modulation vectors, and the GEMM that follows the
 * LayerNorm (QKV, MLP first layer) applies r, mu, c1, c0 in its epilogue: the
 * separate LayerNorm pass over the residual stream disappears (all but the
 * first one of block 0, whose input no GEMM produced).  Same result up to
 * rounding: z is rounded to bf16 where the separate pass rounds the normalised
 * row, and the variance is E[x^2] - mu^2 in fp32.
 * Covered: FREE_BF16, hidden % 128 == 0, tokens per sample % 32 == 0.
 *   FREE_LN_FOLD_AUTO (initial state): folded when covered and the batch has at
 *     least 4096 token rows (its GEMMs use the two large tile shapes only),
 *     the separate LayerNorm kernel otherwise.
 *   FREE_LN_FOLD_OFF: always the separate kernel.
 *   FREE_LN_FOLD_REQUIRE: always folded; free_dit_set_ln_fold returns
 *     FREE_ERR_SHAPE when the model is not covered - never a silent switch.
 * free_dit_ln_fold_active(h, B): 1 if a forward on B packed states would take
 * the folded path now, else 0.  The drafter's blocks always use the separate
 * kernel. */
#define FREE_LN_FOLD_OFF     0
#define FREE_LN_FOLD_AUTO    1
#define FREE_LN_FOLD_REQUIRE 2
int32_t free_dit_set_ln_fold(free_dit_t h, int32_t mode);
int32_t free_dit_ln_fold_active(free_dit_t h, int32_t B);

/* ---- the packed target forward (Alg. 1, "in parallel"; Sec. 3.3) ----------
 * One forward of the class-conditional DiT on B packed states, each with its
 * own timestep t[b] and label y[b] (int32, device).
 *   x        [B, C, H, W] fp32
 *   eps_out  [B, c_out, H, W] fp32, c_out = 2C with learn_sigma: channels
 *            [0, C) are the noise prediction, [C, 2C) the unused variance.
 *   top_feat [B, N, hidden] fp32 or NULL: output of the last block (the
 *            feature f of Alg. 1).
 * Enqueues on `stream` and returns without waiting for the device; results are
 * ordered after the call on that stream.  A handle owns two internal side
 * streams (see free_dit_set_streams), so two calls on the SAME handle must not
 * be in flight from different streams at the same time; calls on different
 * handles are independent.  The call allocates nothing and can be captured in a
 * HIP graph. */
int32_t dit_forward_packed(free_dit_t h, const float* x, const int32_t* t, const int32_t* y,
                           int32_t B, float* eps_out, float* top_feat,
                           void* workspace, size_t ws_bytes, void* stream);

/* ---- verification (Alg. 2; Eq. qp; Eq. acc_relax; Alg. 1 inner loop) ------
 * n_traj independent trajectories, K drafts each, d elements per state.
 *   m_target, m_draft, x_draft  [n_traj, K, d] fp32
 *   sigma, u                    [n_traj, K] fp32
 *   lambda                      [n_traj, K] fp32 or NULL (strict rule)
 * For every (trajectory, draft):
 *   l = (m - m^)^T (x^ - (m + m^)/2) / sigma^2               (Eq. qp)
 *   accepted iff log u <= min(0, lambda * l)  (u <= min(1, exp(lambda l)));
 *   u = 0 or m^ == m always accepts.
 * Outputs:
 *   log_ratio [n_traj, K] fp32  unscaled l
 *   accept    [n_traj, K] uint8 stand-alone decision of each draft
 *   n_accept  [n_traj]    int32 number of drafts accepted before the first
 *                               rejection (K if none was rejected)
 *   x_out     [n_traj, d] fp32  reflected sample of the first rejected draft,
 *                               x = m + (I - 2 e e^T)(x^ - m^), e = (m^ - m)/||m^ - m||;
 *                               rows with n_accept == K are left untouched.
 * Sums over d are accumulated in fp64 in a fixed order: results are
 * deterministic run to run.
 * Workspace: spec_verify_workspace_bytes(n_traj, K, d) bytes of device memory,
 * 8-byte aligned, contents arbitrary (the partial sums of the first launch);
 * FREE_ERR_WORKSPACE if missing or too small.  Limits: 1 <= K <= FREE_MAX_DRAFTS;
 * n_traj <= 65535 (second grid dimension of the finishing launch) and
 * n_traj * K * ceil(d / chunk) workgroups must fit a one-dimensional grid
 * (2^31 - 1; chunk >= 1024 elements); FREE_ERR_SHAPE otherwise.  Enqueues two
 * kernels (streaming sums; decisions + reflection); no host synchronisation. */
size_t spec_verify_workspace_bytes(int32_t n_traj, int32_t K, int64_t d);
int32_t spec_verify(const float* m_target, const float* m_draft, const float* x_draft,
                    const float* sigma, const float* u, const float* lambda,
                    int32_t n_traj, int32_t K, int64_t d,
                    float* log_ratio, uint8_t* accept, int32_t* n_accept, float* x_out,
                    void* workspace, size_t ws_bytes, void* stream);

/* Verification with one variance per ELEMENT (App. C: fixed-variance schedules richer
 * than one scalar per step; Sec. 3.3 requires only that draft and target share the
 * covariance).  Both transitions are N(mean, diag(s^2)) with the same vector s, so in
 * the whitened coordinates (x - c) / s Alg. 2 applies unchanged:
 *   l = sum_i (m_i - m^_i)(x^_i - (m_i + m^_i)/2) / s_i^2,
 *   e = ((m^ - m)/s) / ||(m^ - m)/s||,  x = m + s * (I - 2 e e^T)((x^ - m^)/s).
 * sigma_elem [n_traj, K, d] fp32 (> 0) takes the place of sigma [n_traj, K]; every
 * other argument, the outputs, the workspace, the limits and the status codes are
 * those of spec_verify.  Streams 16 bytes per latent element and draft. */
int32_t spec_verify_diag(const float* m_target, const float* m_draft, const float* x_draft,
                         const float* sigma_elem, const float* u, const float* lambda,
                         int32_t n_traj, int32_t K, int64_t d,
                         float* log_ratio, uint8_t* accept, int32_t* n_accept, float* x_out,
                         void* workspace, size_t ws_bytes, void* stream);

/* spec_verify for callers that cannot allocate device memory or bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (minus the workspace), same kernels, same results and
 * status codes as spec_verify; the partial sums live in a static device array of
 * FREE_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the
 * process ends).  The call allocates and frees nothing.  Problems whose partial
 * sums do not fit - spec_verify_workspace_bytes(n_traj, K, d) >
 * FREE_STATIC_SCRATCH_BYTES, i.e. more than 65536 streaming workgroups - are
 * refused with FREE_ERR_LIMIT before anything is launched; the headline
 * verification workload (64 x 6 x 16384) needs 24 KiB.  The first call on a
 * device looks the array's address up (hipGetSymbolAddress, once per device):
 * make that call outside a stream capture.  Nothing in the array has to start at
 * zero (every partial sum is written before it is read), but all calls on one
 * GPU share it: calls that overlap in time on one GPU - different streams, or
 * replays of two captured graphs - race and must be ordered by the caller. */
#define FREE_STATIC_SCRATCH_BYTES (1u << 20)
int32_t spec_verify_static(const float* m_target, const float* m_draft, const float* x_draft,
                           const float* sigma, const float* u, const float* lambda,
                           int32_t n_traj, int32_t K, int64_t d,
                           float* log_ratio, uint8_t* accept, int32_t* n_accept, float* x_out,
                           void* stream);

/* Benchmark helper, NOT a hot-path call: spec_verify with a start and a stop HIP event
 * attached to each of its two dispatches on `stream` (the events are created and
 * destroyed inside the call); waits for the call to finish and returns [host] the
 * milliseconds the streaming kernel and the finishing kernel ran.  Same arguments, results and status codes as spec_verify,
 * n_traj >= 1. */
int32_t spec_verify_timed(const float* m_target, const float* m_draft, const float* x_draft,
                          const float* sigma, const float* u, const float* lambda,
                          int32_t n_traj, int32_t K, int64_t d,
                          float* log_ratio, uint8_t* accept, int32_t* n_accept, float* x_out,
                          void* workspace, size_t ws_bytes, void* stream,
                          float* stream_ms, float* finish_ms);

/* ---- one verification round of one trajectory (Alg. 1 body after drafting) -
 * Packed forward on the K states x_states = (x_a, x^_{a+1}, ..., x^_{a+K-1})
 * at timesteps t[0..K) with label y; with cfg_scale > 1 the batch is doubled
 * with the null label and eps = eps_null + cfg_scale (eps_cond - eps_null);
 * then m_k = coef_x[k] x_k + coef_eps[k] eps_k (Eq. ddpm_update) and draft
 * k+1 (x_states[k+1]; x_last for k = K-1) is verified against
 * (m_draft[k], m_k, sigma[k]) exactly as in spec_verify with n_traj = 1.
 *   x_states [K, C, H, W], x_last [C, H, W], m_draft [K, d]   fp32, device
 *   t [K] int32 device; y, cfg_scale [host] scalars
 *   coef_x, coef_eps, sigma, u [K] fp32 device; lambda [K] or NULL
 *   m_target_out [K, d] or NULL; log_ratio [K]; accept [K]; n_accept [1];
 *   x_out [d] (written only when n_accept < K). */
int32_t spec_round(free_dit_t h, const float* x_states, const float* x_last, const float* m_draft,
                   const int32_t* t, int32_t y, float cfg_scale,
                   const float* coef_x, const float* coef_eps, const float* sigma,
                   const float* u, const float* lambda, int32_t K,
                   float* m_target_out, float* log_ratio, uint8_t* accept,
                   int32_t* n_accept, float* x_out,
                   void* workspace, size_t ws_bytes, void* stream);

/* ---- drafter and drafting loop (Sec. 3.2 "Feature-Level Autoregressive Drafting";
 *      Alg. 1, inner drafting loop) ------------------------------------------
 * The drafter shares the target's embedding layers (patch embedding with the
 * positional table, timestep and label embedding), fuses the embedded latent
 * with the propagated top-block feature by one fully connected layer on their
 * concatenation [embedding | feature], runs `drafter_depth` DiT blocks of its
 * own (one in the paper's main setting) and an output projection of the form
 * of the target's final layer.
 *
 * Weights [device], borrowed until free_drafter_destroy, in this order, the
 * large matrices in the target's compute type, the rest fp32, all 16-byte
 * aligned, matrices [out, in] row-major:
 *   fuse_w [D, 2D], fuse_b [D],
 *   per block: the 10 tensors of a target block (ada_w .. fc2_b),
 *   fin_ada_w [2D, D], fin_ada_b [2D], fin_w [p*p*c_out, D], fin_b.
 * free_drafter_weight_count(depth) = 2 + 10 depth + 4.  The target handle must
 * outlive the drafter. */
typedef struct free_drafter_s* free_drafter_t;
int32_t free_drafter_weight_count(int32_t drafter_depth);
int32_t free_drafter_create(free_dit_t target, int32_t drafter_depth, const void* const* weight_ptrs,
                            int32_t n_ptrs, free_drafter_t* out);
int32_t free_drafter_destroy(free_drafter_t dr);
/* Workspace of drafter_forward on B samples; also sufficient for draft_round
 * (which runs B = 1, or 2 with guidance).  0 on bad arguments. */
size_t free_drafter_workspace_bytes(free_dit_t target, int32_t drafter_depth, int32_t B);

/* One drafter evaluation p(. | x^_{t-1}, f_{t-1}) on B samples.
 *   x [B, C, H, W], f_prev [B, N, D] fp32, t, y [B] int32  [device]
 *   eps_out [B, c_out, H, W] fp32: noise estimate in channels [0, C)
 *   f_out   [B, N, D] fp32: predicted next top-block feature; may alias f_prev
 * Enqueues on `stream`; FREE_ERR_* as for dit_forward_packed. */
int32_t drafter_forward(free_drafter_t dr, const float* x, const float* f_prev, const int32_t* t,
                        const int32_t* y, int32_t B, float* eps_out, float* f_out,
                        void* workspace, size_t ws_bytes, void* stream);

/* The drafting loop of one trajectory: for k = 0..K-1 the drafter runs on
 * (x^_k, f_{k-1}) at timestep t[k] (x^_0 = x_a, f_{-1} = f_a), its noise estimate
 * gives the draft mean m^_k = coef_x[k] x^_k + coef_eps[k] eps^_k (Eq. ddpm_update)
 * and the next draft is x^_{k+1} = m^_k + sigma[k] xi[k].  With cfg_scale > 1 the
 * drafter runs on the label y and on the null label, each branch with its own
 * feature, and the two estimates are combined as in spec_round.
 *   x_a [C, H, W]; f_a [dup, N, D] (dup = 2 with guidance: label branch first);
 *   t [K] int32; coef_x, coef_eps, sigma [K]; xi [K, d] standard normal draws
 *   (an input: the library has no generator)                         [device]
 *   outputs, the inputs of spec_round: x_states [K, C, H, W] (x_states[0] = x_a),
 *   x_last [d], m_draft [K, d]; f_last [dup, N, D] (optional, may be NULL): the
 *   feature after the last step. */
int32_t draft_round(free_drafter_t dr, const float* x_a, const float* f_a, const int32_t* t, int32_t y,
                    float cfg_scale, const float* coef_x, const float* coef_eps, const float* sigma,
                    const float* xi, int32_t K, float* x_states, float* x_last, float* m_draft,
                    float* f_last, void* workspace, size_t ws_bytes, void* stream);

/* ---- the whole sampler (Alg. 1): target step, drafting, packed verification, advance
 * Steps are indexed i = 0..S-1: step i takes the state x_i (network timestep tmap[i], transition
 * coefficients coef_x[i], coef_eps[i], sigma[i]) and produces x_{i+1}; x_S is the result.
 *   - a plain target step x_{i+1} = m_i + sigma[i] xi[i] is taken at i = 0 (no feature exists yet)
 *     and for the steps i >= n_spec, which are never speculated (sigma = 0: the noise-free last step);
 *   - otherwise one round drafts K = min(L, n_spec - i) steps from (x_i, feature) with draft_round
 *     (noise xi[i .. i+K-1]), runs ONE packed target forward on (x_i, x^_{i+1}, .., x^_{i+K-1}) and
 *     verifies the drafts in order with u[i .. i+K-1] (and lambda, when given), as spec_round does;
 *   - with n drafts accepted the sampler moves to x^_{i+K} (n = K) or to the reflected sample
 *     x_{i+n+1}; the feature handed to the next round is the target's top-block feature of the packed
 *     state whose transition was just taken.  (The listing's last line would draw an already
 *     verified state again; this reading does not, and every round costs one target call.)
 * All arrays [device] unless marked: x_init [C, H, W]; tmap [S] int32; coef_x, coef_eps, sigma [S];
 * xi [S, d]; u [S]; lambda [S] or NULL; x_result [C, H, W].
 * stats [host, 4 x int32, may be NULL]: target calls, rounds, accepted drafts, drafter steps.
 * n_accept_log [host, S x int32, may be NULL]: accepted drafts of round r in entry r.
 * The call is SYNCHRONOUS: it reads the accepted count back after every round (4 bytes) and returns
 * when x_result is complete.  Workspace: free_sample_workspace_bytes. */
size_t free_sample_workspace_bytes(free_drafter_t dr, int32_t L, float cfg_scale);
int32_t free_sample(free_drafter_t dr, const float* x_init, int32_t y, float cfg_scale, int32_t S,
                    int32_t n_spec, int32_t L, const int32_t* tmap, const float* coef_x,
                    const float* coef_eps, const float* sigma, const float* xi, const float* u,
                    const float* lambda, float* x_result, int32_t* stats, int32_t* n_accept_log,
                    void* workspace, size_t ws_bytes, void* stream);

/* ---- relaxation profile (Sec. 3.4 "Uncertainty-Guided Verification Relaxation") ----
 * free_self_speculative: the offline run in which the target both proposes and verifies.  Same loop
 * and arguments as free_sample, with frozen-target drafting instead of a drafter: the guided noise
 * estimate of the latest target evaluation is reused for the next K steps,
 * m^_k = coef_x[k] x^_k + coef_eps[k] eps_frozen.  For every checked draft at step i it records
 *   eps_delta[i] = || eps_frozen - eps_target(x^_i) ||_2   and   accepted[i] in {0, 1}
 * [host arrays of S entries, either may be NULL]; steps that were never checked (plain target steps,
 * drafts behind a rejection) hold NaN and -1.  Synchronous.
 * free_lambda_profile [host only]: lambda from the measured deviations - a non-decreasing least-squares
 * fit over the step index (NaN entries carry no weight), a centred moving average of odd width
 * `window` (1 = none) with the ends held, then lambda_i = g_0 / g_i in (0, 1].  FREE_ERR_RANGE when no
 * entry is measured, FREE_ERR_SHAPE for S < 1 or an even window. */
size_t free_self_speculative_workspace_bytes(free_dit_t target, int32_t L, float cfg_scale);
int32_t free_self_speculative(free_dit_t target, const float* x_init, int32_t y, float cfg_scale, int32_t S,
                              int32_t n_spec, int32_t L, const int32_t* tmap, const float* coef_x,
                              const float* coef_eps, const float* sigma, const float* xi, const float* u,
                              const float* lambda, float* x_result, int32_t* stats, int32_t* n_accept_log,
                              float* eps_delta, int8_t* accepted, void* workspace, size_t ws_bytes,
                              void* stream);
int32_t free_lambda_profile(const float* eps_delta, int32_t S, int32_t window, float* lambda_out);

/* ---- per-kernel timing for benchmarks -------------------------------------
 * Between free_profile_begin(h) and free_profile_end(h) every kernel launch that
 * a hot-path call makes on behalf of handle h (dit_forward_packed, spec_round,
 * the drafter and the samplers built on it) is bracketed by two HIP events
 * recorded on the launch stream, and the forward uses one stream.
 * free_profile_end waits for the last event and returns, per category, the
 * summed elapsed milliseconds and the number of bracketed launches ([host]
 * arrays of FREE_PROF_NCAT entries).  The state belongs to the handle (events
 * are created on first use and released with it); off by default, and a handle
 * that never profiles records nothing.  Categories, in order:
 * conditioning, adaln, patch_embed, ln_modulate, gemm_qkv, attention,
 * gemm_proj, gemm_fc1, gemm_fc2, final_layer, eps_to_mean, verify. */
#define FREE_PROF_NCAT 12
int32_t free_profile_begin(free_dit_t h);
int32_t free_profile_end(free_dit_t h, float* ms, int32_t* launches);
const char* free_profile_category_name(int32_t category);

/* Matrix-core calibration for the "mfma" roofline of the benchmark: runs a
 * register-only loop of `iters` x 4 v_mfma_f32_32x32x16_bf16 per wavefront on
 * every compute unit (8 wavefronts each, no memory traffic), once untimed and
 * once timed with HIP events on `stream`, and returns [host] the sustained
 * TFLOP/s and the shader clock in MHz observed meanwhile (shader cycles over
 * the constant-rate wall clock, mean over workgroups).  Blocking; allocates
 * and frees two small device buffers.  iters in [1, 2^24]; about 75 ns per
 * iteration.  FREE_ERR_NULL / FREE_ERR_RANGE / FREE_ERR_HIP on failure. */
int32_t free_mfma_ceiling(int32_t iters, double* tflops, double* mhz, void* stream);

/* ---- single DiT operators, exported for per-kernel parity tests -----------
 * (the pieces of the adaLN-Zero block that dit_forward_packed chains).
 * dtype = FREE_FP32 (A, W, out fp32) or FREE_BF16 (A, W, out bf16). */
#define FREE_EPI_BIAS       0   /* out = A W^T + bias                          */
#define FREE_EPI_BIAS_GELU  1   /* out = gelu_tanh(A W^T + bias)               */
#define FREE_EPI_GATE_RESID 2   /* resid[m,n] += gate[m / rows_per_sample, n] *
                                   (A W^T + bias)[m,n]; resid fp32 [M, N],
                                   gate fp32 with row stride gate_stride       */
int32_t free_op_linear(const void* A, const void* W, const float* bias, int32_t M, int32_t N,
                       int32_t Kdim, int32_t dtype, int32_t epilogue, void* out,
                       float* resid, const float* gate, int32_t gate_stride,
                       int32_t rows_per_sample, void* stream);
/* out[b, n, h*dh + :] = softmax(q k^T / sqrt(dh)) v per (sample, head);
 * qkv [B*N, 3*heads*dh] rows ordered q | k | v, out [B*N, heads*dh]; dh <= 128. */
int32_t free_op_attention(const void* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh,
                          int32_t dtype, void* out, void* stream);
/* out[m, :] = LayerNorm(x[m, :]) * (1 + scale[m / rows_per_sample, :]) + shift[...]
 * (no affine, biased variance, eps 1e-6); x fp32 [M, D]; shift/scale fp32 with
 * row stride mod_stride; out fp32 or bf16 per dtype. */
int32_t free_op_ln_modulate(const float* x, const float* shift, const float* scale,
                            int32_t mod_stride, int32_t M, int32_t D, int32_t rows_per_sample,
                            int32_t dtype, void* out, void* stream);

/* The three pieces of the folded LayerNorm (see free_dit_set_ln_fold), bf16 only, for parity tests.
 * free_op_ln_fold_vectors: c1 | c0 for `depth` blocks from mod [B, mod_stride] (block l: shift1, scale1, gate1,
 *   shift2, scale2, gate2, `hidden` floats each, at l * 6 hidden); w_qkv / b_qkv / w_fc1 / b_fc1: host arrays of
 *   `depth` device pointers (bf16 [3 hidden, hidden] / fp32 [3 hidden] / bf16 [ffn, hidden] / fp32 [ffn]);
 *   fold [B, fold_stride] fp32 out, fold_stride >= 2 depth (3 hidden + ffn): c1 of block l's QKV rows at
 *   l (3 hidden + ffn), its MLP-1 rows behind them, and c0 depth (3 hidden + ffn) floats further.  Blocks: it
 *   copies the pointer tables to the device and waits (a test entry point, not a hot-path call).
 * free_op_linear_resid_prep: resid += gate * (A W^T + bias) as FREE_EPI_GATE_RESID, and z [M, N] bf16 =
 *   resid_new * (1 + scale_next[m / rows_per_sample, :]), stats [M, N / 128, 2] fp32 = per row and 128-column
 *   slot the sums of resid_new and resid_new^2.  N % 128 == 0; gate and scale_next share mod_stride.
 * free_op_linear_ln: out [M, N] bf16 = act(r (z W^T) - r mu c1 + c0), r and mu of row m from stats
 *   [M, Kdim / 128, 2], c1 / c0 of sample s at c1[s * fold_stride + n]; gelu != 0 applies gelu_tanh. */
int32_t free_op_ln_fold_vectors(const float* mod, int32_t B, int32_t hidden, int32_t ffn, int32_t mod_stride,
                                int32_t depth, const void* const* w_qkv, const float* const* b_qkv,
                                const void* const* w_fc1, const float* const* b_fc1, float* fold,
                                int64_t fold_stride, void* stream);
int32_t free_op_linear_resid_prep(const void* A, const void* W, const float* bias, int32_t M, int32_t N,
                                  int32_t Kdim, float* resid, const float* gate, const float* scale_next,
                                  int32_t mod_stride, int32_t rows_per_sample, void* z, float* stats,
                                  void* stream);
int32_t free_op_linear_ln(const void* z, const void* W, int32_t M, int32_t N, int32_t Kdim, const float* stats,
                          const float* c1, const float* c0, int64_t fold_stride, int32_t rows_per_sample,
                          int32_t gelu, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FREE_MI355X_H */
