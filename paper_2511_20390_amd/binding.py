"""ctypes binding over libfree_mi355x.so (the C ABI declared in include/free_mi355x.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch is used for device memory and the current HIP stream.  There
is no fallback: a missing library raises, a non-zero status raises FreeError.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfree_mi355x.so")

FREE_OK = 0
FREE_ERR_NULL, FREE_ERR_SHAPE, FREE_ERR_RANGE, FREE_ERR_DTYPE, FREE_ERR_WORKSPACE, FREE_ERR_HIP = -1, -2, -3, -4, -5, -6
FREE_ERR_LIMIT = -7
STATIC_SCRATCH_BYTES = 1 << 20
FREE_FP32, FREE_BF16 = 0, 1
EPI_BIAS, EPI_BIAS_GELU, EPI_GATE_RESID = 0, 1, 2
LN_FOLD_OFF, LN_FOLD_AUTO, LN_FOLD_REQUIRE = 0, 1, 2
LN_SLOT_COLS = 128
MODES = {"fp32": FREE_FP32, "bf16": FREE_BF16}

EXPORTED_SYMBOLS = [
    "free_version", "free_status_string", "free_last_hip_error", "free_dit_set_streams",
    "free_dit_tune", "free_dit_stream_choice", "free_ddpm_schedule", "free_sde_schedule",
    "free_weight_count", "free_dit_create", "free_dit_destroy", "free_workspace_bytes",
    "dit_forward_packed", "spec_verify_workspace_bytes", "spec_verify", "spec_verify_diag", "spec_verify_static", "spec_verify_timed", "spec_round",
    "free_drafter_weight_count", "free_drafter_create", "free_drafter_destroy", "free_drafter_workspace_bytes",
    "drafter_forward", "draft_round", "free_sample_workspace_bytes", "free_sample",
    "free_self_speculative_workspace_bytes", "free_self_speculative", "free_lambda_profile",
    "free_op_linear", "free_op_attention", "free_op_ln_modulate",
    "free_dit_set_ln_fold", "free_dit_ln_fold_active", "free_op_ln_fold_vectors", "free_op_linear_resid_prep",
    "free_op_linear_ln",
    "free_profile_begin", "free_profile_end", "free_profile_category_name", "free_mfma_ceiling", "free_validate_inputs",
]
PROF_NCAT = 12


class FreeError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = load().free_status_string(status).decode()
        if status == FREE_ERR_HIP:
            msg += f" (hipError {load().free_last_hip_error()})"
        super().__init__(f"{where}: status {status}: {msg}")


class FreeDitConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("in_ch", "lat_h", "lat_w", "patch", "hidden", "depth", "heads",
                                          "mlp_hidden", "num_classes", "learn_sigma", "t_freq_dim", "mode")]


_lib = None


def load():
    """Open the library (once) and declare the signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` to build it")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    lib.free_version.restype = C.c_char_p
    lib.free_status_string.restype = C.c_char_p
    lib.free_status_string.argtypes = [i32]
    lib.free_last_hip_error.restype = i32
    lib.free_dit_set_streams.restype = i32
    lib.free_dit_set_streams.argtypes = [vp, i32]
    lib.free_dit_tune.restype = i32
    lib.free_dit_tune.argtypes = [vp, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.free_dit_stream_choice.restype = i32
    lib.free_dit_stream_choice.argtypes = [vp, i32]
    lib.free_ddpm_schedule.restype = i32
    lib.free_ddpm_schedule.argtypes = [i32, C.c_double, C.c_double, vp, vp, vp]
    lib.free_sde_schedule.restype = i32
    lib.free_sde_schedule.argtypes = [i32, C.c_double, C.c_double, C.c_double, vp, vp, vp]
    lib.free_weight_count.restype = i32
    lib.free_weight_count.argtypes = [C.POINTER(FreeDitConfig)]
    lib.free_dit_create.restype = i32
    lib.free_dit_create.argtypes = [C.POINTER(FreeDitConfig), C.POINTER(vp), i32, C.POINTER(vp)]
    lib.free_dit_destroy.restype = i32
    lib.free_dit_destroy.argtypes = [vp]
    lib.free_workspace_bytes.restype = sz
    lib.free_workspace_bytes.argtypes = [C.POINTER(FreeDitConfig), i32]
    lib.dit_forward_packed.restype = i32
    lib.dit_forward_packed.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.spec_verify_workspace_bytes.restype = sz
    lib.spec_verify_workspace_bytes.argtypes = [i32, i32, i64]
    lib.spec_verify.restype = i32
    lib.spec_verify.argtypes = [vp] * 6 + [i32, i32, i64] + [vp] * 4 + [vp, sz, vp]
    lib.spec_verify_diag.restype = i32
    lib.spec_verify_diag.argtypes = [vp] * 6 + [i32, i32, i64] + [vp] * 4 + [vp, sz, vp]
    lib.spec_verify_static.restype = i32
    lib.spec_verify_static.argtypes = [vp] * 6 + [i32, i32, i64] + [vp] * 4 + [vp]
    lib.spec_verify_timed.restype = i32
    lib.spec_verify_timed.argtypes = [vp] * 6 + [i32, i32, i64] + [vp] * 4 + [vp, sz, vp, vp, vp]
    lib.spec_round.restype = i32
    lib.spec_round.argtypes = [vp, vp, vp, vp, vp, i32, f32, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.free_drafter_weight_count.restype = i32
    lib.free_drafter_weight_count.argtypes = [i32]
    lib.free_drafter_create.restype = i32
    lib.free_drafter_create.argtypes = [vp, i32, C.POINTER(vp), i32, C.POINTER(vp)]
    lib.free_drafter_destroy.restype = i32
    lib.free_drafter_destroy.argtypes = [vp]
    lib.free_drafter_workspace_bytes.restype = sz
    lib.free_drafter_workspace_bytes.argtypes = [vp, i32, i32]
    lib.drafter_forward.restype = i32
    lib.drafter_forward.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.draft_round.restype = i32
    lib.draft_round.argtypes = [vp, vp, vp, vp, i32, f32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.free_sample_workspace_bytes.restype = sz
    lib.free_sample_workspace_bytes.argtypes = [vp, i32, f32]
    lib.free_sample.restype = i32
    lib.free_sample.argtypes = [vp, vp, i32, f32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.free_self_speculative_workspace_bytes.restype = sz
    lib.free_self_speculative_workspace_bytes.argtypes = [vp, i32, f32]
    lib.free_self_speculative.restype = i32
    lib.free_self_speculative.argtypes = [vp, vp, i32, f32, i32, i32, i32] + [vp] * 12 + [vp, sz, vp]
    lib.free_lambda_profile.restype = i32
    lib.free_lambda_profile.argtypes = [vp, i32, i32, vp]
    lib.free_op_linear.restype = i32
    lib.free_op_linear.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, i32, i32, vp]
    lib.free_op_attention.restype = i32
    lib.free_op_attention.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp]
    lib.free_op_ln_modulate.restype = i32
    lib.free_op_ln_modulate.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
    lib.free_dit_set_ln_fold.restype = i32
    lib.free_dit_set_ln_fold.argtypes = [vp, i32]
    lib.free_dit_ln_fold_active.restype = i32
    lib.free_dit_ln_fold_active.argtypes = [vp, i32]
    lib.free_op_ln_fold_vectors.restype = i32
    lib.free_op_ln_fold_vectors.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, i64, vp]
    lib.free_op_linear_resid_prep.restype = i32
    lib.free_op_linear_resid_prep.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.free_op_linear_ln.restype = i32
    lib.free_op_linear_ln.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, i64, i32, i32, vp, vp]
    lib.free_profile_begin.restype = i32
    lib.free_profile_begin.argtypes = [vp]
    lib.free_profile_end.restype = i32
    lib.free_profile_end.argtypes = [vp, vp, vp]
    lib.free_validate_inputs.restype = i32
    lib.free_validate_inputs.argtypes = [vp, i64, i32, vp, vp, vp, i64, vp, vp]
    lib.free_mfma_ceiling.restype = i32
    lib.free_mfma_ceiling.argtypes = [i32, vp, vp, vp]
    lib.free_profile_category_name.restype = C.c_char_p
    lib.free_profile_category_name.argtypes = [i32]
    _lib = lib
    return lib


def _check(status, where):
    if status != FREE_OK:
        raise FreeError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dev(t, dtype, name, shape=None, optional=False):
    """Pointer of a device tensor handed to the library, after the checks the C side cannot make: the
    library reads raw memory, so a tensor of another element type (torch integers default to int64), a
    strided view or a host tensor would give wrong results or out-of-bounds device reads, not an error."""
    if t is None:
        if optional:
            return None
        raise FreeError(FREE_ERR_NULL, name)
    if not getattr(t, "is_cuda", False):
        raise FreeError(FREE_ERR_NULL, f"{name}: not a device tensor")
    if t.dtype != dtype:
        raise FreeError(FREE_ERR_DTYPE, f"{name}: element type {t.dtype}, expected {dtype}")
    if not t.is_contiguous():
        raise FreeError(FREE_ERR_SHAPE, f"{name}: not contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise FreeError(FREE_ERR_SHAPE, f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_config(cfg: dict, mode: str) -> FreeDitConfig:
    return FreeDitConfig(cfg["in_ch"], cfg["lat_h"], cfg["lat_w"], cfg["patch"], cfg["hidden"], cfg["depth"],
                         cfg["heads"], cfg["mlp_hidden"], cfg["num_classes"], cfg["learn_sigma"],
                         cfg["t_freq_dim"], MODES[mode])


def free_ddpm_schedule(T: int = 1000, beta_start: float = 1e-4, beta_end: float = 0.02):
    """Host-only: (coef_x, coef_eps, sigma) float64 arrays of length T."""
    cx, ce, sg = (np.empty(T, np.float64) for _ in range(3))
    _check(load().free_ddpm_schedule(T, beta_start, beta_end, cx.ctypes.data, ce.ctypes.data, sg.ctypes.data),
           "free_ddpm_schedule")
    return cx, ce, sg


def free_sde_schedule(stochasticity: float, T: int = 1000, beta_start: float = 1e-4, beta_end: float = 0.02):
    """Host-only: (coef_x, coef_eps, sigma) of the reverse process with the given stochasticity parameter."""
    cx, ce, sg = (np.empty(T, np.float64) for _ in range(3))
    _check(load().free_sde_schedule(T, beta_start, beta_end, float(stochasticity), cx.ctypes.data, ce.ctypes.data,
                                    sg.ctypes.data), "free_sde_schedule")
    return cx, ce, sg


def validate_inputs(t=None, T: int = 1000, sigma=None, u=None, lam=None) -> int:
    """Blocking range check of device tensors (any may be None); returns the bit mask of violations
    (0 = all in range; bit 0 t, bit 1 sigma, bit 2 u, bit 3 lambda)."""
    n = max([x.numel() for x in (sigma, u, lam) if x is not None], default=0)
    for x in (sigma, u, lam):
        if x is not None and x.numel() != n:
            raise ValueError("sigma, u and lambda must have the same number of elements")
    mask = C.c_uint32(0)
    import torch
    f32, i32 = torch.float32, torch.int32
    st = load().free_validate_inputs(_dev(t, i32, "t", optional=True), 0 if t is None else t.numel(), int(T),
                                     _dev(sigma, f32, "sigma", optional=True), _dev(u, f32, "u", optional=True),
                                     _dev(lam, f32, "lambda", optional=True), n, C.addressof(mask), _stream())
    if st not in (FREE_OK, FREE_ERR_RANGE):
        _check(st, "free_validate_inputs")
    return int(mask.value)


def mfma_ceiling(iters: int = 200000) -> dict:
    """Sustained TFLOP/s of a register-only bf16 MFMA loop on every CU and the shader clock meanwhile."""
    import torch
    tf, mhz = C.c_double(0.0), C.c_double(0.0)
    _check(load().free_mfma_ceiling(int(iters), C.addressof(tf), C.addressof(mhz), _stream()),
           "free_mfma_ceiling")
    return {"tflops": tf.value, "shader_clock_mhz": mhz.value}


def spec_verify_workspace_bytes(n_traj: int, K: int, d: int) -> int:
    return load().spec_verify_workspace_bytes(n_traj, K, d)


def _verify_out(out, n_traj, K, d, dev):
    import torch
    if out is None:
        out = dict(log_ratio=torch.empty(n_traj, K, dtype=torch.float32, device=dev),
                   accept=torch.empty(n_traj, K, dtype=torch.uint8, device=dev),
                   n_accept=torch.empty(n_traj, dtype=torch.int32, device=dev),
                   x_out=torch.zeros(n_traj, d, dtype=torch.float32, device=dev))
    return out


def spec_verify(m_target, m_draft, x_draft, sigma, u, lam=None, out=None, workspace=None, timed=False):
    """Device tensors in, dict of device tensors out.  m_*, x_draft: [n_traj, K, d] fp32.
    timed: blocking benchmark variant; the dict then also holds "stream_us" and "finish_us", the durations
    of the call's two launches by HIP events on the launch stream."""
    import torch
    f32 = torch.float32
    n_traj, K, d = m_target.shape
    dev = m_target.device
    out = _verify_out(out, n_traj, K, d, dev)
    if workspace is None:
        workspace = torch.empty(max(256, spec_verify_workspace_bytes(n_traj, K, d)), dtype=torch.uint8, device=dev)
    args = [_dev(m_target, f32, "m_target"), _dev(m_draft, f32, "m_draft", (n_traj, K, d)),
            _dev(x_draft, f32, "x_draft", (n_traj, K, d)), _dev(sigma, f32, "sigma", (n_traj, K)),
            _dev(u, f32, "u", (n_traj, K)), _dev(lam, f32, "lambda", (n_traj, K), optional=True),
            n_traj, K, d, _dev(out["log_ratio"], f32, "log_ratio", (n_traj, K)),
            _dev(out["accept"], torch.uint8, "accept", (n_traj, K)),
            _dev(out["n_accept"], torch.int32, "n_accept", (n_traj,)),
            _dev(out["x_out"], f32, "x_out", (n_traj, d)),
            _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()]
    if timed:
        a, b = C.c_float(0.0), C.c_float(0.0)
        _check(load().spec_verify_timed(*args, C.addressof(a), C.addressof(b)), "spec_verify_timed")
        out = dict(out, stream_us=a.value * 1e3, finish_us=b.value * 1e3)
    else:
        _check(load().spec_verify(*args), "spec_verify")
    return out


def spec_verify_diag(m_target, m_draft, x_draft, sigma_elem, u, lam=None, out=None, workspace=None):
    """spec_verify with one standard deviation per element: sigma_elem [n_traj, K, d] fp32."""
    import torch
    f32 = torch.float32
    n_traj, K, d = m_target.shape
    dev = m_target.device
    out = _verify_out(out, n_traj, K, d, dev)
    if workspace is None:
        workspace = torch.empty(max(256, spec_verify_workspace_bytes(n_traj, K, d)), dtype=torch.uint8, device=dev)
    _check(load().spec_verify_diag(
        _dev(m_target, f32, "m_target"), _dev(m_draft, f32, "m_draft", (n_traj, K, d)),
        _dev(x_draft, f32, "x_draft", (n_traj, K, d)), _dev(sigma_elem, f32, "sigma_elem", (n_traj, K, d)),
        _dev(u, f32, "u", (n_traj, K)), _dev(lam, f32, "lambda", (n_traj, K), optional=True), n_traj, K, d,
        _dev(out["log_ratio"], f32, "log_ratio", (n_traj, K)), _dev(out["accept"], torch.uint8, "accept", (n_traj, K)),
        _dev(out["n_accept"], torch.int32, "n_accept", (n_traj,)), _dev(out["x_out"], f32, "x_out", (n_traj, d)),
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()), "spec_verify_diag")
    return out


def spec_verify_static(m_target, m_draft, x_draft, sigma, u, lam=None, out=None):
    """spec_verify through the entry point that allocates nothing (static scratch inside the library); the
    outputs are the caller's (allocated here when `out` is None)."""
    import torch
    f32 = torch.float32
    n_traj, K, d = m_target.shape
    out = _verify_out(out, n_traj, K, d, m_target.device)
    _check(load().spec_verify_static(
        _dev(m_target, f32, "m_target"), _dev(m_draft, f32, "m_draft", (n_traj, K, d)),
        _dev(x_draft, f32, "x_draft", (n_traj, K, d)), _dev(sigma, f32, "sigma", (n_traj, K)),
        _dev(u, f32, "u", (n_traj, K)), _dev(lam, f32, "lambda", (n_traj, K), optional=True), n_traj, K, d,
        _dev(out["log_ratio"], f32, "log_ratio", (n_traj, K)), _dev(out["accept"], torch.uint8, "accept", (n_traj, K)),
        _dev(out["n_accept"], torch.int32, "n_accept", (n_traj,)), _dev(out["x_out"], f32, "x_out", (n_traj, d)),
        _stream()), "spec_verify_static")
    return out


class FreeDit:
    """Model handle: borrows the caller's device weight tensors (kept alive here)."""

    def __init__(self, cfg: dict, weights: dict, mode: str = "bf16", device="cuda:0"):
        import torch
        from . import synth
        self.cfg, self.mode, self.device = dict(cfg), mode, torch.device(device)
        self.ccfg = make_config(cfg, mode)
        self.tensors = []
        for name, shape in synth.weight_spec(cfg):
            a = torch.from_numpy(np.ascontiguousarray(weights[name], dtype=np.float32)).reshape(shape)
            a = a.to(self.device)
            if mode == "bf16" and synth.is_big_matrix(name):
                a = a.to(torch.bfloat16)
            self.tensors.append(a.contiguous())
        n = load().free_weight_count(C.byref(self.ccfg))
        if n != len(self.tensors):
            raise FreeError(n if n < 0 else FREE_ERR_SHAPE, "free_weight_count")
        arr = (C.c_void_p * n)(*[t.data_ptr() for t in self.tensors])
        self.handle = C.c_void_p()
        _check(load().free_dit_create(C.byref(self.ccfg), arr, n, C.byref(self.handle)), "free_dit_create")
        self._ws = {}
        self.C, self.H, self.W = cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]
        self.c_out = self.C * (2 if cfg["learn_sigma"] else 1)
        self.ntok = (self.H // cfg["patch"]) * (self.W // cfg["patch"])
        self.d = self.C * self.H * self.W

    def set_streams(self, n: int) -> None:
        """1, 2 or 3: force that schedule of the block stack (the batch in one piece, two halves or three thirds on
        as many streams) for every batch size; 0: what tune() measured per batch size, one stream where nothing
        was measured (the initial state)."""
        _check(load().free_dit_set_streams(self.handle, int(n)), "free_dit_set_streams")

    def set_ln_fold(self, mode: int) -> None:
        """LN_FOLD_OFF / LN_FOLD_AUTO / LN_FOLD_REQUIRE: whether the LayerNorms of the blocks are folded into the
        GEMMs around them (bf16 only).  REQUIRE on a model the folded path does not cover raises."""
        _check(load().free_dit_set_ln_fold(self.handle, int(mode)), "free_dit_set_ln_fold")

    def ln_fold_active(self, B: int) -> bool:
        st = int(load().free_dit_ln_fold_active(self.handle, int(B)))
        _check(min(st, 0), "free_dit_ln_fold_active")
        return bool(st)

    def stream_choice(self, B: int) -> int:
        """The schedule (1, 2 or 3 streams) a forward on B packed states would use now."""
        st = int(load().free_dit_stream_choice(self.handle, int(B)))
        _check(min(st, 0), "free_dit_stream_choice")
        return st

    def tune(self, x, t, y) -> int:
        """Blocking, not a hot-path call: times the schedules this batch allows (one, two, three streams) on these
        inputs and keeps the fastest for this batch size.  Returns the choice."""
        import torch
        B = x.shape[0]
        eps = torch.empty(B, self.c_out, self.H, self.W, dtype=torch.float32, device=self.device)
        ws = self.workspace(B)
        _check(load().free_dit_tune(self.handle, _dev(x, torch.float32, "x", (B, self.C, self.H, self.W)),
                                    _dev(t, torch.int32, "t", (B,)), _dev(y, torch.int32, "y", (B,)), B, _ptr(eps),
                                    _ptr(ws), ws.numel(), _stream()), "free_dit_tune")
        return self.stream_choice(B)

    def profile_begin(self) -> None:
        _check(load().free_profile_begin(self.handle), "free_profile_begin")

    def profile_end(self) -> dict:
        """{category: (total_ms, launches)} for this handle's launches since profile_begin."""
        ms = np.zeros(PROF_NCAT, np.float32)
        cnt = np.zeros(PROF_NCAT, np.int32)
        _check(load().free_profile_end(self.handle, ms.ctypes.data, cnt.ctypes.data), "free_profile_end")
        return {load().free_profile_category_name(c).decode(): (float(ms[c]), int(cnt[c])) for c in range(PROF_NCAT)}

    def close(self):
        if getattr(self, "handle", None) is not None and self.handle.value:
            load().free_dit_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self, B: int) -> int:
        return load().free_workspace_bytes(C.byref(self.ccfg), B)

    def workspace(self, B: int):
        import torch
        if B not in self._ws:
            self._ws[B] = torch.empty(self.workspace_bytes(B), dtype=torch.uint8, device=self.device)
        return self._ws[B]

    def dit_forward_packed(self, x, t, y, want_feat=False):
        import torch
        B = x.shape[0]
        eps = torch.empty(B, self.c_out, self.H, self.W, dtype=torch.float32, device=self.device)
        feat = torch.empty(B, self.ntok, self.cfg["hidden"], dtype=torch.float32, device=self.device) if want_feat else None
        ws = self.workspace(B)
        _check(load().dit_forward_packed(self.handle, _dev(x, torch.float32, "x", (B, self.C, self.H, self.W)),
                                         _dev(t, torch.int32, "t", (B,)), _dev(y, torch.int32, "y", (B,)), B,
                                         _ptr(eps), _ptr(feat), _ptr(ws), ws.numel(), _stream()), "dit_forward_packed")
        return (eps, feat) if want_feat else eps

    def spec_round(self, x_states, x_last, m_draft, t, y: int, cfg_scale: float, coef_x, coef_eps, sigma, u,
                   lam=None, want_means=True, out=None):
        import torch
        K = x_states.shape[0]
        B = K * (2 if cfg_scale > 1.0 else 1)
        dev = self.device
        if out is None:
            out = dict(m_target=torch.empty(K, self.d, dtype=torch.float32, device=dev) if want_means else None,
                       log_ratio=torch.empty(K, dtype=torch.float32, device=dev),
                       accept=torch.empty(K, dtype=torch.uint8, device=dev),
                       n_accept=torch.empty(1, dtype=torch.int32, device=dev),
                       x_out=torch.zeros(self.d, dtype=torch.float32, device=dev))
        ws = self.workspace(B)
        f32 = torch.float32
        if x_last.numel() != self.d:
            raise FreeError(FREE_ERR_SHAPE, "x_last: wrong number of elements")
        _check(load().spec_round(self.handle, _dev(x_states, f32, "x_states", (K, self.C, self.H, self.W)),
                                 _dev(x_last, f32, "x_last"), _dev(m_draft, f32, "m_draft", (K, self.d)),
                                 _dev(t, torch.int32, "t", (K,)), int(y), float(cfg_scale),
                                 _dev(coef_x, f32, "coef_x", (K,)), _dev(coef_eps, f32, "coef_eps", (K,)),
                                 _dev(sigma, f32, "sigma", (K,)), _dev(u, f32, "u", (K,)),
                                 _dev(lam, f32, "lambda", (K,), optional=True), K,
                                 _dev(out["m_target"], f32, "m_target", (K, self.d), optional=True),
                                 _dev(out["log_ratio"], f32, "log_ratio", (K,)),
                                 _dev(out["accept"], torch.uint8, "accept", (K,)),
                                 _dev(out["n_accept"], torch.int32, "n_accept", (1,)),
                                 _dev(out["x_out"], f32, "x_out", (self.d,)), _ptr(ws), ws.numel(), _stream()),
               "spec_round")
        return out


class FreeDrafter:
    """Drafter handle on top of a FreeDit target (shares its embedding layers); borrows the caller's
    drafter weight tensors (kept alive here).  The target must outlive it."""

    def __init__(self, target: FreeDit, weights: dict, drafter_depth: int = 1):
        import torch
        from . import synth
        self.target, self.depth = target, int(drafter_depth)
        self.device = target.device
        self.tensors = []
        for name, shape in synth.drafter_weight_spec(target.cfg, self.depth):
            a = torch.from_numpy(np.ascontiguousarray(weights[name], dtype=np.float32)).reshape(shape).to(self.device)
            if target.mode == "bf16" and synth.is_big_matrix(name):
                a = a.to(torch.bfloat16)
            self.tensors.append(a.contiguous())
        n = load().free_drafter_weight_count(self.depth)
        if n != len(self.tensors):
            raise FreeError(FREE_ERR_SHAPE, "free_drafter_weight_count")
        arr = (C.c_void_p * n)(*[t.data_ptr() for t in self.tensors])
        self.handle = C.c_void_p()
        _check(load().free_drafter_create(target.handle, self.depth, arr, n, C.byref(self.handle)), "free_drafter_create")
        self._ws = {}

    def close(self):
        if getattr(self, "handle", None) is not None and self.handle.value:
            load().free_drafter_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace(self, B: int):
        import torch
        if B not in self._ws:
            n = load().free_drafter_workspace_bytes(self.target.handle, self.depth, B)
            self._ws[B] = torch.empty(n, dtype=torch.uint8, device=self.device)
        return self._ws[B]

    def drafter_forward(self, x, f_prev, t, y):
        """One drafter evaluation on B samples: returns (eps [B, c_out, H, W], f [B, N, D])."""
        import torch
        tg = self.target
        B = x.shape[0]
        eps = torch.empty(B, tg.c_out, tg.H, tg.W, dtype=torch.float32, device=self.device)
        f = torch.empty(B, tg.ntok, tg.cfg["hidden"], dtype=torch.float32, device=self.device)
        ws = self.workspace(B)
        _check(load().drafter_forward(self.handle, _dev(x, torch.float32, "x", (B, tg.C, tg.H, tg.W)),
                                      _dev(f_prev, torch.float32, "f_prev", (B, tg.ntok, tg.cfg["hidden"])),
                                      _dev(t, torch.int32, "t", (B,)), _dev(y, torch.int32, "y", (B,)), B, _ptr(eps),
                                      _ptr(f), _ptr(ws), ws.numel(), _stream()), "drafter_forward")
        return eps, f

    def draft_round(self, x_a, f_a, t, y: int, cfg_scale: float, coef_x, coef_eps, sigma, xi, want_feat=False,
                    out=None):
        """K drafting steps: returns dict(x_states [K, C, H, W], x_last [d], m_draft [K, d], f_last)."""
        import torch
        tg = self.target
        K = t.shape[0]
        dup = 2 if cfg_scale > 1.0 else 1
        dev = self.device
        if out is None:
            out = dict(x_states=torch.empty(K, tg.C, tg.H, tg.W, dtype=torch.float32, device=dev),
                       x_last=torch.empty(tg.d, dtype=torch.float32, device=dev),
                       m_draft=torch.empty(K, tg.d, dtype=torch.float32, device=dev),
                       f_last=torch.empty(dup, tg.ntok, tg.cfg["hidden"], dtype=torch.float32, device=dev)
                       if want_feat else None)
        ws = self.workspace(dup)
        f32 = torch.float32
        if x_a.numel() != tg.d:
            raise FreeError(FREE_ERR_SHAPE, "x_a: wrong number of elements")
        _check(load().draft_round(self.handle, _dev(x_a, f32, "x_a"),
                                  _dev(f_a, f32, "f_a", (dup, tg.ntok, tg.cfg["hidden"])),
                                  _dev(t, torch.int32, "t", (K,)), int(y), float(cfg_scale),
                                  _dev(coef_x, f32, "coef_x", (K,)), _dev(coef_eps, f32, "coef_eps", (K,)),
                                  _dev(sigma, f32, "sigma", (K,)), _dev(xi, f32, "xi", (K, tg.d)), K,
                                  _dev(out["x_states"], f32, "x_states", (K, tg.C, tg.H, tg.W)),
                                  _dev(out["x_last"], f32, "x_last", (tg.d,)),
                                  _dev(out["m_draft"], f32, "m_draft", (K, tg.d)),
                                  _dev(out["f_last"], f32, "f_last", optional=True), _ptr(ws), ws.numel(), _stream()),
               "draft_round")
        return out


def free_sample(drafter: "FreeDrafter", x_init, y: int, cfg_scale: float, n_spec: int, L: int, tmap, coef_x,
                coef_eps, sigma, xi, u, lam=None):
    """The whole sampler (synchronous): returns (x_result, stats dict, per-round accepted counts)."""
    import torch
    S = tmap.shape[0]
    n = load().free_sample_workspace_bytes(drafter.handle, L, float(cfg_scale))
    key = ("loop", L, cfg_scale > 1.0)
    if key not in drafter._ws:
        drafter._ws[key] = torch.empty(n, dtype=torch.uint8, device=drafter.device)
    ws = drafter._ws[key]
    x_out = torch.empty_like(x_init)
    stats = (C.c_int32 * 4)()
    log = (C.c_int32 * S)()
    f32, d = torch.float32, drafter.target.d
    if x_init.numel() != d:
        raise FreeError(FREE_ERR_SHAPE, "x_init: wrong number of elements")
    _check(load().free_sample(drafter.handle, _dev(x_init, f32, "x_init"), int(y), float(cfg_scale), S, int(n_spec), int(L),
                              _dev(tmap, torch.int32, "tmap", (S,)), _dev(coef_x, f32, "coef_x", (S,)),
                              _dev(coef_eps, f32, "coef_eps", (S,)), _dev(sigma, f32, "sigma", (S,)),
                              _dev(xi, f32, "xi", (S, d)), _dev(u, f32, "u", (S,)),
                              _dev(lam, f32, "lambda", (S,), optional=True),
                              _ptr(x_out), stats, log, _ptr(ws), ws.numel(), _stream()), "free_sample")
    st = dict(target_calls=stats[0], rounds=stats[1], accepted=stats[2], drafter_steps=stats[3])
    return x_out, st, [log[r] for r in range(stats[1])]


def free_self_speculative(target: FreeDit, x_init, y: int, cfg_scale: float, n_spec: int, L: int, tmap, coef_x,
                          coef_eps, sigma, xi, u, lam=None):
    """The offline self-speculative run (synchronous): returns (x_result, stats, per-round accepted counts,
    eps_delta [S] float32 with NaN where unchecked, accepted [S] int8 with -1 where unchecked)."""
    import torch
    S = tmap.shape[0]
    n = load().free_self_speculative_workspace_bytes(target.handle, L, float(cfg_scale))
    key = ("self", L, cfg_scale > 1.0)
    if key not in target._ws:
        target._ws[key] = torch.empty(n, dtype=torch.uint8, device=target.device)
    ws = target._ws[key]
    x_out = torch.empty_like(x_init)
    stats = (C.c_int32 * 4)()
    log = (C.c_int32 * S)()
    delta = np.empty(S, np.float32)
    acc = np.empty(S, np.int8)
    f32, d = torch.float32, target.d
    if x_init.numel() != d:
        raise FreeError(FREE_ERR_SHAPE, "x_init: wrong number of elements")
    _check(load().free_self_speculative(target.handle, _dev(x_init, f32, "x_init"), int(y), float(cfg_scale), S,
                                        int(n_spec), int(L), _dev(tmap, torch.int32, "tmap", (S,)),
                                        _dev(coef_x, f32, "coef_x", (S,)), _dev(coef_eps, f32, "coef_eps", (S,)),
                                        _dev(sigma, f32, "sigma", (S,)), _dev(xi, f32, "xi", (S, d)),
                                        _dev(u, f32, "u", (S,)), _dev(lam, f32, "lambda", (S,), optional=True),
                                        _ptr(x_out), stats, log, delta.ctypes.data, acc.ctypes.data,
                                        _ptr(ws), ws.numel(), _stream()), "free_self_speculative")
    st = dict(target_calls=stats[0], rounds=stats[1], accepted=stats[2], drafter_steps=stats[3])
    return x_out, st, [log[r] for r in range(stats[1])], delta, acc


def free_lambda_profile(eps_delta, window: int = 1) -> np.ndarray:
    """Host only: the relaxation profile lambda [S] from measured deviations (NaN = not measured)."""
    e = np.ascontiguousarray(eps_delta, np.float32)
    out = np.empty(e.shape[0], np.float32)
    _check(load().free_lambda_profile(e.ctypes.data, e.shape[0], int(window), out.ctypes.data), "free_lambda_profile")
    return out


def op_linear(A, W, bias, mode: str, epilogue: int = EPI_BIAS, resid=None, gate=None, rows_per_sample: int = 1):
    import torch
    M, K = A.shape
    N = W.shape[0]
    out = None
    if epilogue != EPI_GATE_RESID:
        out = torch.empty(M, N, dtype=A.dtype, device=A.device)
    _check(load().free_op_linear(_ptr(A), _ptr(W), _ptr(bias), M, N, K, MODES[mode], epilogue, _ptr(out),
                                 _ptr(resid), _ptr(gate), 0 if gate is None else gate.stride(0),
                                 rows_per_sample, _stream()), "free_op_linear")
    return resid if epilogue == EPI_GATE_RESID else out


def op_attention(qkv, B: int, N: int, heads: int, dh: int, mode: str):
    import torch
    out = torch.empty(B * N, heads * dh, dtype=qkv.dtype, device=qkv.device)
    _check(load().free_op_attention(_ptr(qkv), B, N, heads, dh, MODES[mode], _ptr(out), _stream()),
           "free_op_attention")
    return out


def op_ln_fold_vectors(mod, hidden: int, ffn: int, w_qkv, b_qkv, w_fc1, b_fc1):
    """mod [B, >= 6 depth hidden] fp32; w_qkv ...: lists of `depth` device tensors.  Returns fold [B, 2 depth (3 hidden + ffn)]:
    c1 of all layers, then c0 (free_op_ln_fold_vectors)."""
    import torch
    depth = len(w_qkv)
    B = mod.shape[0]
    rows = depth * (3 * hidden + ffn)
    fold = torch.empty(B, 2 * rows, dtype=torch.float32, device=mod.device)
    arr = lambda ts: (C.c_void_p * depth)(*[t.data_ptr() for t in ts])
    _check(load().free_op_ln_fold_vectors(_ptr(mod), B, hidden, ffn, mod.stride(0), depth, arr(w_qkv), arr(b_qkv),
                                          arr(w_fc1), arr(b_fc1), _ptr(fold), fold.stride(0), _stream()),
           "free_op_ln_fold_vectors")
    return fold


def op_linear_resid_prep(A, W, bias, resid, gate, scale_next, rows_per_sample: int):
    """resid += gate * (A W^T + bias) in place; returns (z bf16 [M, N], stats fp32 [M, N / 128, 2])."""
    import torch
    M, K = A.shape
    N = W.shape[0]
    z = torch.empty(M, N, dtype=torch.bfloat16, device=A.device)
    stats = torch.empty(M, N // LN_SLOT_COLS, 2, dtype=torch.float32, device=A.device)
    assert gate.stride(0) == scale_next.stride(0)
    _check(load().free_op_linear_resid_prep(_ptr(A), _ptr(W), _ptr(bias), M, N, K, _ptr(resid), _ptr(gate),
                                            _ptr(scale_next), gate.stride(0), rows_per_sample, _ptr(z), _ptr(stats),
                                            _stream()), "free_op_linear_resid_prep")
    return z, stats


def op_linear_ln(z, W, stats, c1, c0, rows_per_sample: int, gelu: bool):
    """out bf16 [M, N] = act(r (z W^T) - r mu c1 + c0); c1 / c0 [samples, N] views with a common row stride."""
    import torch
    M, K = z.shape
    N = W.shape[0]
    out = torch.empty(M, N, dtype=torch.bfloat16, device=z.device)
    assert c1.stride(0) == c0.stride(0)
    _check(load().free_op_linear_ln(_ptr(z), _ptr(W), M, N, K, _ptr(stats), _ptr(c1), _ptr(c0), c1.stride(0),
                                    rows_per_sample, int(bool(gelu)), _ptr(out), _stream()), "free_op_linear_ln")
    return out


def op_ln_modulate(x, shift, scale, rows_per_sample: int, mode: str):
    import torch
    M, D = x.shape
    out = torch.empty(M, D, dtype=torch.float32 if mode == "fp32" else torch.bfloat16, device=x.device)
    _check(load().free_op_ln_modulate(_ptr(x), _ptr(shift), _ptr(scale), shift.stride(0), M, D, rows_per_sample,
                                      MODES[mode], _ptr(out), _stream()), "free_op_ln_modulate")
    return out
