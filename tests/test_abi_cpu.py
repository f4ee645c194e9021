"""CPU-only checks of the C-ABI library: it loads, exports every symbol the public
header declares, its host-side schedule helper agrees with the oracle, and argument
errors are reported as status codes before any GPU call is made."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import free_oracle as fo
from paper_2511_20390_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "free_mi355x.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_][a-z0-9_]*)\s*\(", text)) - {"defined"})


def test_header_symbols_are_exported_and_bound(lib):
    names = _declared_functions()
    assert {"dit_forward_packed", "spec_verify", "spec_round"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_version_and_status_strings(lib):
    assert b"gfx950" in lib.free_version()
    seen = {lib.free_status_string(s) for s in range(0, -8, -1)}
    assert len(seen) == 8 and lib.free_status_string(-99) == b"unknown status"


def test_schedule_helper_matches_oracle(lib):
    cx, ce, sg = binding.free_ddpm_schedule()
    s = fo.ddpm_schedule()
    ocx, oce = fo.mean_coefficients(np.arange(1000), s)
    np.testing.assert_allclose(cx, ocx, rtol=1e-13)
    np.testing.assert_allclose(ce, oce, rtol=1e-12)
    np.testing.assert_allclose(sg, s["sigma_clipped"], rtol=1e-12)
    assert lib.free_ddpm_schedule(1, 1e-4, 0.02, None, None, None) == binding.FREE_ERR_SHAPE
    assert lib.free_ddpm_schedule(10, 0.0, 0.02, None, None, None) == binding.FREE_ERR_RANGE
    assert lib.free_ddpm_schedule(10, 1e-4, 0.02, None, None, None) == binding.FREE_OK


def test_weight_count_and_workspace(lib):
    for name in ("tiny", "small", "xl2_512"):
        cfg = synth.dit_config(name)
        cc = binding.make_config(cfg, "bf16")
        assert lib.free_weight_count(C.byref(cc)) == len(synth.weight_spec(cfg)) == 7 + 10 * cfg["depth"] + 4
        b6, b12 = lib.free_workspace_bytes(C.byref(cc), 6), lib.free_workspace_bytes(C.byref(cc), 12)
        assert 0 < b6 < b12 and b6 % 256 == 0
        cc32 = binding.make_config(cfg, "fp32")
        assert lib.free_workspace_bytes(C.byref(cc32), 6) > b6
    bad = binding.make_config(dict(synth.dit_config("tiny"), hidden=60), "fp32")     # 60 % 8 != 0
    assert lib.free_weight_count(C.byref(bad)) == binding.FREE_ERR_SHAPE
    assert lib.free_workspace_bytes(C.byref(bad), 6) == 0
    bad = binding.make_config(dict(synth.dit_config("tiny"), lat_h=7), "fp32")
    assert lib.free_workspace_bytes(C.byref(bad), 6) == 0
    assert lib.free_workspace_bytes(C.byref(cc), 0) == 0


def test_argument_errors_are_status_codes(lib):
    one = C.c_void_p(256)            # never dereferenced: the checks fail first
    # calibration loop: null outputs and iteration counts outside [1, 2^24] fail before any device call
    assert lib.free_mfma_ceiling(1000, None, one, None) == binding.FREE_ERR_NULL
    assert lib.free_mfma_ceiling(0, one, one, None) == binding.FREE_ERR_RANGE
    assert lib.free_mfma_ceiling((1 << 24) + 1, one, one, None) == binding.FREE_ERR_RANGE
    # validation helper: negative counts and T < 1 fail before any device call
    assert lib.free_validate_inputs(one, -1, 1000, None, None, None, 0, None, None) == binding.FREE_ERR_SHAPE
    assert lib.free_validate_inputs(one, 4, 0, None, None, None, 0, None, None) == binding.FREE_ERR_SHAPE
    assert lib.free_validate_inputs(None, 0, 1000, one, None, None, -5, None, None) == binding.FREE_ERR_SHAPE
    # spec_verify: null pointer, bad shape
    assert lib.spec_verify(None, one, one, one, one, None, 1, 6, 64, one, one, one, one, one, 4096, None) == binding.FREE_ERR_NULL
    assert lib.spec_verify(one, one, one, one, one, None, 1, 0, 64, one, one, one, one, one, 4096, None) == binding.FREE_ERR_SHAPE
    assert lib.spec_verify(one, one, one, one, one, None, 1, 257, 64, one, one, one, one, one, 4096, None) == binding.FREE_ERR_SHAPE
    assert lib.spec_verify(one, one, one, one, one, None, 1, 6, 0, one, one, one, one, one, 4096, None) == binding.FREE_ERR_SHAPE
    assert lib.spec_verify(one, one, one, one, one, None, 0, 6, 64, one, one, one, one, one, 4096, None) == binding.FREE_OK
    # missing / too small workspace
    assert lib.spec_verify(one, one, one, one, one, None, 1, 6, 64, one, one, one, one, None, 0, None) == binding.FREE_ERR_WORKSPACE
    assert lib.spec_verify(one, one, one, one, one, None, 4, 6, 4096, one, one, one, one, one, 8, None) == binding.FREE_ERR_WORKSPACE
    assert lib.spec_verify_diag(one, one, one, None, one, None, 1, 6, 64, one, one, one, one, one, 4096, None) == binding.FREE_ERR_NULL
    assert lib.spec_verify_diag(one, one, one, one, one, None, 1, 6, 0, one, one, one, one, one, 4096, None) == binding.FREE_ERR_SHAPE
    assert lib.spec_verify_diag(one, one, one, one, one, None, 1, 6, 64, one, one, one, one, None, 0, None) == binding.FREE_ERR_WORKSPACE
    # the entry point with built-in scratch: argument checks first, then the size limit, all before any device call
    assert lib.spec_verify_static(None, one, one, one, one, None, 1, 6, 64, one, one, one, one, None) == binding.FREE_ERR_NULL
    assert lib.spec_verify_static(one, one, one, one, one, None, 1, 0, 64, one, one, one, one, None) == binding.FREE_ERR_SHAPE
    assert lib.spec_verify_static(one, one, one, one, one, None, 0, 6, 64, one, one, one, one, None) == binding.FREE_OK
    assert lib.spec_verify_workspace_bytes(20000, 6, 16384) > binding.STATIC_SCRATCH_BYTES
    assert lib.spec_verify_static(one, one, one, one, one, None, 20000, 6, 16384, one, one, one, one, None) == binding.FREE_ERR_LIMIT
    assert lib.spec_verify_workspace_bytes(64, 6, 16384) >= 64 * 6 * 16
    assert lib.spec_verify_workspace_bytes(64, 300, 16384) == 0
    # model handle
    cc = binding.make_config(synth.dit_config("tiny"), "fp32")
    h = C.c_void_p()
    assert lib.free_dit_create(C.byref(cc), None, 31, C.byref(h)) == binding.FREE_ERR_NULL
    arr = (C.c_void_p * 31)(*([256] * 31))
    assert lib.free_dit_create(C.byref(cc), arr, 30, C.byref(h)) == binding.FREE_ERR_SHAPE
    arr[3] = None
    assert lib.free_dit_create(C.byref(cc), arr, 31, C.byref(h)) == binding.FREE_ERR_NULL
    arr[3] = 260                     # misaligned
    assert lib.free_dit_create(C.byref(cc), arr, 31, C.byref(h)) == binding.FREE_ERR_SHAPE
    cc.mode = 5
    assert lib.free_dit_create(C.byref(cc), arr, 31, C.byref(h)) == binding.FREE_ERR_DTYPE
    assert lib.free_dit_destroy(None) == binding.FREE_ERR_NULL
    # schedule of the packed forward and per-kernel timing: settings of a handle
    assert lib.free_dit_set_streams(None, 1) == binding.FREE_ERR_NULL
    assert lib.free_dit_stream_choice(None, 12) == binding.FREE_ERR_NULL
    assert lib.free_dit_tune(None, one, one, one, 12, one, one, 1 << 20, None) == binding.FREE_ERR_NULL
    assert lib.free_profile_begin(None) == binding.FREE_ERR_NULL
    assert lib.free_profile_end(None, one, one) == binding.FREE_ERR_NULL
    assert lib.dit_forward_packed(None, one, one, one, 6, one, None, one, 1 << 20, None) == binding.FREE_ERR_NULL
    assert lib.spec_round(None, one, one, one, one, 0, 4.0, one, one, one, one, None, 6, None, one, one, one, one,
                          one, 1 << 20, None) == binding.FREE_ERR_NULL
    # single operators
    assert lib.free_op_linear(one, one, one, 4, 4, 8, 7, 0, one, None, None, 0, 1, None) == binding.FREE_ERR_DTYPE
    assert lib.free_op_linear(one, one, one, 4, 4, 8, 0, 9, one, None, None, 0, 1, None) == binding.FREE_ERR_RANGE
    assert lib.free_op_linear(one, one, one, 4, 4, 8, 0, 2, one, None, None, 0, 1, None) == binding.FREE_ERR_NULL
    assert lib.free_op_attention(one, 1, 16, 2, 200, 0, one, None) == binding.FREE_ERR_SHAPE
    assert lib.free_op_ln_modulate(one, one, None, 8, 4, 8, 1, 0, one, None) == binding.FREE_ERR_NULL
    # LayerNorm folded into the GEMMs: setting of a handle, and the three pieces as operators
    assert lib.free_dit_set_ln_fold(None, binding.LN_FOLD_OFF) == binding.FREE_ERR_NULL
    assert lib.free_dit_ln_fold_active(None, 12) == binding.FREE_ERR_NULL
    assert lib.free_op_ln_fold_vectors(None, 2, 128, 256, 1024, 1, one, one, one, one, one, 1 << 20, None) == binding.FREE_ERR_NULL
    assert lib.free_op_ln_fold_vectors(one, 2, 128, 256, 100, 1, one, one, one, one, one, 1 << 20, None) == binding.FREE_ERR_SHAPE
    assert lib.free_op_ln_fold_vectors(one, 2, 100, 256, 1024, 1, one, one, one, one, one, 1 << 20, None) == binding.FREE_ERR_SHAPE
    assert lib.free_op_linear_resid_prep(one, one, one, 64, 128, 64, one, one, None, 384, 32, one, one, None) == binding.FREE_ERR_NULL
    assert lib.free_op_linear_resid_prep(one, one, one, 64, 100, 64, one, one, one, 384, 32, one, one, None) == binding.FREE_ERR_SHAPE
    assert lib.free_op_linear_ln(one, one, 64, 128, 128, None, one, one, 256, 32, 0, one, None) == binding.FREE_ERR_NULL
    assert lib.free_op_linear_ln(one, one, 64, 128, 100, one, one, one, 256, 32, 0, one, None) == binding.FREE_ERR_SHAPE
    assert lib.free_op_linear_ln(one, one, 64, 128, 128, one, one, one, 256, 33, 0, one, None) == binding.FREE_ERR_SHAPE


def test_synth_is_deterministic_and_bf16_rounding_is_exact():
    cfg = synth.dit_config("tiny")
    a, b = synth.make_weights(cfg, 3), synth.make_weights(cfg, 3)
    assert all(np.array_equal(a[k], b[k]) for k in a)
    w = synth.make_weights(cfg, 3, bf16_values=True)
    import torch
    for k, v in w.items():
        assert np.array_equal(torch.from_numpy(v).to(torch.bfloat16).float().numpy(), v)
    # round-to-nearest-even against torch's conversion
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    assert np.array_equal(synth.bf16_round(x), torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    s = fo.ddpm_schedule()
    r1 = synth.make_round_inputs(cfg, 6, 5, s["sigma_clipped"])
    assert list(r1["t"]) == list(range(r1["t"][0], r1["t"][0] - 6, -1)) and r1["t"][-1] >= 0
    v = synth.make_verify_inputs(3, 6, 64, 0.1, 1, s["sigma_clipped"])
    assert v["m_target"].shape == (3, 6, 64) and (v["sigma"] > 0).all() and ((v["lam"] > 0) & (v["lam"] <= 1)).all()


def test_drafter_argument_errors_are_status_codes(lib):
    one = C.c_void_p(256)
    assert lib.free_drafter_weight_count(1) == len(synth.drafter_weight_spec(synth.dit_config("tiny"), 1)) == 16
    assert lib.free_drafter_weight_count(2) == 26 and lib.free_drafter_weight_count(0) < 0
    h = C.c_void_p()
    assert lib.free_drafter_create(None, 1, None, 16, C.byref(h)) == binding.FREE_ERR_NULL
    assert lib.free_drafter_destroy(None) == binding.FREE_ERR_NULL
    assert lib.free_drafter_workspace_bytes(None, 1, 2) == 0
    assert lib.drafter_forward(None, one, one, one, one, 2, one, one, one, 4096, None) == binding.FREE_ERR_NULL
    assert lib.draft_round(None, one, one, one, 0, 4.0, one, one, one, one, 6, one, one, one, None, one, 4096,
                           None) == binding.FREE_ERR_NULL


def test_lambda_profile_host_helper_matches_oracle(lib):
    rng = np.random.default_rng(0)
    for S, window in ((5, 1), (60, 1), (60, 9), (250, 21)):
        v = (np.linspace(1, 4, S) + 0.4 * rng.standard_normal(S)).astype(np.float32)
        v[rng.random(S) < 0.3] = np.nan
        v[0] = 1.0
        ref = fo.relaxation_profile_from_deltas(v.astype(np.float64), window)
        got = binding.free_lambda_profile(v, window)
        np.testing.assert_allclose(got, ref, rtol=2e-6)
    out = np.empty(4, np.float32)
    nan = np.full(4, np.nan, np.float32)
    assert lib.free_lambda_profile(nan.ctypes.data, 4, 1, out.ctypes.data) == binding.FREE_ERR_RANGE
    assert lib.free_lambda_profile(nan.ctypes.data, 4, 2, out.ctypes.data) == binding.FREE_ERR_SHAPE
    assert lib.free_lambda_profile(None, 4, 1, out.ctypes.data) == binding.FREE_ERR_NULL
    assert lib.free_self_speculative_workspace_bytes(None, 4, 4.0) == 0


def test_sde_schedule_helper_matches_oracle(lib):
    for e in (0.0, 0.7, 1.0, 2.5):
        cx, ce, sg = binding.free_sde_schedule(e)
        ocx, oce, osg = fo.sde_coefficients(e)
        np.testing.assert_allclose(cx, ocx, rtol=1e-14)
        np.testing.assert_allclose(ce, oce, rtol=1e-12)
        np.testing.assert_allclose(sg, osg, rtol=1e-14, atol=0)
    assert lib.free_sde_schedule(10, 1e-4, 0.02, -1.0, None, None, None) == binding.FREE_ERR_RANGE
    assert lib.free_sde_schedule(1, 1e-4, 0.02, 1.0, None, None, None) == binding.FREE_ERR_SHAPE


def _function_body(text, signature_start):
    """Source text of the function whose definition starts with `signature_start` (brace matching)."""
    at = text.index(signature_start)
    i = text.index("{", at)
    depth, j = 0, i
    while True:
        depth += {"{": 1, "}": -1}.get(text[j], 0)
        j += 1
        if depth == 0:
            return text[at:j]


def test_hot_path_calls_never_wait_for_the_device():
    """The hot-path entry points only enqueue: no host-side wait (stream, event or device synchronisation,
    blocking copies, allocation) appears in their bodies or in the launch chains they call."""
    csrc = os.path.join(ROOT, "paper_2511_20390_amd", "csrc")
    abi = open(os.path.join(csrc, "free_abi.hip")).read()
    ver = open(os.path.join(csrc, "verify.hip")).read()
    bodies = [_function_body(abi, "int32_t forward_impl("), _function_body(abi, "int32_t run_block_stack("),
              _function_body(abi, "int32_t dit_forward_packed("), _function_body(abi, "int32_t spec_round("),
              _function_body(abi, "int32_t spec_verify("), _function_body(abi, "int32_t drafter_forward_impl("),
              _function_body(abi, "int32_t draft_round("), _function_body(ver, "int32_t launch_verify(")]
    banned = ("Synchronize", "hipMalloc", "hipFree", "hipMemcpy(", "hipMemset", "hipEventElapsedTime",
              "hipEventQuery", "hipStreamQuery")
    for body in bodies:
        for word in banned:
            assert word not in body, f"{word} in {body[:60]!r}"
    # the blocking calls exist, outside the hot path, and say so
    assert "Synchronize" in _function_body(abi, "int32_t free_dit_tune(")


def test_verify_workspace_sizes():
    """Workspace of the verification: one pair of fp64 partial sums per workgroup of the streaming launch;
    positive and 256-byte granular over a sweep of shapes, zero for shapes the call refuses."""
    lib = binding.load()
    for d in (1, 5, 1023, 1024, 4096, 16384, 65536, 1 << 20, (1 << 22) + 3):
        for K in (1, 2, 6, 12, 64, 256):
            for n in (1, 3, 64, 1000):
                b = lib.spec_verify_workspace_bytes(n, K, d)
                assert b % 256 == 0 and b >= 16 * n * K
    assert lib.spec_verify_workspace_bytes(0, 6, 64) == 0
    assert lib.spec_verify_workspace_bytes(4, 0, 64) == 0
    assert lib.spec_verify_workspace_bytes(4, 6, 0) == 0


def test_binding_refuses_tensors_the_library_would_misread():
    """The C side sees raw pointers: the binding checks device, element type, contiguity and shape first
    and raises without making a call (host tensors here, so nothing touches a GPU)."""
    import torch
    binding.load()
    f = torch.zeros(2, 3, 8)
    with pytest.raises(binding.FreeError) as e:
        binding._dev(f, torch.float32, "m_target")
    assert e.value.status == binding.FREE_ERR_NULL                      # not a device tensor
    with pytest.raises(binding.FreeError):
        binding._dev(None, torch.float32, "sigma")
    assert binding._dev(None, torch.float32, "lambda", optional=True) is None

    class Fake:                       # stands in for a device tensor: only the attributes _dev looks at
        is_cuda = True

        def __init__(self, t):
            self.t = t
            self.dtype, self.shape = t.dtype, t.shape

        def is_contiguous(self):
            return self.t.is_contiguous()

        def data_ptr(self):
            return self.t.data_ptr()

    good = torch.zeros(4, 6)
    assert binding._dev(Fake(good), torch.float32, "sigma", (4, 6)).value == good.data_ptr()
    for bad, status in [(Fake(torch.zeros(4, 6, dtype=torch.float64)), binding.FREE_ERR_DTYPE),
                        (Fake(torch.zeros(6, dtype=torch.int64)), binding.FREE_ERR_DTYPE),
                        (Fake(torch.zeros(4, 12)[:, ::2]), binding.FREE_ERR_SHAPE),
                        (Fake(torch.zeros(4, 5)), binding.FREE_ERR_SHAPE)]:
        with pytest.raises(binding.FreeError) as e:
            binding._dev(bad, torch.int32 if bad.dtype == torch.int64 else torch.float32, "x", (4, 6))
        assert e.value.status == status
