"""The verification entry point that allocates nothing (static device scratch inside the library) against
spec_verify with a caller workspace: same kernels, so every output must be identical, on two calls in a row,
the second on a smaller input (the scratch then still holds the first call's partial sums)."""
import numpy as np
import pytest

from oracle import free_oracle as fo
from paper_2511_20390_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _case(n_traj, K, d, seed, relaxed):
    import torch
    sched = fo.ddpm_schedule()
    vi = synth.make_verify_inputs(n_traj, K, d, 1.349 / np.sqrt(d), seed, sched["sigma_clipped"])
    args = [pu.to_dev(vi[k]) for k in ("m_target", "m_draft", "x_draft", "sigma", "u")]
    args.append(pu.to_dev(vi["lam"]) if relaxed else None)

    def outputs():
        return dict(log_ratio=torch.empty(n_traj, K, dtype=torch.float32, device="cuda:0"),
                    accept=torch.empty(n_traj, K, dtype=torch.uint8, device="cuda:0"),
                    n_accept=torch.empty(n_traj, dtype=torch.int32, device="cuda:0"),
                    x_out=torch.full((n_traj, d), 7.25, dtype=torch.float32, device="cuda:0"))
    return vi, args, outputs


def test_static_scratch_entry_point_matches_spec_verify():
    import torch
    from paper_2511_20390_amd import binding
    for n_traj, K, d, seed, relaxed in [(64, 6, 16384, 1, False), (5, 3, 3220, 2, True)]:
        vi, args, outputs = _case(n_traj, K, d, seed, relaxed)
        ref = binding.spec_verify(*args, out=outputs())
        got = binding.spec_verify_static(*args, out=outputs())
        torch.cuda.synchronize()
        for k in ("log_ratio", "accept", "n_accept", "x_out"):
            assert torch.equal(got[k], ref[k]), f"{k} differs at n_traj={n_traj} K={K} d={d}"
        nacc = got["n_accept"].cpu().numpy()
        assert (nacc < K).any() and (got["x_out"].cpu().numpy()[nacc == K] == 7.25).all()
        # and against the oracle, to the bar of the other verification tests
        lam = vi["lam"] if relaxed else None
        oracle = fo.spec_verify(vi["m_target"], vi["m_draft"], vi["x_draft"], vi["sigma"], vi["u"], lam)
        pu.compare_verify(got, oracle, lam, vi["u"], f"static scratch n_traj={n_traj} K={K} d={d}")


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    from paper_2511_20390_amd import binding
    n_traj, K, d = 70000 // 6 + 1, 6, 1024           # more partial sums than the built-in scratch holds
    assert binding.spec_verify_workspace_bytes(n_traj, K, d) > binding.STATIC_SCRATCH_BYTES
    z = torch.zeros(n_traj, K, d, device="cuda:0")
    s = torch.ones(n_traj, K, device="cuda:0")
    with pytest.raises(binding.FreeError) as e:
        binding.spec_verify_static(z, z, z, s, s)
    assert e.value.status == binding.FREE_ERR_LIMIT
