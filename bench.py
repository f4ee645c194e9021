#!/usr/bin/env python3
"""Benchmark of the parallel verification pass on one MI355X.

A step is one whole verification round (spec_round): packed DiT-XL/2 forward on
K=6 states (x2 with classifier-free guidance 4.0 -> 12 states, 12288 tokens) at
the 512^2 latent shape, guidance + eps->mean, and the sequential verification of
the six drafts.  Inputs and random-init weights are synthetic and resident in
HBM before the timed region.  Prints ONE JSON line.

  python bench.py --gpus 1 --steps 20 --warmup 3
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def forward_flops(cfg, B):
    """Algorithmic FLOPs of one packed forward: 2MNK for the linear layers, 4 N D per token per
    block for attention, plus the adaLN modulation GEMV."""
    from paper_2511_20390_amd import synth
    N, D, F, L = synth.n_tokens(cfg), cfg["hidden"], cfg["mlp_hidden"], cfg["depth"]
    M = B * N
    per = {"gemm_qkv": 2.0 * M * D * 3 * D, "gemm_proj": 2.0 * M * D * D, "gemm_fc1": 2.0 * M * D * F,
           "gemm_fc2": 2.0 * M * D * F, "attention": 4.0 * M * N * D}
    total = L * sum(per.values()) + 2.0 * B * D * (L * 6 * D + 2 * D)
    return per, total


# kernel symbol (as rocprofv3 prints it) behind each profiled category, to look its measured
# HBM traffic up in the committed rocprofv3 --pmc summary
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "spec_round_xl2_512_hbm_traffic.md")
# (epilogue codes in the kernel names: 0 bias, 1 bias + GELU, 2 gated residual update; with the LayerNorms folded
# into the GEMMs 3 / 4 = the same two after a folded LayerNorm, 5 = residual update that prepares the next one)
CATEGORY_SYMBOL = {"gemm_fc1": "gemm_bf16_kernel<bf16_t, 384, 192, 4, 2, 4, true>`",
                   "gemm_qkv": "gemm_bf16_kernel<bf16_t, 256, 256, 4, 2, 3, true>`",
                   "gemm_fc2": "gemm_bf16_kernel<bf16_t, 256, 256, 4, 2, 5, true>` FC2",
                   "gemm_proj": "gemm_bf16_kernel<bf16_t, 256, 256, 4, 2, 5, true>` out-projection",
                   "attention": "attn_mfma_kernel<72, 1>`",
                   "verify_partial": "verify_partial_kernel<256, 4, true, true, false>`"}


CATEGORY_SYMBOL_PLAIN = {"gemm_fc1": "gemm_bf16_kernel<bf16_t, 384, 192, 4, 2, 1, true>`",
                         "gemm_qkv": "gemm_bf16_kernel<bf16_t, 256, 256, 4, 2, 0, true>`",
                         "gemm_fc2": "gemm_bf16_kernel<bf16_t, 256, 256, 4, 2, 2, true>` FC2",
                         "gemm_proj": "gemm_bf16_kernel<bf16_t, 256, 256, 4, 2, 2, true>` out-projection"}


def measured_traffic(category, folded=True):
    """{'fetch_MB', 'write_MB'} per launch from the committed FETCH_SIZE / WRITE_SIZE summary, or None."""
    sym = (CATEGORY_SYMBOL if folded else {**CATEGORY_SYMBOL, **CATEGORY_SYMBOL_PLAIN}).get(category)
    if sym is None or not os.path.exists(TRAFFIC_FILE):
        return None
    for line in open(TRAFFIC_FILE):
        if line.startswith("| `" + sym + " ("):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            try:
                return {"fetch_MB": float(cells[2]), "write_MB": float(cells[3]), "unit": "MB per launch",
                        "source": "profiles/spec_round_xl2_512_hbm_traffic.md (rocprofv3 --pmc, copy-kernel scaled)"}
            except (ValueError, IndexError):
                return None
    return None


def bench_round(args):
    import torch
    from paper_2511_20390_amd import binding, synth
    cfg = synth.dit_config(args.config)
    K, scale, mode = args.K, args.cfg_scale, args.mode
    B = K * (2 if scale > 1 else 1)
    t0 = time.time()
    w = synth.make_weights(cfg, seed=0, bf16_values=(mode == "bf16"))
    model = binding.FreeDit(cfg, w, mode)
    cx, ce, sg = binding.free_ddpm_schedule()
    ri = synth.make_round_inputs(cfg, K, seed=0, sigma_table=sg, draft_noise=0.1)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    a = dict(x_states=dev(ri["x_states"]), x_last=dev(ri["x_last"]), m_draft=dev(ri["m_draft"]), t=dev(ri["t"]),
             coef_x=dev(cx[ri["t"]].astype(np.float32)), coef_eps=dev(ce[ri["t"]].astype(np.float32)),
             sigma=dev(ri["sigma"]), u=dev(ri["u"]), lam=dev(ri["lam"]))
    out = model.spec_round(a["x_states"], a["x_last"], a["m_draft"], a["t"], ri["y"], scale, a["coef_x"],
                           a["coef_eps"], a["sigma"], a["u"], a["lam"] if args.relaxed else None)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def step():
        model.spec_round(a["x_states"], a["x_last"], a["m_draft"], a["t"], ri["y"], scale, a["coef_x"],
                         a["coef_eps"], a["sigma"], a["u"], a["lam"] if args.relaxed else None, out=out)

    if args.draft_only:
        res = {"drafting": bench_draft(args, cfg, model, ri, (cx, ce, sg), a, step)}
        model.close()
        return res, cfg, w, ri, (cx, ce, sg)

    # set-up, untimed: --streams 0 asks the library to time the schedules (one, two, three streams) of the block stack on these inputs
    # (free_dit_tune, a blocking call outside the hot path) and to keep the faster one for this batch size
    tp = torch.cat([a["t"], a["t"]]) if B == 2 * K else a["t"]
    yp = torch.tensor([ri["y"]] * K + [cfg["num_classes"]] * (B - K), dtype=torch.int32, device="cuda:0")
    xp = torch.cat([a["x_states"], a["x_states"]]) if B == 2 * K else a["x_states"]
    if args.ln_fold != "auto":
        model.set_ln_fold({"off": binding.LN_FOLD_OFF, "require": binding.LN_FOLD_REQUIRE}[args.ln_fold])
    model.set_streams(args.streams)
    if args.streams == 0:
        model.tune(xp, tp, yp)
    stream_choice = model.stream_choice(B)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # the same steps with each schedule forced (the per-kernel figures below refer to one stream)
    forced = {}
    for n in (1, 2, 3):
        model.set_streams(n)
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        forced[n] = (time.perf_counter() - t0) * 1e3 / args.steps
    model.set_streams(args.streams)
    ms_one_stream, ms_two_streams, ms_three_streams = forced[1], forced[2], forced[3]

    # per-kernel durations: the same steps again, every launch bracketed by HIP events on its stream
    # (the library runs them in sequence on one stream while it profiles)
    model.profile_begin()
    for _ in range(args.steps):
        step()
    prof = model.profile_end()
    per, total_flops = forward_flops(cfg, B)
    kernels = {}
    for name, (ms, n) in prof.items():
        if n == 0:
            continue
        ent = {"ms_per_step": ms / args.steps, "launches_per_step": n // args.steps, "avg_us": ms * 1e3 / n}
        if name in per:
            ent["tflops"] = per[name] / (ms / n * 1e-3) / 1e12
        kernels[name] = ent
    dom = max((k for k in kernels if k in per), key=lambda k: kernels[k]["ms_per_step"])
    peak = PEAK_BF16_TFLOPS if mode == "bf16" else PEAK_FP32_TFLOPS
    # both modes run the GEMMs and attention on the matrix cores: bf16 against the dense bf16 peak, fp32
    # (v_mfma_f32_32x32x2_f32) against the fp32 matrix peak of 157.3 TFLOP/s (the same figure as the vector peak:
    # 256 CUs x 4 SIMDs x 64 lanes x 2 flop x 2.4 GHz)
    roofline = {"kernel": dom, "bound": "mfma", "achieved": kernels[dom]["tflops"], "peak": peak,
                "unit": "TFLOP/s", "frac": kernels[dom]["tflops"] / peak,
                "traffic": (measured_traffic(dom, bool(model.ln_fold_active(B)))
                            if args.config == "xl2_512" and mode == "bf16" else None),
                "avg_launch_us": kernels[dom]["avg_us"],
                "measured": "HIP events around every launch of this kernel, same steps repeated right after the "
                            "timed region with all kernels in sequence on one stream"}
    if mode == "bf16" and not args.no_mfma_calibration:
        # what a register-only MFMA loop sustains on this device right now, and at which shader clock: the
        # published peak assumes the 2.4 GHz peak clock, which a chip under matrix load does not hold
        cal = binding.mfma_ceiling(200000)
        roofline["mfma_calibration"] = {"register_only_loop_tflops": cal["tflops"],
                                        "shader_clock_mhz": cal["shader_clock_mhz"],
                                        "frac_of_calibrated": kernels[dom]["tflops"] / cal["tflops"]}
    ln_folded = bool(model.ln_fold_active(B))
    roofline["note"] = ("the LayerNorms of the blocks are folded into the GEMMs: this kernel's time includes writing the "
                        "next LayerNorm's input and row sums" if ln_folded and dom in ("gemm_fc2", "gemm_proj") else
                        "the LayerNorms of the blocks are folded into the GEMMs: this kernel's time includes applying one"
                        if ln_folded else "separate LayerNorm kernel")
    ln_separate = None
    if ln_folded:
        # the same steps with the separate LayerNorm kernel, for the per-kernel comparison (not part of `value`)
        model.set_ln_fold(binding.LN_FOLD_OFF)
        model.set_streams(1)
        step()
        model.profile_begin()
        for _ in range(args.steps):
            step()
        prof_off = model.profile_end()
        model.set_ln_fold(binding.LN_FOLD_AUTO if args.ln_fold == "auto" else binding.LN_FOLD_REQUIRE)
        model.set_streams(args.streams)
        ln_separate = {name: {"avg_us": ms * 1e3 / n, "launches_per_step": n // args.steps,
                              **({"tflops": per[name] / (ms / n * 1e-3) / 1e12} if name in per else {})}
                       for name, (ms, n) in prof_off.items() if n}
    fwd_ms = sum(v["ms_per_step"] for k, v in kernels.items() if not k.startswith("verify") and k != "eps_to_mean")
    res = {
        "ms_per_step": ms_per_step, "ms_per_step_one_stream": ms_one_stream, "ms_per_step_two_streams": ms_two_streams,
        "ms_per_step_three_streams": ms_three_streams,
        "batch_streams": args.streams, "stream_choice": stream_choice, "kernels": kernels, "roofline": roofline,
        "ln_folded": ln_folded, "kernels_with_separate_layer_norm": ln_separate,
        "forward": {"algorithmic_tflop": total_flops / 1e12, "ms_sum_of_kernels": fwd_ms,
                    "tflops_whole_step": total_flops / (ms_per_step * 1e-3) / 1e12,
                    "frac_of_peak_whole_step": total_flops / (ms_per_step * 1e-3) / 1e12 / peak},
        "tokens_per_round": B * synth.n_tokens(cfg), "setup_s": setup_s,
        "n_accept": int(out["n_accept"].item()), "B": B,
    }
    if not args.no_draft_bench:
        res["drafting"] = bench_draft(args, cfg, model, ri, (cx, ce, sg), a, step)
    model.close()
    return res, cfg, w, ri, (cx, ce, sg)


def bench_draft(args, cfg, model, ri, sched, a, verify_step):
    """The step before the hot path (Alg. 1, drafting loop): K sequential drafter evaluations on the
    reference state and the propagated feature (two samples with guidance), then the same followed
    by the verification round that consumes the drafts."""
    import torch
    from paper_2511_20390_amd import binding, synth
    K, scale = args.K, args.cfg_scale
    dup = 2 if scale > 1 else 1
    cx, ce, sg = sched
    wd = synth.make_drafter_weights(cfg, 1, seed=1, bf16_values=(args.mode == "bf16"))
    drafter = binding.FreeDrafter(model, wd, 1)
    di = synth.make_draft_inputs(cfg, K, 0, scale, t0=int(ri["t"][0]))
    dev = lambda v: torch.from_numpy(np.ascontiguousarray(v)).to("cuda:0")
    x_a, f_a, xi = dev(di["x_a"]), dev(di["f_a"]), dev(di["xi"])
    out = drafter.draft_round(x_a, f_a, a["t"], ri["y"], scale, a["coef_x"], a["coef_eps"], a["sigma"], xi)

    def draft():
        drafter.draft_round(x_a, f_a, a["t"], ri["y"], scale, a["coef_x"], a["coef_eps"], a["sigma"], xi, out=out)

    def timed(fn, n):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    ms_draft = timed(draft, args.steps)
    ms_both = timed(lambda: (draft(), verify_step()), args.steps)
    N, D, F = synth.n_tokens(cfg), cfg["hidden"], cfg["mlp_hidden"]
    M = dup * N
    per, _ = forward_flops(cfg, dup)
    flops_step = sum(per.values()) + 2.0 * M * D * 2 * D + 2.0 * dup * D * 8 * D
    drafter.close()
    return {"workload": f"draft_round: {K} sequential drafter steps (1 block, {dup} samples x {N} tokens)",
            "ms_per_draft_round": ms_draft, "us_per_drafter_step": ms_draft * 1e3 / K,
            "gflop_per_step": flops_step / 1e9, "tflops": flops_step * K / (ms_draft * 1e-3) / 1e12,
            "ms_draft_plus_verify_round": ms_both,
            "drafter_params_M": sum(int(np.prod(sh)) for _, sh in synth.drafter_weight_spec(cfg, 1)) / 1e6}


def bench_verify(args, n_sets=6):
    """spec_verify alone at 64 x 6 x 16384 fp32, rotating over n_sets distinct input sets
    (> 256 MB in total) so that the Infinity Cache cannot stand in for HBM.  A call is two launches: the
    streaming kernel (verify_partial_kernel, the dominant one: 12 bytes per latent element and draft) and
    the finishing kernel (decisions + reflected samples).  Per-launch durations come from the library's
    benchmark variant of the call, which brackets both launches with HIP events on the launch stream;
    whole calls are also timed back to back with events before and after every call."""
    import torch
    from paper_2511_20390_amd import binding, synth
    n_traj, K, d = 64, 6, 16384
    _, _, sg = binding.free_ddpm_schedule()
    blocker = torch.ones(256 << 20, device="cuda:0", dtype=torch.float32)       # 1 GiB: a copy takes ~0.4 ms
    blocker_out = torch.empty_like(blocker)

    def event_us(calls):
        """Time of every call from events recorded before the first and after every call."""
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)]
        torch.cuda.synchronize()
        # a few milliseconds of unrelated device work first: the host then enqueues all the calls while the
        # device is still busy, so the events measure the device, not the time Python takes between calls
        for _ in range(6):
            torch.mul(blocker, 1.0, out=blocker_out)
        ev[0].record()
        for i, c in enumerate(calls):
            c()
            ev[i + 1].record()
        torch.cuda.synchronize()
        return sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(len(calls)))

    def timed_us(call_args, out, ws, reps):
        """(streaming launch, finishing launch) microseconds per call, by events inside the call.  The timed
        variant blocks, so the device would idle between samples and the first launch after an idle spell is
        slower (14.0 us mean with an 18 us tail against 13.8): every sample therefore queues a 0.4 ms copy and
        three untimed calls on other input sets ahead of the timed one, which then meets the device as
        back-to-back calls do."""
        a, b = [], []
        n = len(call_args)
        for _ in range(reps):
            for i, ca in enumerate(call_args):
                torch.mul(blocker, 1.0, out=blocker_out)
                for j in range(3):
                    binding.spec_verify(*call_args[(i + 1 + j) % n], out=out, workspace=ws)
                r = binding.spec_verify(*ca, out=out, workspace=ws, timed=True)
                a.append(r["stream_us"])
                b.append(r["finish_us"])
        return sum(a) / len(a), sum(b) / len(b), sorted(a)[len(a) // 2]

    sets = []
    for i in range(n_sets):
        vi = synth.make_verify_inputs(n_traj, K, d, 0.01, 100 + i, sg)
        sets.append([torch.from_numpy(vi[k]).to("cuda:0") for k in ("m_target", "m_draft", "x_draft", "sigma", "u")])
    out = binding.spec_verify(*sets[0])
    ws = torch.empty(binding.spec_verify_workspace_bytes(n_traj, K, d), dtype=torch.uint8, device="cuda:0")
    reps = 8
    rot = [lambda i=i: binding.spec_verify(*sets[i], out=out, workspace=ws) for _ in range(reps) for i in range(n_sets)]
    for c in rot[:n_sets]:
        c()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for c in rot:
        c()
    torch.cuda.synchronize()
    host_call_us = (time.perf_counter() - t0) * 1e6 / len(rot)
    us = event_us(rot)
    call_us = sum(us) / len(us)
    stream_us, finish_us, stream_med = timed_us(sets, out, ws, reps)
    warm_us, _, _ = timed_us(sets[:1], out, ws, reps * n_sets)
    nrej = int((out["n_accept"] < K).sum().item())
    # the same kernel on a problem large enough to leave the launch ramp behind: 384 trajectories (453 MB)
    nl = 384
    vl = synth.make_verify_inputs(nl, K, d, 0.01, 200, sg)
    big = [torch.from_numpy(vl[k]).to("cuda:0") for k in ("m_target", "m_draft", "x_draft", "sigma", "u")]
    out_l = binding.spec_verify(*big)
    ws_l = torch.empty(binding.spec_verify_workspace_bytes(nl, K, d), dtype=torch.uint8, device="cuda:0")
    large_us, _, _ = timed_us([big], out_l, ws_l, 8)
    del big, out_l, ws_l
    bytes_stream = n_traj * K * 3 * d * 4            # 12 bytes per latent element and draft
    bytes_reflect = nrej * 4 * d * 4                 # + 16 bytes per element of a rejected draft
    gbs = bytes_stream / (stream_us * 1e-6) / 1e9
    return {"kernel": "verify_partial_kernel", "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": gbs / PEAK_HBM_GBS, "traffic": measured_traffic("verify_partial"), "avg_launch_us": stream_us,
            "median_launch_us": stream_med,
            "measured": "HIP events on the launch stream around each of the call's two launches, 6 rotating input sets",
            "finish_avg_us": finish_us, "warm_cache_GBs": bytes_stream / (warm_us * 1e-6) / 1e9,
            "GBs_at_384_trajectories_453MB": nl * K * 3 * d * 4 / (large_us * 1e-6) / 1e9,
            "whole_call": {"avg_us": call_us, "median_us": us[len(us) // 2],
                           "algorithmic_bytes": bytes_stream + bytes_reflect,
                           "GBs": (bytes_stream + bytes_reflect) / (call_us * 1e-6) / 1e9,
                           "frac": (bytes_stream + bytes_reflect) / (call_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
                           "measured": "events before and after every call, calls enqueued back to back"},
            "host_call_us_back_to_back": host_call_us, "rounds_per_s_64traj": 64e6 / max(call_us, host_call_us),
            "algorithmic_bytes": bytes_stream, "reflected_rows": nrej,
            "workload": "64 traj x 6 drafts x 16384 fp32, 6 rotating input sets (453 MB)"}


def _nanmean0(a):
    """Column means ignoring NaN; NaN where a column has no value."""
    cnt = (~np.isnan(a)).sum(axis=0)
    return np.where(cnt > 0, np.nansum(a, axis=0) / np.maximum(cnt, 1), np.nan)


def bench_loop(args):
    """The whole sampler (Alg. 1) at the DiT-XL/2 512^2 shape: 250 respaced DDPM steps, guidance 4.0,
    6 drafts per round, two-block drafter, random-init target and drafter, strict and relaxed rule,
    beside 250 sequential target steps run through the same entry point (n_spec = 0)."""
    import torch
    from paper_2511_20390_amd import binding, synth
    cfg = synth.dit_config(args.config)
    mode, scale, L, S, depth = args.mode, args.cfg_scale, args.K, args.loop_steps, 2
    w = synth.make_weights(cfg, seed=0, bf16_values=(mode == "bf16"))
    model = binding.FreeDit(cfg, w, mode)
    wd = synth.make_drafter_weights(cfg, depth, seed=1, bf16_values=(mode == "bf16"))
    drafter = binding.FreeDrafter(model, wd, depth)
    # respaced schedule: S of the 1000 timesteps, evenly spaced, each transition with the coefficients of its
    # own timestep (the library takes them as inputs); the last step is noise-free and never speculated
    cx, ce, sg = binding.free_ddpm_schedule()
    tmap = np.linspace(999, 0, S).round().astype(np.int32)
    sigma = sg[tmap].astype(np.float32)
    sigma[-1] = 0.0
    dev = lambda v: torch.from_numpy(np.ascontiguousarray(v)).to("cuda:0")
    rng = np.random.default_rng(0)
    d = synth.latent_dim(cfg)
    a = dict(tmap=dev(tmap), cx=dev(cx[tmap].astype(np.float32)), ce=dev(ce[tmap].astype(np.float32)), sigma=dev(sigma),
             lam=dev(synth.relaxation_profile(tmap)))
    res = {"workload": f"free_sample: DiT-XL/2 {args.config}, {S} steps, guidance {scale}, {L} drafts per round, "
                       f"{depth}-block drafter, random-init weights, {args.loop_images} image(s) per mode",
           "modes": {}}

    def run(n_spec, lam):
        tot = dict(target_calls=0, rounds=0, accepted=0, drafter_steps=0)
        t_wall = 0.0
        for img in range(args.loop_images):
            x0 = dev(rng.standard_normal((cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]), dtype=np.float32))
            xi = dev(rng.standard_normal((S, d), dtype=np.float32))
            u = dev(rng.random(S, dtype=np.float32))
            y = int(rng.integers(0, cfg["num_classes"]))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            _, st, _ = binding.free_sample(drafter, x0, y, scale, n_spec, L, a["tmap"], a["cx"], a["ce"], a["sigma"], xi, u, lam)
            t_wall += time.perf_counter() - t0
            for k in tot:
                tot[k] += st[k]
        n = args.loop_images
        out = {"wall_s_per_image": t_wall / n, "target_calls_per_image": tot["target_calls"] / n,
               "rounds_per_image": tot["rounds"] / n,
               "mean_accepted_per_round": tot["accepted"] / max(1, tot["rounds"])}
        return out

    def run_self(lam):
        """Frozen-target drafting (the target's latest noise estimate reused for the next L steps)."""
        tot = dict(target_calls=0, rounds=0, accepted=0, drafter_steps=0)
        t_wall, deltas = 0.0, []
        for img in range(args.loop_images):
            x0 = dev(rng.standard_normal((cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]), dtype=np.float32))
            xi = dev(rng.standard_normal((S, d), dtype=np.float32))
            u = dev(rng.random(S, dtype=np.float32))
            y = int(rng.integers(0, cfg["num_classes"]))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            _, st, _, delta, acc = binding.free_self_speculative(model, x0, y, scale, S - 1, L, a["tmap"], a["cx"], a["ce"],
                                                                 a["sigma"], xi, u, lam)
            t_wall += time.perf_counter() - t0
            deltas.append(delta)
            for k in tot:
                tot[k] += st[k]
        n = args.loop_images
        return {"wall_s_per_image": t_wall / n, "target_calls_per_image": tot["target_calls"] / n,
                "rounds_per_image": tot["rounds"] / n,
                "mean_accepted_per_round": tot["accepted"] / max(1, tot["rounds"])}, _nanmean0(np.stack(deltas))

    # set-up, untimed: let the library time its schedules for the packed batch of a full round (free_dit_tune)
    Bp = L * (2 if scale > 1.0 else 1)
    xt = dev(rng.standard_normal((Bp, cfg["in_ch"], cfg["lat_h"], cfg["lat_w"]), dtype=np.float32))
    model.tune(xt, dev(np.full(Bp, 500, np.int32)), dev(np.full(Bp, 1, np.int32)))
    res["stream_choice"] = model.stream_choice(Bp)
    run(0, None)                                      # warm-up (also sizes the workspaces)
    res["modes"]["sequential"] = run(0, None)
    res["modes"]["free"] = run(S - 1, None)
    res["modes"]["free_relax"] = run(S - 1, a["lam"])
    # Sec. 3.4: offline self-speculative run -> deviation curve -> relaxation profile -> relaxed run with it
    with np.errstate(all="ignore"):
        res["modes"]["self_speculative"], delta = run_self(None)
        lam_fit = binding.free_lambda_profile(delta, 9)
        res["modes"]["self_speculative_relax"], _ = run_self(dev(lam_fit))
    q = np.linspace(0, S - 1, 6).round().astype(int)
    res["fitted_profile"] = {"steps": q.tolist(), "lambda": [float(lam_fit[i]) for i in q],
                             "eps_delta_measured": [None if np.isnan(delta[i]) else float(delta[i]) for i in q]}
    for k in ("self_speculative", "self_speculative_relax"):
        res["modes"][k]["speedup_vs_sequential"] = res["modes"]["sequential"]["wall_s_per_image"] / res["modes"][k]["wall_s_per_image"]
    seq = res["modes"]["sequential"]["wall_s_per_image"]
    for k in ("free", "free_relax"):
        res["modes"][k]["speedup_vs_sequential"] = seq / res["modes"][k]["wall_s_per_image"]
    # cost model from the measured pieces: a round = drafting + one packed forward, advancing tau + 1 steps
    r = res["modes"]["free"]
    t_round = r["wall_s_per_image"] / max(1.0, r["rounds_per_image"] + 2)
    t_step = seq / S
    res["cost_model"] = {"s_per_round_incl_drafting": t_round, "s_per_sequential_step": t_step,
                         "speedup_at_mean_accepted": {str(tau): (tau + 1) * t_step / t_round for tau in (0, 1, 2, 3, 4, 5)},
                         "note": "with random-init weights the drafter is unrelated to the target, so the measured "
                                 "acceptance says nothing about the method; the model gives the wall-time ratio a "
                                 "trained drafter with mean accepted length tau per round would obtain on these kernels"}
    drafter.close()
    model.close()
    return res


def cpu_baseline(cfg, w, ri, sched, args):
    """The oracle on the host cores: one of the K packed states (with its null-label twin under
    guidance: 2 of the 12 forwards) plus the verification of one draft, scaled to a round."""
    from oracle import free_oracle as fo
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    cx, ce, sg = sched
    t = ri["t"][:1]
    t0 = time.perf_counter()
    fo.spec_round(w, cfg, ri["x_states"][:1], ri["x_states"][1], ri["m_draft"][:1], t, ri["y"], args.cfg_scale,
                  cx[t], ce[t], ri["sigma"][:1], ri["u"][:1], None)
    dt = time.perf_counter() - t0
    per_round = dt * args.K
    return {"value": 1.0 / per_round, "unit": "rounds/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 of {args.K} packed states (2 of {2 * args.K} DiT forwards + 1 draft verified) in "
                      f"{dt:.1f} s, scaled x{args.K}", "seconds_per_round_scaled": per_round}


def bench_gemm(args):
    """One linear layer of the given shape on seeded normal data (weights scaled by K^-1/2), timed with
    events on the launch stream."""
    import torch
    from paper_2511_20390_amd import binding
    M, N, K, epi = (int(v) for v in args.gemm_only.split(","))
    g = torch.Generator(device="cuda").manual_seed(0)
    dt = torch.bfloat16 if args.mode == "bf16" else torch.float32
    X = torch.randn(M, K, device="cuda", generator=g).to(dt)
    W = (torch.randn(N, K, device="cuda", generator=g) / K ** 0.5).to(dt)
    bias = torch.randn(N, device="cuda", generator=g)
    resid = torch.zeros(M, N, device="cuda") if epi == 2 else None
    gate = torch.randn(1, N, device="cuda", generator=g) if epi == 2 else None

    def run():
        binding.op_linear(X, W, bias, args.mode, epi, resid=resid, gate=gate, rows_per_sample=M)

    for _ in range(args.warmup):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / args.steps
    return {"metric": "one linear layer", "unit": "us", "value": us, "higher_is_better": False, "n_gpus": 1,
            "dtype": args.mode, "data": "synthetic", "steps": args.steps, "warmup": args.warmup,
            "config": {"workload": f"linear {M} x {N} x {K}, epilogue {epi}"},
            "tflops": 2.0 * M * N * K / us / 1e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="xl2_512")
    ap.add_argument("--mode", default="bf16", choices=["bf16", "fp32"])
    ap.add_argument("--K", type=int, default=6)
    ap.add_argument("--cfg-scale", type=float, default=4.0)
    ap.add_argument("--relaxed", action="store_true")
    ap.add_argument("--ln-fold", default="auto", choices=["auto", "off", "require"],
                    help="LayerNorm folded into the GEMMs around it (bf16): the library's rule, never, or always")
    ap.add_argument("--streams", type=int, default=0, choices=[0, 1, 2, 3],
                    help="0: free_dit_tune times the schedules in the set-up and the faster one is kept; "
                         "2 / 3: the halves / thirds of the packed batch run concurrently on as many streams; "
                         "1: every kernel in sequence on one stream (use this under rocprofv3 --kernel-trace so "
                         "that kernel durations are not inflated by overlap)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-verify-bench", action="store_true")
    ap.add_argument("--no-mfma-calibration", action="store_true",
                    help="skip the register-only MFMA loop that reports the device's sustained matrix rate and clock")
    ap.add_argument("--no-draft-bench", action="store_true")
    ap.add_argument("--draft-only", action="store_true",
                    help="time only the drafting round (the step before the hot path), e.g. under rocprofv3")
    ap.add_argument("--gemm-only", default=None, metavar="M,N,K,EPI",
                    help="time one linear layer out = epilogue(X W^T + b) of the given shape through the C ABI "
                         "(EPI 0: bias, 1: bias + GELU, 2: gated fp32 residual update), e.g. under rocprofv3")
    ap.add_argument("--verify-only", action="store_true",
                    help="time only spec_verify at 64 x 6 x 16384 (the HBM roofline), e.g. under rocprofv3")
    ap.add_argument("--loop", action="store_true", help="time the whole sampler (Alg. 1) instead of the verification round")
    ap.add_argument("--loop-steps", type=int, default=250)
    ap.add_argument("--loop-images", type=int, default=1)
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run plain device copies of a known size (256 MiB) so that a rocprofv3 --pmc "
                         "run of this command has a reference for scaling FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the packed states of a round share one device); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2511_20390_amd import binding
    binding.load()          # fails loudly when the HIP library is missing
    torch.cuda.set_device(0)

    if args.pmc_calibration:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(4):
            torch.mul(src, 1.0, out=dst)      # one elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    if args.gemm_only:
        print(json.dumps(bench_gemm(args)))
        return
    if args.verify_only:
        r = bench_verify(args)
        print(json.dumps({"metric": "spec_verify call", "unit": "us", "value": r["avg_launch_us"], "higher_is_better": False,
                          "n_gpus": 1, "dtype": "f32", "data": "synthetic", "config": {"workload": r["workload"]},
                          "roofline": r}))
        return
    if args.loop:
        print(json.dumps({"metric": "whole sampler (Alg. 1), wall time per image", "unit": "s", "n_gpus": 1,
                          "dtype": args.mode, "data": "synthetic", "higher_is_better": False, **bench_loop(args)}))
        return
    res, cfg, w, ri, sched = bench_round(args)
    if args.draft_only:
        print(json.dumps({"metric": "drafting round (K sequential drafter steps)", "unit": "ms", "n_gpus": 1,
                          "dtype": args.mode, "data": "synthetic", "higher_is_better": False,
                          "value": res["drafting"]["ms_per_draft_round"], **res["drafting"]}))
        return
    rounds_per_s = 1e3 / res["ms_per_step"]
    line = {
        "metric": "packed DiT-XL/2 verify rounds/s at 512^2 (K=6)", "value": rounds_per_s, "unit": "rounds/s",
        "tokens_per_s": rounds_per_s * res["tokens_per_round"],
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.mode, "data": "synthetic",
        "config": {"workload": f"spec_round: DiT-XL/2 {args.config} latent, K={args.K} drafts, "
                               f"guidance {args.cfg_scale} (packed batch {res['B']}, {res['tokens_per_round']} tokens), "
                               f"{'relaxed' if args.relaxed else 'strict'} rule",
                   "packed_batch": res["B"], "tokens": res["tokens_per_round"]},
        "batch_streams": res["batch_streams"], "stream_choice": res["stream_choice"], "ms_per_step_one_stream": res["ms_per_step_one_stream"],
        "ms_per_step_two_streams": res["ms_per_step_two_streams"],
        "ms_per_step_three_streams": res["ms_per_step_three_streams"],
        "roofline": res["roofline"], "forward": res["forward"], "kernels": res["kernels"],
        "ln_folded": res["ln_folded"], "kernels_with_separate_layer_norm": res["kernels_with_separate_layer_norm"],
    }
    if "drafting" in res:
        line["drafting"] = res["drafting"]
    if not args.no_verify_bench:
        line["roofline_verify"] = bench_verify(args)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, w, ri, sched, args)
        line["cpu_baseline"]["gpu_over_cpu"] = rounds_per_s / line["cpu_baseline"]["value"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
