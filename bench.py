#!/usr/bin/env python3
"""Benchmark of the Nature-CNN hot path on one MI355X.

A step is one pass of the whole training hot path (forward, objective,
backward, ordered gradient reduction) over one synthetic batch that is already
resident in HBM: the A2C gradient step at B=2048 (256 envs x 8-step rollouts).
Prints ONE JSON line: whole-step throughput, the roofline of the longest kernel (event-timed in this run, HBM
traffic from the stored counter profile) and the CPU oracle's rate on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# algorithmic multiply-accumulates per sample (dense, nothing avoided), A = 18 heads
MACS = {"conv1": 3_276_800, "conv2": 2_654_208, "conv3": 1_806_336, "fc": 1_605_632, "head_pv": 19 * 512}
FWD_FLOPS = 2 * sum(MACS.values())                                  # 18,705,408
FWDBWD_FLOPS = 3 * FWD_FLOPS - 2 * MACS["conv1"]                    # no conv1 input gradient: 49,562,624
KERNEL_FLOPS = {  # per sample, by instrumented kernel name
    "conv1_fwd": 2 * MACS["conv1"], "conv2_fwd": 2 * MACS["conv2"], "conv3_fwd": 2 * MACS["conv3"],
    "fc_fwd": 2 * MACS["fc"], "head_fwd": 2 * MACS["head_pv"],
    "conv23_fwd": 2 * MACS["conv2"] + 2 * MACS["conv3"],   # conv2 and conv3 forward, one kernel (act2 through LDS)
    "conv123_fwd": 2 * MACS["conv1"] + 2 * MACS["conv2"] + 2 * MACS["conv3"],   # ... with conv1 ahead of them in each workgroup
    "conv1_wgrad": 2 * MACS["conv1"], "conv2_wgrad": 2 * MACS["conv2"], "conv3_wgrad": 2 * MACS["conv3"],
    "fc_wgrad": 2 * MACS["fc"], "head_wgrad": 2 * MACS["head_pv"],
    "conv2_dgrad": 2 * MACS["conv2"], "conv3_dgrad": 2 * MACS["conv3"], "fc_dgrad": 2 * MACS["fc"],
    "head_dgrad": 2 * MACS["head_pv"],
    # conv2 input gradient + conv1 weight gradient + conv2 and conv3 weight gradients, one launch
    "conv_bwd": 2 * MACS["conv2"] + 2 * MACS["conv1"] + 2 * MACS["conv2"] + 2 * MACS["conv3"],
}
# algorithmic HBM bytes per sample: every bf16 activation / gradient tensor written once and read once,
# observations read as uint8 (weights and the flat gradient are per-launch constants, added below)
ACT = {"obs": 28224, "a1": 25600, "a2": 10368, "a3": 6272, "h": 1024, "z": 76}
KERNEL_BYTES = {
    "conv1_fwd": ACT["obs"] + ACT["a1"], "conv2_fwd": ACT["a1"] + ACT["a2"], "conv3_fwd": ACT["a2"] + ACT["a3"],
    "fc_fwd": ACT["a3"] + ACT["h"], "head_fwd": ACT["h"] + ACT["z"],
    "conv23_fwd": ACT["a1"] + ACT["a2"] + ACT["a3"],       # act2 is written once, for the backward pass
    "conv123_fwd": ACT["obs"] + 2 * ACT["a1"] + ACT["a2"] + ACT["a3"],
    "conv1_wgrad": ACT["obs"] + ACT["a1"], "conv2_wgrad": ACT["a1"] + ACT["a2"], "conv3_wgrad": ACT["a2"] + ACT["a3"],
    "fc_wgrad": ACT["a3"] + ACT["h"], "head_wgrad": ACT["h"] + ACT["z"],
    "conv2_dgrad": ACT["a2"] + 2 * ACT["a1"], "conv3_dgrad": ACT["a3"] + 2 * ACT["a2"],
    "fc_dgrad": ACT["h"] + 2 * ACT["a3"], "head_dgrad": ACT["z"] + 2 * ACT["h"],
    # d(pre1) stays on chip; d(pre2) is read by two of the three parts
    "conv_bwd": ACT["a2"] + ACT["obs"] + ACT["a1"] + ACT["a2"] + ACT["a2"] + ACT["a3"],
}
KERNEL_BYTES_PER_LAUNCH = {  # bf16 weights read (forward / input gradient) or fp32 gradient written (weight gradient)
    "conv1_fwd": 2 * 8192, "conv2_fwd": 2 * 32768, "conv3_fwd": 2 * 36864, "conv23_fwd": 2 * 32768 + 2 * 36864, "conv123_fwd": 2 * 8192 + 2 * 32768 + 2 * 36864, "fc_fwd": 2 * 1605632, "head_fwd": 2 * 9728,
    "conv2_dgrad": 2 * 32768, "conv3_dgrad": 2 * 36864, "fc_dgrad": 2 * 1605632, "head_dgrad": 2 * 9728,
    "conv1_wgrad": 4 * 8192, "conv2_wgrad": 4 * 32768, "conv3_wgrad": 4 * 36864, "fc_wgrad": 4 * 1605632,
    "head_wgrad": 4 * 9728, "conv_bwd": 2 * 32768 + 4 * 8192 + 4 * 32768 + 4 * 36864,
}
# whole step, per sample: the forward's bytes, then observations again, saved activations once, and every
# activation gradient written and read once
FWDBWD_BYTES = sum(KERNEL_BYTES[k] for k in ("conv1_fwd", "conv2_fwd", "conv3_fwd", "fc_fwd", "head_fwd")) \
    + ACT["obs"] + (ACT["a1"] + ACT["a2"] + ACT["a3"] + ACT["h"]) + 2 * (ACT["a1"] + ACT["a2"] + ACT["a3"] + ACT["h"])
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
SETTLE_S = 0.25             # seconds the device is driven before the timed steps (see workload_report)


def per_step_event_ms(torch, fn, steps):
    """Duration of each of `steps` calls, from an event pair around every call on the current stream (the calls
    are issued back to back; a call's duration is the time from the previous call's end to its own)."""
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(steps):
        fn()
        evs[i + 1].record()
    torch.cuda.synchronize()
    return [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]


def wall_ms(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def kernel_profile(arn, torch, step, steps):
    """(average us per launch, launches per step) by instrumented kernel name over `steps` more steps, with the
    event pair's own contribution (a pair around nothing, once per step) subtracted."""
    stream = torch.cuda.current_stream()
    arn.profile_enable(True)
    for _ in range(steps):
        step()
        arn.profile_null(stream)
    torch.cuda.synchronize()
    per = {}
    for name, ms in arn.profile_collect(cap=128 * steps + 64):
        tot, cnt = per.get(name, (0.0, 0))
        per[name] = (tot + ms, cnt + 1)
    arn.profile_enable(False)
    null_ms = per.pop("null")[0] / steps
    avg_us = {n: max(t / c - null_ms, 0.0) * 1e3 for n, (t, c) in per.items()}
    calls = {n: c / steps for n, (t, c) in per.items()}
    return avg_us, calls, null_ms * 1e3


def roofline_of(avg_us, B, kernel_flops, kernel_bytes, bytes_per_launch, tag):
    """Roofline of the kernel with the largest average launch duration among those with a byte / flop model:
    algorithmic bytes (or flops) per launch over its event-timed duration, against the published peak of the
    resource whose time at peak is larger."""
    known = [n for n in avg_us if n in kernel_flops]
    dominant = max(known, key=avg_us.get)
    dom_s = avg_us[dominant] * 1e-6
    dom_flops = kernel_flops[dominant] * B
    dom_bytes = kernel_bytes[dominant] * B + bytes_per_launch[dominant]
    if dom_bytes / (PEAK_HBM_GBS * 1e9) >= dom_flops / (PEAK_BF16_TFLOPS * 1e12):
        achieved = dom_bytes / dom_s / 1e9
        r = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": round(achieved / PEAK_HBM_GBS, 4)}
    else:
        achieved = dom_flops / dom_s / 1e12
        r = {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
             "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4)}
    r["traffic"] = measured_traffic(dominant, tag)
    r["traffic_source"] = "profiles/%s_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, see its .md)" % tag \
        if r["traffic"] is not None else None
    r["avg_launch_us"] = round(avg_us[dominant], 2)
    r["algorithmic_bytes_per_launch"] = dom_bytes
    r["algorithmic_flops_per_launch"] = dom_flops
    return r


def measured_traffic(kernel, tag):
    """HBM bytes per launch of `kernel` from the committed counter summary of this workload (written by
    `bench.py --summarise-counters`): FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a
    plain copy of known size; None if no summary covers the workload or the kernel."""
    path = os.path.join(ROOT, "profiles", "%s_traffic.json" % tag)
    try:
        with open(path) as f:
            prof = json.load(f)
    except (OSError, ValueError):
        return None
    return prof.get("hbm_bytes_per_launch", {}).get(kernel)


def head_macs(A, head):
    return (A * 51 if head == "c51" else A + 1) * 512


def flop_models(A, head):
    """Algorithmic flops and HBM bytes per sample (and bytes per launch) by instrumented kernel name."""
    hm = head_macs(A, head)
    flops = dict(KERNEL_FLOPS)
    flops.update({"head_fwd": 2 * hm, "head_wgrad": 2 * hm, "head_dgrad": 2 * hm,
                  "conv_infer": 2 * (MACS["conv1"] + MACS["conv2"] + MACS["conv3"])})
    z = 4 * (A * 51 if head == "c51" else A + 1)
    kb = dict(KERNEL_BYTES)
    kb.update({"head_fwd": ACT["h"] + z, "head_wgrad": ACT["h"] + z // 2, "head_dgrad": z // 2 + 2 * ACT["h"],
               "conv_infer": ACT["obs"] + ACT["a3"]})          # frames in, act3 (fp16) out: nothing else leaves the chip
    per_launch = dict(KERNEL_BYTES_PER_LAUNCH)
    per_launch.update({"head_fwd": 2 * hm, "head_dgrad": 2 * hm, "head_wgrad": 4 * hm,
                       "conv_infer": 2 * 8192 + 2 * 32768 + 2 * 36864})
    return flops, kb, per_launch


def oracle_baseline(np, fn, n, what, budget_s=12.0, max_reps=50):
    """The oracle as it stands on the host cores, repeated for about 10-30 s on a bounded slice of the workload."""
    from oracle import nature_cnn as orc
    reps, t_total = 0, 0.0
    while reps < 1 or (t_total < budget_s and reps < max_reps):
        t0 = time.perf_counter()
        fn()
        t_total += time.perf_counter() - t0
        reps += 1
    return {"value": round(n * reps / t_total, 1), "unit": "samples/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "%s, %d repetitions, %.1f s (rate scales linearly to the full batch)" % (what, reps, t_total)}


def stats_ms(np, xs):
    a = np.asarray(xs, dtype=np.float64)
    return {"mean": round(float(a.mean()), 4), "median": round(float(np.median(a)), 4), "min": round(float(a.min()), 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--dqn", action="store_true",
                    help="report the Double-DQN (dueling head) gradient step and the action-drawing inference "
                         "instead (secondary lines)")
    ap.add_argument("--alternating", action="store_true",
                    help="latency study of the two-group alternating sampler inference, host buffers included "
                         "(secondary line)")
    ap.add_argument("--paper-geometry", action="store_true",
                    help="secondary report: the A2C gradient step and inference on the paper's own 104x80 frames with "
                         "padded conv2/conv3, per-kernel times included")
    ap.add_argument("--a3c-net", action="store_true",
                    help="secondary report: the same on the 2-convolution policy-gradient network (104x80 frames)")
    ap.add_argument("--library-baseline", action="store_true",
                    help="time the same network written with PyTorch's own layers (MIOpen / hipBLASLt) on this GPU: "
                         "context for the A2C step and the forward pass, not part of the product path")
    ap.add_argument("--update-rules", action="store_true",
                    help="report the parameter-update kernels instead (secondary line)")
    ap.add_argument("--workload", type=int, default=3, choices=[1, 2, 3, 4, 5],
                    help="3 (default) = the headline A2C step at B=2048; 1, 2 = inference; 4 = PPO; 5 = C51")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run a plain device-to-device copy of MIB mebibytes a few times (reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--summarise-counters", metavar="DIR",
                    help="no GPU needed: turn the rocprofv3 CSV output under DIR (runs made as profiles/*_traffic.md "
                         "says) into profiles/<tag>_traffic.json/.md, or with --sq into profiles/<tag>_sq_counters.md")
    ap.add_argument("--summarise-stats", metavar="DIR",
                    help="no GPU needed: turn rocprofv3 --kernel-trace --stats output under DIR (bench_kernel_stats.csv and "
                         "log.txt with the bench line) into profiles/<tag>_kernel_stats.md; --cmd gives the command to quote")
    ap.add_argument("--cmd", default="", help="--summarise-stats: the profiled command, quoted in the summary")
    ap.add_argument("--tag", default="", help="workload tag of --summarise-counters output (default: from --workload)")
    ap.add_argument("--sq", action="store_true", help="--summarise-counters: shader-core counters instead of traffic")
    ap.add_argument("--cpu-samples", type=int, default=0, help="oracle sample size (0 = auto, ~10-30 s)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path shards by sample; "
              "one gradient all-reduce per step would follow)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    if args.summarise_stats:
        summarise_stats(args.summarise_stats, args.tag, args.cmd)
        return
    if args.summarise_counters:
        import workloads as wl
        tag = args.tag or wl.WORKLOADS[args.workload]["name"]
        summarise_counters(args.summarise_counters, tag, args.sq)
        return

    import numpy as np
    import torch

    import paper_1803_02811_amd as arn
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    if args.calibrate_copy:
        n = args.calibrate_copy * 1024 * 1024
        src = torch.zeros(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "copies": 5}))
        return
    if args.library_baseline:
        library_baseline_report(args, wl, np, torch)
        return
    if args.update_rules:
        update_rules_report(args, arn, wl, np, torch)
        return
    if args.dqn:
        dqn_report(args, arn, wl, np, torch)
        return
    if args.alternating:
        alternating_report(args, arn, wl, np, torch)
        return
    if args.paper_geometry or args.a3c_net:
        paper_geometry_report(args, arn, wl, np, torch, "a3c" if args.a3c_net else "nature")
        return
    workload_report(args, arn, wl, np, torch)


def workload_report(args, arn, wl, np, torch):
    """One JSON line for workload k: whole-step throughput (wall clock over exactly K steps after W warm-ups),
    per-step median / min, per-kernel event times, the roofline of the longest kernel, and the oracle's rate."""
    dev, k = "cuda:0", args.workload
    w = wl.WORKLOADS[k]
    A, B, head, kind = w["A"], args.batch or w["B"], w["head"], w["kind"]
    cfg = arn.Config(A, arn.ARN_HEAD_PV if head == "pv" else arn.ARN_HEAD_C51)
    flat = wl.he_normal_params(A, head, 2000 + k)
    packed = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev)
    arn.weights_prepare(cfg, torch.from_numpy(flat).to(dev), packed)
    stream = None   # the binding then takes the stream that is current at call time (it differs under graph capture)
    to_dev = lambda d: {n: torch.from_numpy(np.ascontiguousarray(v)).to(dev) for n, v in d.items()}
    conv_macs = MACS["conv1"] + MACS["conv2"] + MACS["conv3"] + MACS["fc"]
    fwd_flops = 2 * (conv_macs + head_macs(A, head))
    tflat = None
    wsf = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_FORWARD), dtype=torch.uint8, device=dev)
    if kind == "forward":
        batch_np = {"obs": wl.frames_for(k, B)}
        obs = torch.from_numpy(batch_np["obs"]).to(dev)
        logits = torch.empty(B, A, dtype=torch.float32, device=dev)
        value = torch.empty(B, dtype=torch.float32, device=dev)
        probs = torch.empty(B, A, dtype=torch.float32, device=dev)
        greedy = torch.empty(B, dtype=torch.int32, device=dev)
        step = lambda: arn.policy_forward(cfg, packed, obs, logits, value, probs, greedy, workspace=wsf, stream=stream)
        flops, bytes_alg, name, dtype = fwd_flops, ACT["obs"] + 4 * (2 * A + 2), "policy_forward", "f16"
        bytes_launch = 2 * (8192 + 32768 + 36864 + 1605632 + head_macs(A, head))      # one fp16 copy of every weight matrix
    else:
        ws = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_TRAIN), dtype=torch.uint8, device=dev)
        dW = torch.empty(arn.param_count(cfg), dtype=torch.float32, device=dev)
        loss = torch.empty(4, dtype=torch.float32, device=dev)
        tgt_flops = 0
        if kind == "c51":
            batch_np = wl.c51_batch(k, B=B)
            batch = to_dev(batch_np)
            tflat = wl.he_normal_params(A, head, 3000 + k)
            tpacked = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev)
            arn.weights_prepare(cfg, torch.from_numpy(tflat).to(dev), tpacked)
            batch["w_target_packed"] = tpacked
            tgt_flops = fwd_flops
        else:
            batch_np = wl.actor_critic_batch(k, B=B, normalise_adv=(kind == "ppo"))
            batch = to_dev(batch_np)
            if kind == "ppo":
                # sampling-policy log-probs: the current logits (from this library) perturbed by N(0, 0.05^2)
                logits = torch.empty(B, A, dtype=torch.float32, device=dev)
                value = torch.empty(B, dtype=torch.float32, device=dev)
                arn.policy_forward(cfg, packed, batch["obs"], logits, value, workspace=wsf, stream=stream)
                noisy = logits + torch.from_numpy(wl.logit_noise(k, B, A).astype(np.float32)).to(dev)
                batch["old_logp"] = torch.log_softmax(noisy, dim=1).gather(1, batch["action"].long()[:, None])[:, 0].contiguous()
                batch_np["old_logp"] = batch["old_logp"].cpu().numpy()
        step = lambda: arn.train_step_grads(cfg, packed, batch, kind, dW, loss, workspace=ws, stream=stream)
        flops = 3 * fwd_flops - 2 * MACS["conv1"] + tgt_flops
        bytes_alg = FWDBWD_BYTES + (sum(KERNEL_BYTES[q] for q in ("conv1_fwd", "conv2_fwd", "conv3_fwd", "fc_fwd")) if kind == "c51" else 0)
        bytes_launch, name, dtype = 0, "train_step_grads:" + kind, "bf16"

    # A process that has just started runs its first few hundred steps 5-10 % slower than it does from then on
    # (every kernel alike: the GPU leaves its idle clocks).  The figure of interest is the rate of a training job,
    # so the device is first driven for SETTLE_S seconds; the rate of the K steps right after the W warm-ups of a
    # fresh process is measured before that and printed too (startup_ms_per_step).
    for _ in range(args.warmup):
        step()
    startup_ms = wall_ms(torch, step, args.steps)
    t0, preroll = time.perf_counter(), 0
    while time.perf_counter() - t0 < SETTLE_S:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
        preroll += 20
    # ---- the contract: W untimed warm-up steps, then exactly K timed steps ----
    for _ in range(args.warmup):
        step()
    ms = wall_ms(torch, step, args.steps)
    value_sps = B / (ms * 1e-3)
    # the same K steps again, each with its own event pair: spread of the step time
    per_step = per_step_event_ms(torch, step, args.steps)

    avg_us, calls, null_us = kernel_profile(arn, torch, step, min(args.steps, 50))
    kflops, kbytes, klaunch = flop_models(A, head)
    roofline = roofline_of(avg_us, B, kflops, kbytes, klaunch, w["name"] if not args.batch else "none")
    roofline["event_pair_overhead_us"] = round(null_us, 2)

    out = {
        "metric": "Nature-CNN samples/sec (%s) at B=%d on 1 GPU" % ("fwd+bwd" if kind != "forward" else "fwd", B),
        "value": round(value_sps, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s (workload %d: %s, A=%d)" % (w["name"], k, name, A), "global_batch": B,
                   "parallelism": "single-gpu"},
        "step_ms": stats_ms(np, per_step),
        "startup_ms_per_step": round(startup_ms, 4), "settle_steps_before_timing": preroll,
        "mfma_frac_whole_step": round(value_sps * flops / 1e12 / PEAK_BF16_TFLOPS, 4),
        "hbm_frac_whole_step": round((bytes_alg * B + bytes_launch) / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        "algorithmic_flops_per_sample": flops,
        "kernel_us": {n: round(v, 2) for n, v in sorted(avg_us.items(), key=lambda kv: -kv[1])},
        "kernel_launches_per_step": {n: round(c, 2) for n, c in calls.items() if c != 1.0},
        "roofline": roofline,
    }

    if kind == "forward":
        # cold figure: a 512 MiB buffer is rewritten between calls, which evicts the L2s and the 256 MiB memory-side
        # cache, so weights and frames come from HBM; each call is timed on its own (warm figure: step_ms above)
        junk = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        cold = []
        for i in range(min(args.steps, 30)):
            junk.fill_(i & 0xff)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            step()
            e1.record()
            torch.cuda.synchronize()
            cold.append(e0.elapsed_time(e1))
        out["cold_cache_call_ms"] = stats_ms(np, cold)
        out["hbm_frac_cold"] = round((bytes_alg * B + bytes_launch) / (float(np.median(cold)) * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
        del junk
        # the same call captured once into a HIP graph and replayed (what a sampler loop that cannot afford the
        # launch gaps of three kernels does; arn_policy_forward_static exists for callers under capture)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(args.warmup):
            g.replay()
        out["graph_replay_ms_per_call"] = round(wall_ms(torch, g.replay, args.steps), 4)
    else:
        # forward-only (action-selection inference, the fp16 single-product path) on the same frames, for the report
        lg = torch.empty(B, A * (51 if head == "c51" else 1), dtype=torch.float32, device=dev)
        vl = torch.empty(B, A if head == "c51" else 1, dtype=torch.float32, device=dev)
        fwd = lambda: arn.policy_forward(cfg, packed, batch["obs"], lg, vl, workspace=wsf, stream=stream)
        for _ in range(args.warmup):
            fwd()
        f_ms = wall_ms(torch, fwd, args.steps)
        out["forward_ms"] = round(f_ms, 4)
        out["forward_samples_per_s"] = round(B / (f_ms * 1e-3), 1)
        if k == 3:
            # the same calls captured once into HIP graphs and replayed
            def graph_time(fn):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    fn()
                for _ in range(args.warmup):
                    g.replay()
                return wall_ms(torch, g.replay, args.steps)
            out["graph_replay_ms_per_step"] = round(graph_time(step), 4)
            out["graph_replay_forward_ms"] = round(graph_time(fwd), 4)

    if not args.no_cpu_baseline:
        from oracle import nature_cnn as orc
        spec = orc.NetSpec(A, head)
        if kind == "forward":
            n = args.cpu_samples or B
            params = orc.unflatten(flat, spec)
            sub = batch_np["obs"][:n]
            out["cpu_baseline"] = oracle_baseline(np, lambda: orc.forward(params, sub, spec), n,
                                                  "forward of the first %d samples of the same batch" % n)
        else:
            n = args.cpu_samples or min(B, 2048 if kind != "c51" else 1024)
            sub = {kk: v[:n] for kk, v in batch_np.items()}
            fn = lambda: orc.train_step_grads(flat, sub, kind, spec, flat_target_params=tflat)
            what = "first %d samples of the same batch, %sforward + objective + backward" % (
                n, "target-network forward + " if kind == "c51" else "")
            out["cpu_baseline"] = oracle_baseline(np, fn, n, what)
    print(json.dumps(out))


# ---------------------------------------------------------------------------
# rocprofv3 counter CSVs -> committed summaries (no GPU needed)
# ---------------------------------------------------------------------------
KERNEL_NAME_PATTERNS = [   # first match wins: mangled or demangled rocprofv3 kernel name -> instrumented launch name
    (r"conv123_fwd_kernel", "conv123_fwd"), (r"conv23_fwd_fused", "conv23_fwd"), (r"infer_conv_(pipelined_)?kernel", "conv_infer"),
    (r"conv_backward_kernel", "conv_bwd"), (r"conv1_fwd_resident", "conv1_fwd"), (r"ResConv2Fwd", "conv2_fwd"),
    (r"ResConv3Fwd", "conv3_fwd"), (r"ResConv3Dgrad", "conv3_dgrad"), (r"FcFwd", "fc_fwd"), (r"FcDgrad", "fc_dgrad"),
    (r"pv_head_kernel<true>|pv_head_kernelILb1", "pv_head"), (r"pv_head_kernel<false>|pv_head_kernelILb0", "pv_head_infer"),
    (r"HeadWgrad", "head_wgrad"), (r"HeadFwdC51", "head_fwd"), (r"HeadDgrad", "head_dgrad"),
    (r"UnmapHeadBias", "head_bias"), (r"UnmapHead", "head_reduce"),
    (r"gemm_tn_kernel.*DenseGather", "fc_wgrad"), (r"fc_reduce", "fc_reduce"), (r"fc_finish", "fc_finish"),
    (r"conv_reduce_kernel", "conv_reduce"), (r"loss_finalize", "loss_finalize"), (r"c51_dist", "c51_dist"),
    (r"c51_loss", "loss"), (r"pack_all", "pack_all"), (r"__amd_rocclr_copyBuffer", "copy"),
]


def summarise_stats(root, tag, cmd):
    """rocprofv3's per-kernel statistics of one profiled bench run as a table, with the same run's bench line."""
    import csv
    import glob
    import re
    src = glob.glob(os.path.join(root, "**", "*_kernel_stats.csv"), recursive=True)
    if not src or not tag:
        raise SystemExit("need --tag and a *_kernel_stats.csv under " + root)

    def short(n):
        n = re.sub(r"void |arn::", "", n)
        n = re.sub(r"\(.*$", "", n)
        return re.sub(r"^_ZN3arn\d+", "", n)[:100]
    md = ["# %s: kernel trace" % tag, "", "Command (on one MI355X, from the repository root):", "", "    " + cmd, "",
          "    python3 bench.py --summarise-stats DIR --tag %s --cmd '...'" % tag, "",
          "Per-kernel summary from rocprofv3's `*_kernel_stats.csv` (durations in microseconds).", "",
          "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    with open(src[0]) as f:
        for r in csv.DictReader(f):
            if float(r["Percentage"]) >= 0.05:
                md.append("| `%s` | %s | %.2f | %.2f | %.2f | %.2f |" % (
                    short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
                    float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
    log = os.path.join(root, "log.txt")
    if os.path.exists(log):
        lines = [x for x in open(log) if x.startswith("{")]
        if lines:
            j = json.loads(lines[-1])
            ku = j.get("kernel_us") or {}
            md += ["", "The same run's bench line (profiler attached): %.1f us per step; its HIP-event durations per launch "
                       "(event-pair overhead subtracted), for comparison with the averages above:" % (j["ms_per_step"] * 1e3), "",
                   ", ".join("%s %.1f" % (n, v) for n, v in ku.items()) + "."]
    path = os.path.join(ROOT, "profiles", "%s_kernel_stats.md" % tag)
    with open(path, "w") as f:
        f.write("\n".join(md) + "\n")
    print("wrote", path)


def _short_kernel_name(k):
    import re
    for pat, n in KERNEL_NAME_PATTERNS:
        if re.search(pat, k):
            return n
    return None


def _counter_means(path):
    """{short kernel name: {counter: mean value per dispatch}} of one rocprofv3 *_counter_collection.csv."""
    import collections
    import csv
    acc = collections.defaultdict(lambda: collections.defaultdict(float))
    cnt = collections.defaultdict(lambda: collections.defaultdict(int))
    with open(path) as f:
        for r in csv.DictReader(f):
            n = _short_kernel_name(r["Kernel_Name"])
            if n is None:
                continue
            acc[n][r["Counter_Name"]] += float(r["Counter_Value"])
            cnt[n][r["Counter_Name"]] += 1
    return {n: {c: acc[n][c] / cnt[n][c] for c in acc[n]} for n in acc}


def _find_csv(root, sub, prefix):
    import glob
    g = glob.glob(os.path.join(root, sub, "**", "%s_counter_collection.csv" % prefix), recursive=True)
    if not g:
        raise SystemExit("no %s_counter_collection.csv under %s/%s" % (prefix, root, sub))
    return g[0]


def summarise_counters(root, tag, sq):
    """DIR layout (what the commands quoted in the written .md produce):
         DIR/FETCH_SIZE/{bench,copy}_counter_collection.csv, DIR/WRITE_SIZE/{bench,copy}_counter_collection.csv
       or, with --sq, DIR/sq_a and DIR/sq_b with pmc_counter_collection.csv."""
    prof = os.path.join(ROOT, "profiles")
    if sq:
        a = _counter_means(_find_csv(root, "sq_a", "pmc"))
        b = _counter_means(_find_csv(root, "sq_b", "pmc"))
        md = ["# %s: shader-core counters per kernel" % tag, "",
              "Commands (one MI355X, repository root; one pass of eight SQ counters each; weight gradients kept on the "
              "caller's stream so that dispatches do not overlap):", "",
              "    ARN_SINGLE_STREAM=1 rocprofv3 --pmc SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_WAIT_INST_ANY SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE -d DIR/sq_a -o pmc --output-format csv -- python3 bench.py <workload flags> --steps 3 --warmup 1 --no-cpu-baseline",
              "    ARN_SINGLE_STREAM=1 rocprofv3 --pmc SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_ACTIVE_INST_ANY SQ_INSTS_LDS SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INST_LEVEL_LDS -d DIR/sq_b -o pmc --output-format csv -- python3 bench.py <workload flags> --steps 3 --warmup 1 --no-cpu-baseline",
              "    python3 bench.py --summarise-counters DIR --sq --tag %s" % tag, "",
              "Per-dispatch averages. SQ_BUSY_CYCLES sums the 32 shader engines, SQ_VALU_MFMA_BUSY_CYCLES the 1024 SIMDs, "
              "SQ_LDS_IDX_ACTIVE the 256 CUs; shares of the wavefronts' resident cycles (SQ_WAVE_CYCLES): waiting at an "
              "s_waitcnt, waiting to issue, issuing. Executed MFMA work = SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 flop.", "",
              "| kernel | busy cycles (per SE) | MFMA pipe busy % | LDS busy % | bank-conflict cycles / LDS active % | s_waitcnt % | wait to issue % | issuing % | executed MFMA GFLOP |",
              "|---|---|---|---|---|---|---|---|---|"]
        rows = []
        for n, c in a.items():
            busy = c.get("SQ_BUSY_CYCLES", 0.0) / 32
            if busy < 100 or n in ("copy", "pack_all"):
                continue
            d = b.get(n, {})
            wc = d.get("SQ_WAVE_CYCLES", 0.0) or float("nan")
            rows.append((busy, "| %s | %s | %.0f | %.0f | %.0f | %.0f | %.0f | %.0f | %.1f |" % (
                n, format(int(busy), ","), c["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024 / busy * 100,
                c["SQ_LDS_IDX_ACTIVE"] / 256 / busy * 100, c["SQ_LDS_BANK_CONFLICT"] / max(c["SQ_LDS_IDX_ACTIVE"], 1) * 100,
                d.get("SQ_WAIT_ANY", 0) / wc * 100, d.get("SQ_WAIT_INST_ANY", 0) / wc * 100,
                d.get("SQ_ACTIVE_INST_ANY", 0) / wc * 100, d.get("SQ_INSTS_VALU_MFMA_MOPS_BF16", 0) * 512 / 1e9)))
        md += [r for _, r in sorted(rows, reverse=True)]
        path = os.path.join(prof, "%s_sq_counters.md" % tag)
        with open(path, "w") as f:
            f.write("\n".join(md) + "\n")
        print("wrote", path)
        return
    fb = _counter_means(_find_csv(root, "FETCH_SIZE", "bench"))
    fc = _counter_means(_find_csv(root, "FETCH_SIZE", "copy"))
    wb = _counter_means(_find_csv(root, "WRITE_SIZE", "bench"))
    wc = _counter_means(_find_csv(root, "WRITE_SIZE", "copy"))
    copy_kib = 256 * 1024
    fs, ws = copy_kib / fc["copy"]["FETCH_SIZE"], copy_kib / wc["copy"]["WRITE_SIZE"]
    rows = []
    for n in fb:
        if n in ("copy", "pack_all"):
            continue
        f_kib, w_kib = fb[n].get("FETCH_SIZE", 0.0), wb.get(n, {}).get("WRITE_SIZE", 0.0)
        rows.append((n, f_kib, w_kib, (f_kib * fs + w_kib * ws) * 1024))
    rows.sort(key=lambda r: -r[3])
    md = ["# %s: HBM traffic per kernel launch" % tag, "",
          "Commands (one MI355X, repository root; weight gradients kept on the caller's stream so that dispatches do not overlap):", "",
          "    ARN_SINGLE_STREAM=1 rocprofv3 --pmc FETCH_SIZE -d DIR/FETCH_SIZE -o bench --output-format csv -- python3 bench.py <workload flags> --steps 3 --warmup 1 --no-cpu-baseline",
          "    rocprofv3 --pmc FETCH_SIZE -d DIR/FETCH_SIZE -o copy --output-format csv -- python3 bench.py --calibrate-copy 256",
          "    (the same two with WRITE_SIZE)",
          "    python3 bench.py --summarise-counters DIR --tag %s" % tag, "",
          "Calibration: a plain 256 MiB device copy reads FETCH_SIZE = %.0f KiB and WRITE_SIZE = %.0f KiB per dispatch, so the "
          "counters are scaled by %.3f (fetch) and %.3f (write). Averages over all dispatches of the run." % (
              fc["copy"]["FETCH_SIZE"], wc["copy"]["WRITE_SIZE"], fs, ws), "",
          "| kernel | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled HBM bytes per launch |", "|---|---|---|---|"]
    md += ["| %s | %.0f | %.0f | %s |" % (n, f_kib, w_kib, format(int(b), ",")) for n, f_kib, w_kib, b in rows]
    with open(os.path.join(prof, "%s_traffic.md" % tag), "w") as f:
        f.write("\n".join(md) + "\n")
    with open(os.path.join(prof, "%s_traffic.json" % tag), "w") as f:
        json.dump({"workload": tag, "fetch_scale": round(fs, 4), "write_scale": round(ws, 4),
                   "hbm_bytes_per_launch": {n: int(b) for n, _, _, b in rows}}, f, indent=1)
    print("wrote profiles/%s_traffic.json and .md" % tag)


def library_baseline_report(args, wl, np, torch):
    """Context line: the Nature CNN with torch.nn layers (the vendor libraries' convolutions and GEMMs, channels-last),
    forward and A2C forward + backward on the workload's frames, in bf16 and fp32.  Nothing of the library under test
    runs here; the figures stand beside bench.py's own lines the way the CPU oracle's do."""
    import torch.nn as nn
    import torch.nn.functional as F
    dev = "cuda:0"
    B = args.batch or 2048
    A = 18

    class Net(nn.Module):
        def __init__(self):
            super().__init__()
            self.c1, self.c2, self.c3 = nn.Conv2d(4, 32, 8, 4), nn.Conv2d(32, 64, 4, 2), nn.Conv2d(64, 64, 3, 1)
            self.fc, self.pi, self.v = nn.Linear(3136, 512), nn.Linear(512, A), nn.Linear(512, 1)

        def forward(self, x):
            x = F.relu(self.c3(F.relu(self.c2(F.relu(self.c1(x))))))
            h = F.relu(self.fc(x.flatten(1)))
            return self.pi(h), self.v(h)

    batch = wl.actor_critic_batch(3, B=B)
    x8 = torch.from_numpy(batch["obs"]).to(dev)
    act = torch.from_numpy(batch["action"].astype(np.int64)).to(dev)
    out = {"metric": "Nature-CNN with PyTorch's own layers on the same GPU (context, not the product path)", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
           "config": {"workload": "a2c_b%d, torch.nn, channels-last" % B, "global_batch": B}}
    for name, dt in (("bf16", torch.bfloat16), ("fp32", torch.float32)):
        net = Net().to(dev).to(dt).to(memory_format=torch.channels_last)
        adv = torch.from_numpy(batch["adv"]).to(dev).float()
        ret = torch.from_numpy(batch["ret"]).to(dev).float()

        def fwd():
            with torch.no_grad():
                return net((x8.to(dt) / 255).contiguous(memory_format=torch.channels_last))

        def step():
            z, v = net((x8.to(dt) / 255).contiguous(memory_format=torch.channels_last))
            lp = F.log_softmax(z.float(), 1)
            loss = (-(lp.gather(1, act[:, None])[:, 0] * adv).mean() + 0.5 * ((v[:, 0].float() - ret) ** 2).mean()
                    + 0.01 * (lp.exp() * lp).sum(1).mean())
            net.zero_grad(set_to_none=True)
            loss.backward()

        for fn in (fwd, step):
            for _ in range(args.warmup):
                fn()
        f_ms, s_ms = wall_ms(torch, fwd, args.steps), wall_ms(torch, step, args.steps)
        out[name] = {"forward_ms": round(f_ms, 4), "fwd_bwd_ms": round(s_ms, 4),
                     "fwd_bwd_samples_per_s": round(B / (s_ms * 1e-3), 1)}
    print(json.dumps(out))


UPDATE_BYTES = {"rmsprop": 20, "adam": 28, "adam_local": 52, "adam_merge": 60}   # fp32 arrays read + written per parameter


def update_rules_report(args, arn, wl, np, torch):
    """Secondary line: the update kernels on the A=18 policy/value parameter vector (what one learner
    iteration runs) and on a 64 Mi-entry vector (HBM-resident, shows the streaming rate), plus the whole
    learner iteration gradient + Adam update + re-pack at B=2048."""
    dev = "cuda:0"
    cfg = arn.Config(18, arn.ARN_HEAD_PV)
    stream = torch.cuda.current_stream()
    report = {}
    for label, n in (("params_a18", arn.param_count(cfg)), ("64Mi", 64 << 20)):
        inp = wl.update_rule_inputs(min(n, 1 << 20), 1, seed=1)
        rep = (n + inp["theta"].size - 1) // inp["theta"].size
        th = torch.from_numpy(np.tile(inp["theta"], rep)[:n].copy()).to(dev)
        g = torch.from_numpy(np.tile(inp["grads"][0], rep)[:n].copy()).to(dev)
        st = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(8)]
        packed = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev) if label == "params_a18" else None
        calls = {
            "rmsprop": lambda: arn.rmsprop_update(th, g, st[0], lr=7e-4, rho=0.99, eps=1e-6, stream=stream),
            "adam": lambda: arn.adam_update(th, g, st[0], st[1], t=3, r=4.2e-4, beta1=0.9, beta2=0.999, eps=4e-5,
                                            stream=stream),
            "adam_local": lambda: arn.async_adam_local_step(th, g, st[0], st[1], st[2], st[3], st[4], t=3, r=4.2e-4,
                                                            beta1=0.9, beta2=0.999, eps=4e-5, stream=stream),
            "adam_merge": lambda: arn.async_adam_merge(st[5], st[6], st[7], th, st[0], st[1], st[2], st[3], st[4],
                                                       n_local=2, beta1=0.9, beta2=0.999, stream=stream),
        }
        if packed is not None:
            calls["adam+pack_all"] = lambda: arn.adam_update(th, g, st[0], st[1], t=3, r=4.2e-4, beta1=0.9,
                                                             beta2=0.999, eps=4e-5, cfg=cfg, w_packed=packed,
                                                             stream=stream)
        arn.profile_enable(True)
        for name, fn in calls.items():
            for _ in range(args.warmup + args.steps):
                fn()
        torch.cuda.synchronize()
        recs = arn.profile_collect(cap=16 * (args.warmup + args.steps) + 64)
        arn.profile_enable(False)
        per = {}
        for name, ms in recs:
            per.setdefault(name, []).append(ms)
        rows = {}
        for name, v in per.items():
            us = 1e3 * float(np.mean(v[len(v) // 4:]))
            rows[name] = {"us": round(us, 2)}
            if name in UPDATE_BYTES:
                gbs = UPDATE_BYTES[name] * n / (us * 1e-6) / 1e9
                rows[name].update({"GB/s": round(gbs, 1), "hbm_frac": round(gbs / PEAK_HBM_GBS, 4)})
        report[label] = {"n": n, "kernels": rows}
    # whole learner iteration
    k, B = 3, args.batch or 2048
    flat = wl.he_normal_params(18, "pv", 2000 + k)
    th = torch.from_numpy(flat).to(dev)
    packed = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev)
    arn.weights_prepare(cfg, th, packed)
    batch = {nm: torch.from_numpy(np.ascontiguousarray(v)).to(dev) for nm, v in wl.actor_critic_batch(k, B=B).items()}
    ws = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_TRAIN), dtype=torch.uint8, device=dev)
    dW = torch.empty(arn.param_count(cfg), dtype=torch.float32, device=dev)
    m, v = (torch.zeros_like(dW) for _ in range(2))
    loss = torch.empty(4, dtype=torch.float32, device=dev)

    def iteration(t):
        arn.train_step_grads(cfg, packed, batch, "a2c", dW, loss, workspace=ws, stream=stream)
        arn.adam_update(th, dW, m, v, t=t, r=1e-5, beta1=0.9, beta2=0.999, eps=0.01 / B, cfg=cfg, w_packed=packed,
                        stream=stream)

    for t in range(1, args.warmup + 1):
        iteration(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup + 1, args.warmup + args.steps + 1):
        iteration(t)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    print(json.dumps({
        "metric": "Nature-CNN samples/sec (gradient + Adam update + re-pack) at B=%d on 1 GPU" % B,
        "value": round(B / sec, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "learner iteration a2c_b%d + update rules" % B, "global_batch": B,
                   "parallelism": "single-gpu"},
        "update_kernels": report, "loss_finite": bool(torch.isfinite(loss).all().item())}))


def dqn_report(args, arn, wl, np, torch):
    """Secondary lines: Double-DQN with the dueling head at B = 2048 (three forward passes + backward) and
    the sampler's inference that returns drawn actions at B = 256."""
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    to_dev = lambda d: {n: torch.from_numpy(np.ascontiguousarray(v)).to(dev) for n, v in d.items()}

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    A, B = 18, args.batch or 2048
    cfg = arn.Config(A, arn.ARN_HEAD_DUEL, double_q=1)
    packed, tpacked = (torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev) for _ in range(2))
    arn.weights_prepare(cfg, torch.from_numpy(wl.he_normal_params(A, "duel", 2005)).to(dev), packed)
    arn.weights_prepare(cfg, torch.from_numpy(wl.he_normal_params(A, "duel", 3005)).to(dev), tpacked)
    batch = to_dev(wl.c51_batch(5, B=B))
    batch["w_target_packed"] = tpacked
    ws = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_TRAIN), dtype=torch.uint8, device=dev)
    dW = torch.empty(arn.param_count(cfg), dtype=torch.float32, device=dev)
    loss = torch.empty(4, dtype=torch.float32, device=dev)
    sec = timed(lambda: arn.train_step_grads(cfg, packed, batch, "dqn", dW, loss, workspace=ws, stream=stream))
    fwd = 2 * (MACS["conv1"] + MACS["conv2"] + MACS["conv3"] + MACS["fc"] + (A + 1) * 512)
    flops = 3 * fwd - 2 * MACS["conv1"] + 2 * fwd
    print(json.dumps({
        "metric": "Nature-CNN samples/sec (train_step_grads:dqn, double + dueling) at B=%d on 1 GPU" % B,
        "value": round(B / sec, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "double_dqn_dueling_b%d" % B, "global_batch": B, "parallelism": "single-gpu"},
        "mfma_frac_whole_step": round(B / sec * flops / 1e12 / PEAK_BF16_TFLOPS, 4),
        "algorithmic_flops_per_sample": flops, "loss_finite": bool(torch.isfinite(loss).all().item())}))

    Bi = 256
    cfgp = arn.Config(A, arn.ARN_HEAD_PV)
    pp = torch.empty(arn.packed_bytes(cfgp), dtype=torch.uint8, device=dev)
    arn.weights_prepare(cfgp, torch.from_numpy(wl.he_normal_params(A, "pv", 2002)).to(dev), pp)
    obs = torch.from_numpy(wl.frames_for(2, Bi)).to(dev)
    un = to_dev(wl.action_uniforms(Bi, 3))
    wsf = torch.empty(arn.workspace_bytes(cfgp, Bi, arn.ARN_MODE_FORWARD), dtype=torch.uint8, device=dev)
    act = torch.empty(Bi, dtype=torch.int32, device=dev)
    logp = torch.empty(Bi, dtype=torch.float32, device=dev)
    sec = timed(lambda: arn.policy_act(cfgp, pp, obs, un["u"], un["u2"], act, logp, workspace=wsf, stream=stream))
    print(json.dumps({
        "metric": "Nature-CNN samples/sec (policy_act, categorical draw) at B=%d on 1 GPU" % Bi,
        "value": round(Bi / sec, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "act_b%d (256 simulators, one environment step)" % Bi, "global_batch": Bi,
                   "parallelism": "single-gpu"}}))


def alternating_report(args, arn, wl, np, torch):
    """Section "Synchronized Sampling": the simulators are split into two groups that alternate, so that one
    group's inference runs while the other group's simulators step.  Here the simulators are no-ops; what is
    measured is the GPU side including the host hand-over: observations start in pinned host memory, actions
    end there.  Per group and environment step: H2D copy of uint8 frames -> arn_policy_act -> D2H copy of the
    int32 actions, each group on a stream of its own (default priority).  Reported against one group of all
    simulators handled back to back."""
    dev, A, n_sims = "cuda:0", 18, args.batch or 256
    cfg = arn.Config(A, arn.ARN_HEAD_PV)
    packed = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev)
    arn.weights_prepare(cfg, torch.from_numpy(wl.he_normal_params(A, "pv", 2002)).to(dev), packed)
    frames = wl.frames_for(2, n_sims)
    un = wl.action_uniforms(n_sims, 4)

    class Group:
        def __init__(self, lo, hi):
            n = hi - lo
            self.n = n
            self.stream = torch.cuda.Stream()
            self.h_obs = torch.from_numpy(frames[lo:hi].copy()).pin_memory()
            self.h_act = torch.empty(n, dtype=torch.int32).pin_memory()
            self.d_obs = torch.empty((n, 4, 84, 84), dtype=torch.uint8, device=dev)
            self.d_act = torch.empty(n, dtype=torch.int32, device=dev)
            self.u = torch.from_numpy(un["u"][lo:hi].copy()).to(dev)
            self.u2 = torch.from_numpy(un["u2"][lo:hi].copy()).to(dev)
            self.ws = torch.empty(arn.workspace_bytes(cfg, n, arn.ARN_MODE_FORWARD), dtype=torch.uint8, device=dev)
            self.done = torch.cuda.Event()

        def issue(self):
            with torch.cuda.stream(self.stream):
                self.d_obs.copy_(self.h_obs, non_blocking=True)
                arn.policy_act(cfg, packed, self.d_obs, self.u, self.u2, self.d_act, workspace=self.ws,
                               stream=self.stream)
                self.h_act.copy_(self.d_act, non_blocking=True)
                self.done.record(self.stream)

        def wait(self):
            self.done.synchronize()

    def run(groups, steps):
        # steady state of the alternation: a group's next request is issued as soon as its actions are back
        # (its simulators are no-ops), while the other group's request is in flight
        for g in groups:
            g.issue()
        t0 = time.perf_counter()
        for _ in range(steps):
            for g in groups:
                g.wait()
                g.issue()
        for g in groups:
            g.wait()
        return (time.perf_counter() - t0) / steps

    half = n_sims // 2
    two = [Group(0, half), Group(half, n_sims)]
    one = [Group(0, n_sims)]
    run(two, args.warmup), run(one, args.warmup)
    t_two, t_one = run(two, args.steps), run(one, args.steps)
    torch.cuda.synchronize()
    ok = bool(((two[0].h_act >= 0) & (two[0].h_act < A)).all() and ((one[0].h_act >= 0) & (one[0].h_act < A)).all())
    print(json.dumps({
        "metric": "sampler inference, simulator-steps/sec with host hand-over (two alternating groups of %d)" % half,
        "value": round(n_sims / t_two, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(t_two * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "alternating_act_%d+%d, pinned host frames in, actions out" % (half, n_sims - half),
                   "global_batch": n_sims, "parallelism": "single-gpu, two streams"},
        "one_group_ms_per_step": round(t_one * 1e3, 4), "one_group_samples_per_s": round(n_sims / t_one, 1),
        "actions_valid": ok}))


def paper_geometry_report(args, arn, wl, np, torch, net="nature"):
    """A2C gradient step and action-selection inference on the frame size and padding of the paper's own runs
    (appendix "Atari Frame Processing"): 104x80 frames, 25x19 -> 12x9 -> 12x9 feature maps, fc 6912 -> 512."""
    dev, A, B, k = "cuda:0", 18, args.batch or 2048, 3
    frame, fc_in = wl.PAPER_FRAME, wl.FC_INPUTS[wl.PAPER_FRAME]
    if net == "a3c":   # 2-convolution network: its own algorithmic flops, whatever the embedding executes
        macs = {"conv1": 25 * 19 * 256 * 16, "conv2": 12 * 9 * 256 * 32, "fc": wl.A3C_FC_INPUTS * 256, "head": (A + 1) * 256}
    else:
        macs = {"conv1": 25 * 19 * 256 * 32, "conv2": 12 * 9 * 512 * 64, "conv3": 12 * 9 * 576 * 64, "fc": fc_in * 512,
                "head": (A + 1) * 512}
    fwd_flops = 2 * sum(macs.values())
    fwdbwd_flops = 3 * fwd_flops - 2 * macs["conv1"]
    cfg = arn.Config(A, arn.ARN_HEAD_PV, geometry=arn.ARN_GEOM_A3C if net == "a3c" else arn.ARN_GEOM_PAPER)
    flat = wl.he_normal_params(A, "pv", 2000 + k, fc_inputs=fc_in, net=net)
    packed = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev)
    arn.weights_prepare(cfg, torch.from_numpy(flat).to(dev), packed)
    batch = {n: torch.from_numpy(np.ascontiguousarray(v)).to(dev)
             for n, v in wl.actor_critic_batch(k, B=B, frame=frame).items()}
    ws = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_TRAIN), dtype=torch.uint8, device=dev)
    dW = torch.empty(arn.param_count(cfg), dtype=torch.float32, device=dev)
    loss = torch.empty(4, dtype=torch.float32, device=dev)
    logits = torch.empty(B, A, dtype=torch.float32, device=dev)
    val = torch.empty(B, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    step = lambda: arn.train_step_grads(cfg, packed, batch, "a2c", dW, loss, workspace=ws, stream=stream)
    fwd = lambda: arn.policy_forward(cfg, packed, batch["obs"], logits, val, workspace=ws, stream=stream)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    sec, sec_fwd = timed(step), timed(fwd)
    arn.profile_enable(True)
    for _ in range(args.steps):
        step()
        arn.profile_null(stream)
    torch.cuda.synchronize()
    per = {}
    for name, ms in arn.profile_collect(cap=64 * args.steps + 64):
        tot, cnt = per.get(name, (0.0, 0))
        per[name] = (tot + ms, cnt + 1)
    arn.profile_enable(False)
    null_ms = per.pop("null")[0] / args.steps
    avg_ms = {n: max(t / c - null_ms, 0.0) for n, (t, c) in per.items()}
    print(json.dumps({
        "metric": "%s samples/sec (fwd+bwd, 104x80 frames) at B=%d on 1 GPU" % (
            "2-convolution network" if net == "a3c" else "Nature-CNN, padded conv2/conv3,", B),
        "value": round(B / sec, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": ("a2c_grad_step_B%d_A18 on 104x80 frames, " % B) + ("2 convolutions 16/32 filters (25x19 -> 12x9, fc 3456 -> 256)" if net == "a3c" else "25x19 -> 12x9 -> 12x9, fc 6912"),
                   "global_batch": B, "parallelism": "single-gpu"},
        "mfma_frac_whole_step": round(B / sec * fwdbwd_flops / 1e12 / PEAK_BF16_TFLOPS, 4),
        "forward_samples_per_s": round(B / sec_fwd, 1), "forward_ms": round(sec_fwd * 1e3, 4),
        "algorithmic_flops_per_sample": {"forward": fwd_flops, "forward_backward": fwdbwd_flops},
        "kernel_us": {n: round(v * 1e3, 2) for n, v in sorted(avg_ms.items(), key=lambda kv: -kv[1])}}))


if __name__ == "__main__":
    main()
