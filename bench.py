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


def measured_traffic(kernel, B):
    """HBM bytes per launch of `kernel` from the committed counter summary (FETCH_SIZE + WRITE_SIZE, each
    scaled by what the same counter reads for a plain copy of known size); None if it covers another batch."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "a2c_b2048_traffic.json")
    try:
        with open(path) as f:
            prof = json.load(f)
    except (OSError, ValueError):
        return None
    if prof.get("batch") != B:
        return None
    return prof.get("hbm_bytes_per_launch", {}).get(kernel)


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
                         "padded conv2/conv3 (gathered-contraction kernels), per-kernel times included")
    ap.add_argument("--update-rules", action="store_true",
                    help="report the parameter-update kernels instead (secondary line)")
    ap.add_argument("--workload", type=int, default=3, choices=[1, 2, 3, 4, 5],
                    help="3 (default) = the headline A2C step at B=2048; 1, 2 = inference; 4 = PPO; 5 = C51")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run a plain device-to-device copy of MIB mebibytes a few times (reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--cpu-samples", type=int, default=0, help="oracle sample size (0 = auto, ~10-30 s)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path shards by sample; "
              "one gradient all-reduce per step would follow)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

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
    if args.update_rules:
        update_rules_report(args, arn, wl, np, torch)
        return
    if args.dqn:
        dqn_report(args, arn, wl, np, torch)
        return
    if args.alternating:
        alternating_report(args, arn, wl, np, torch)
        return
    if args.paper_geometry:
        paper_geometry_report(args, arn, wl, np, torch)
        return
    if args.workload != 3:
        other_workload(args, arn, wl, np, torch)
        return
    A, B, k = 18, args.batch or 2048, 3
    cfg = arn.Config(A, arn.ARN_HEAD_PV)
    flat = wl.he_normal_params(A, "pv", 2000 + k)
    w = torch.from_numpy(flat).to(dev)
    packed = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev)
    arn.weights_prepare(cfg, w, packed)
    batch_np = wl.actor_critic_batch(k, B=B)
    batch = {n: torch.from_numpy(np.ascontiguousarray(v)).to(dev) for n, v in batch_np.items()}
    ws = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_TRAIN), dtype=torch.uint8, device=dev)
    dW = torch.empty(arn.param_count(cfg), dtype=torch.float32, device=dev)
    loss = torch.empty(4, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        arn.train_step_grads(cfg, packed, batch, "a2c", dW, loss, workspace=ws, stream=torch.cuda.current_stream())

    def timed(fn, steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    for _ in range(args.warmup):
        step()
    sec = timed(step, args.steps)
    value = B / sec

    # forward-only (action-selection inference) rate on the same batch, for the report
    wsf = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_FORWARD), dtype=torch.uint8, device=dev)
    logits = torch.empty(B, A, dtype=torch.float32, device=dev)
    val = torch.empty(B, dtype=torch.float32, device=dev)

    def fwd():
        arn.policy_forward(cfg, packed, batch["obs"], logits, val, workspace=wsf, stream=torch.cuda.current_stream())

    for _ in range(args.warmup):
        fwd()
    sec_fwd = timed(fwd, args.steps)

    # the same calls captured once into HIP graphs and replayed (what a tight training / serving loop would do)
    def graph_time(fn):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        for _ in range(args.warmup):
            g.replay()
        return timed(g.replay, args.steps)

    sec_graph, sec_fwd_graph = graph_time(step), graph_time(fwd)

    # per-kernel durations: the same K steps again with a HIP event pair around every launch
    arn.profile_enable(True)
    for _ in range(args.steps):
        step()
        arn.profile_null(torch.cuda.current_stream())
    torch.cuda.synchronize()
    recs = arn.profile_collect(cap=64 * args.steps + 64)
    arn.profile_enable(False)
    per = {}
    for name, ms in recs:
        tot, cnt = per.get(name, (0.0, 0))
        per[name] = (tot + ms, cnt + 1)
    # an event pair around nothing measures what the pair itself adds; it is subtracted from every kernel
    null_ms = per.pop("null")[0] / args.steps
    avg_ms = {n: max(t / c - null_ms, 0.0) for n, (t, c) in per.items()}
    dominant = max((n for n in avg_ms if n in KERNEL_FLOPS), key=avg_ms.get)
    dom_s = avg_ms[dominant] * 1e-3
    dom_flops = KERNEL_FLOPS[dominant] * B
    dom_bytes = KERNEL_BYTES[dominant] * B + KERNEL_BYTES_PER_LAUNCH[dominant]
    # the binding resource is the one whose time at peak is larger
    if dom_bytes / (PEAK_HBM_GBS * 1e9) >= dom_flops / (PEAK_BF16_TFLOPS * 1e12):
        achieved = dom_bytes / dom_s / 1e9
        roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None}
    else:
        achieved = dom_flops / dom_s / 1e12
        roofline = {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": None}
    roofline["traffic"] = measured_traffic(dominant, B)
    roofline["avg_launch_us"] = round(avg_ms[dominant] * 1e3, 2)
    roofline["event_pair_overhead_us"] = round(null_ms * 1e3, 2)
    roofline["algorithmic_bytes_per_launch"] = dom_bytes
    roofline["algorithmic_flops_per_launch"] = dom_flops

    out = {
        "metric": "Nature-CNN samples/sec (fwd+bwd) at B=%d on 1 GPU" % B,
        "value": round(value, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "a2c_grad_step_B%d_A18 (256 envs x 8 steps, rectangle frames)" % B,
                   "global_batch": B, "parallelism": "single-gpu"},
        "mfma_frac_whole_step": round(value * FWDBWD_FLOPS / 1e12 / PEAK_BF16_TFLOPS, 4),
        "hbm_frac_whole_step": round(value * FWDBWD_BYTES / 1e9 / PEAK_HBM_GBS, 4),
        "forward_samples_per_s": round(B / sec_fwd, 1),
        "forward_ms": round(sec_fwd * 1e3, 4),
        "graph_replay_ms_per_step": round(sec_graph * 1e3, 4),
        "graph_replay_forward_ms": round(sec_fwd_graph * 1e3, 4),
        "kernel_us": {n: round(v * 1e3, 2) for n, v in sorted(avg_ms.items(), key=lambda kv: -kv[1])},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        from oracle import nature_cnn as orc
        spec = orc.NetSpec(A, "pv")
        n = args.cpu_samples or min(B, 2048)
        sub = {kk: v[:n] for kk, v in batch_np.items()}
        reps, t_total = 0, 0.0
        while reps < 1 or (t_total < 12.0 and reps < 20):     # about 10-30 s of CPU work
            t0 = time.perf_counter()
            orc.train_step_grads(flat, sub, "a2c", spec)
            t_total += time.perf_counter() - t0
            reps += 1
        out["cpu_baseline"] = {"value": round(n * reps / t_total, 1), "unit": "samples/s", "cores": orc.num_threads(),
                               "kind": "oracle",
                               "sample": "first %d samples of the same batch, fwd+loss+bwd, %d repetitions, %.1f s"
                                         % (n, reps, t_total)}
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


def paper_geometry_report(args, arn, wl, np, torch):
    """A2C gradient step and action-selection inference on the frame size and padding of the paper's own runs
    (appendix "Atari Frame Processing"): 104x80 frames, 25x19 -> 12x9 -> 12x9 feature maps, fc 6912 -> 512."""
    dev, A, B, k = "cuda:0", 18, args.batch or 2048, 3
    frame, fc_in = wl.PAPER_FRAME, wl.FC_INPUTS[wl.PAPER_FRAME]
    macs = {"conv1": 25 * 19 * 256 * 32, "conv2": 12 * 9 * 512 * 64, "conv3": 12 * 9 * 576 * 64, "fc": fc_in * 512,
            "head": (A + 1) * 512}
    fwd_flops = 2 * sum(macs.values())
    fwdbwd_flops = 3 * fwd_flops - 2 * macs["conv1"]
    cfg = arn.Config(A, arn.ARN_HEAD_PV, geometry=arn.ARN_GEOM_PAPER)
    flat = wl.he_normal_params(A, "pv", 2000 + k, fc_inputs=fc_in)
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
        "metric": "Nature-CNN samples/sec (fwd+bwd, 104x80 frames, padded conv2/conv3) at B=%d on 1 GPU" % B,
        "value": round(B / sec, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "a2c_grad_step_B%d_A18 on 104x80 frames (25x19 -> 12x9 -> 12x9, fc 6912)" % B,
                   "global_batch": B, "parallelism": "single-gpu"},
        "mfma_frac_whole_step": round(B / sec * fwdbwd_flops / 1e12 / PEAK_BF16_TFLOPS, 4),
        "forward_samples_per_s": round(B / sec_fwd, 1), "forward_ms": round(sec_fwd * 1e3, 4),
        "algorithmic_flops_per_sample": {"forward": fwd_flops, "forward_backward": fwdbwd_flops},
        "kernel_us": {n: round(v * 1e3, 2) for n, v in sorted(avg_ms.items(), key=lambda kv: -kv[1])}}))


def kernel_times_us(arn, torch, step, steps, stream):
    """Average duration per launch site (microseconds, event-pair overhead subtracted) over `steps` more steps;
    sites that launch several times per step (the forward kernels of a step with a target network) are summed."""
    arn.profile_enable(True)
    for _ in range(steps):
        step()
        arn.profile_null(stream)
    torch.cuda.synchronize()
    per = {}
    for name, ms in arn.profile_collect(cap=96 * steps + 64):
        tot, cnt = per.get(name, (0.0, 0))
        per[name] = (tot + ms, cnt + 1)
    arn.profile_enable(False)
    null_ms = per.pop("null")[0] / steps
    us = {n: max(t - c * null_ms, 0.0) / steps * 1e3 for n, (t, c) in per.items()}
    return {n: round(v, 2) for n, v in sorted(us.items(), key=lambda kv: -kv[1])}


def other_workload(args, arn, wl, np, torch):
    """Secondary report lines for the other workloads (same JSON shape, no per-kernel roofline)."""
    dev, k = "cuda:0", args.workload
    w = wl.WORKLOADS[k]
    A, B, head = w["A"], args.batch or w["B"], w["head"]
    cfg = arn.Config(A, arn.ARN_HEAD_PV if head == "pv" else arn.ARN_HEAD_C51)
    flat = wl.he_normal_params(A, head, 2000 + k)
    packed = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev)
    arn.weights_prepare(cfg, torch.from_numpy(flat).to(dev), packed)
    stream = torch.cuda.current_stream()
    to_dev = lambda d: {n: torch.from_numpy(np.ascontiguousarray(v)).to(dev) for n, v in d.items()}
    if w["kind"] == "forward":
        obs = torch.from_numpy(wl.frames_for(k, B)).to(dev)
        ws = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_FORWARD), dtype=torch.uint8, device=dev)
        logits = torch.empty(B, A, dtype=torch.float32, device=dev)
        value = torch.empty(B, dtype=torch.float32, device=dev)
        probs = torch.empty(B, A, dtype=torch.float32, device=dev)
        greedy = torch.empty(B, dtype=torch.int32, device=dev)
        step = lambda: arn.policy_forward(cfg, packed, obs, logits, value, probs, greedy, workspace=ws, stream=stream)
        flops = 2 * (MACS["conv1"] + MACS["conv2"] + MACS["conv3"] + MACS["fc"] + (A + 1) * 512)
        name = "policy_forward"
    else:
        ws = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_TRAIN), dtype=torch.uint8, device=dev)
        dW = torch.empty(arn.param_count(cfg), dtype=torch.float32, device=dev)
        loss = torch.empty(4, dtype=torch.float32, device=dev)
        if w["kind"] == "ppo":
            batch = to_dev(wl.actor_critic_batch(k, B=B, normalise_adv=True))
            # sampling-policy log-probs: the current logits (from this library) perturbed by N(0, 0.05^2)
            wsf = torch.empty(arn.workspace_bytes(cfg, B, arn.ARN_MODE_FORWARD), dtype=torch.uint8, device=dev)
            logits = torch.empty(B, A, dtype=torch.float32, device=dev)
            value = torch.empty(B, dtype=torch.float32, device=dev)
            arn.policy_forward(cfg, packed, batch["obs"], logits, value, workspace=wsf, stream=stream)
            noisy = logits + torch.from_numpy(wl.logit_noise(k, B, A).astype(np.float32)).to(dev)
            batch["old_logp"] = torch.log_softmax(noisy, dim=1).gather(1, batch["action"].long()[:, None])[:, 0].contiguous()
            head_macs = (A + 1) * 512
            tgt_flops = 0
        else:
            batch = to_dev(wl.c51_batch(k, B=B))
            tpacked = torch.empty(arn.packed_bytes(cfg), dtype=torch.uint8, device=dev)
            arn.weights_prepare(cfg, torch.from_numpy(wl.he_normal_params(A, head, 3000 + k)).to(dev), tpacked)
            batch["w_target_packed"] = tpacked
            head_macs = A * 51 * 512
            tgt_flops = 2 * (MACS["conv1"] + MACS["conv2"] + MACS["conv3"] + MACS["fc"] + head_macs)
        fwd = 2 * (MACS["conv1"] + MACS["conv2"] + MACS["conv3"] + MACS["fc"] + head_macs)
        flops = 3 * fwd - 2 * MACS["conv1"] + tgt_flops
        step = lambda: arn.train_step_grads(cfg, packed, batch, w["kind"], dW, loss, workspace=ws, stream=stream)
        name = "train_step_grads:" + w["kind"]
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    print(json.dumps({
        "metric": "Nature-CNN samples/sec (%s) at B=%d on 1 GPU" % (name, B), "value": round(B / sec, 1),
        "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s (workload %d)" % (w["name"], k), "global_batch": B, "parallelism": "single-gpu"},
        "mfma_frac_whole_step": round(B / sec * flops / 1e12 / PEAK_BF16_TFLOPS, 4),
        "algorithmic_flops_per_sample": flops,
        "kernel_us_per_step": kernel_times_us(arn, torch, step, min(args.steps, 50), stream)}))


if __name__ == "__main__":
    main()
