#!/usr/bin/env python3
"""Benchmark of the GA3C hot path on one MI355X.

A step is one balanced pass of the whole path (Sec. 4.2 of the paper: in a
balanced configuration PPS ~ TPS * t_max): t_max = 5 prediction calls of N
frames each, one per action of every agent, followed by one training step on
the N agents x 5 frames those actions produced (the bootstrap value of a
segment is the value of the next segment's first prediction, so no sixth
prediction is needed).  N = 512 agents, the small
network of Sec. 3.2 with 18 actions, synthetic game-like frames that are
resident in HBM before the timed region starts.  By default the step is
submitted the way the paper's predictor and trainer threads do it (Sec. 4.1):
the five predictions on one stream, the training step (on the segment the
previous step predicted) on another, so that the two calls share the GPU;
`--streams 1` issues the six calls one after another (the default run
measures that too and reports both rates).

Prints ONE JSON line.  `value` = frames per second through predict AND
train_step (each frame is predicted once and trained on once).  The line
also carries predict-only and train-only rates, per-stage times measured with
HIP events inside the library, the roofline of the dominant kernel and the
fp64 CPU oracle timed on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA = 157.3e12   # MI355X dense fp32 matrix, FLOP/s
PEAK_HBM = 8.0e12           # B/s

# HBM traffic per launch from hardware counters: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (two runs of
# `python3 bench.py --steps 3 --warmup 1 --streams 1 --no-cpu-baseline --mixed-seconds 0 --rmsprop-big`), KiB per dispatch,
# small net, by frames in the launch.  Every read request on this chip is a 128-byte line while FETCH_SIZE prices
# it at 64 bytes: on the streaming RMSProp kernel over 2^28 parameters (12 B read, 8 B written per parameter) the
# counters read 0.5000 and 1.0000 of the known bytes, hence the scale factors.  The summary is kept under profiles/.
FETCH_SCALE, WRITE_SCALE = 2.0, 1.0
COUNTER_KIB = {   # stage: {frames per launch: (FETCH_SIZE, WRITE_SIZE)}
    "conv12_fwd": {512: (7554.7, 5184.0), 1024: (14626.7, 10368.0), 2560: (36536.2, 94053.3)},   # 2560: training, keeps y1
    "fc_fwd": {512: (4153.0, 7168.0), 1024: (6649.0, 8192.0), 2560: (14425.0, 20480.0)},
    "heads_fwd": {512: (3789.0, 592.0), 1024: (4282.0, 1104.0)},
    "heads_train": {2560: (10524.6, 9396.2)},
    "conv1_wgrad": {2560: (67617.1, 4112.0)},
    "conv2_wgrad": {2560: (45123.3, 16558.4)},
    "conv2_dgrad": {2560: (45193.5, 64000.0)},
    "fc_wgrad": {2560: (19955.3, 20736.0)},
    "fc_dgrad": {2560: (25372.6, 27011.7)},
    "wgrad_reduce": {2560: (24878.8, 2809.9)},
    "rmsprop": {2560: (4019.6, 5394.1)},
}


def counter_traffic(stage, launches):
    """Mean HBM bytes per launch of a stage over `launches` = [(frames, count), ...]; None where not measured."""
    tab = COUNTER_KIB.get(stage)
    if not tab or any(b not in tab for b, _ in launches):
        return None
    tot = sum(n * (FETCH_SCALE * tab[b][0] + WRITE_SCALE * tab[b][1]) * 1024.0 for b, n in launches)
    return round(tot / sum(n for _, n in launches))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--agents", type=int, default=512)
    ap.add_argument("--net", choices=("small", "large"), default="small")
    ap.add_argument("--math", type=int, choices=(0, 1), default=0,
                    help="0: fp32 accuracy (default); 1: operands of every contraction rounded to bfloat16")
    ap.add_argument("--streams", type=int, choices=(1, 2), default=2,
                    help="2: predictions on one stream, training on another (predictor and trainer threads of "
                         "Sec. 4.1 share the GPU); 1: the six calls of a step one after another")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rmsprop-big", action="store_true", help="also time RMSProp on 2^28 parameters")
    ap.add_argument("--mixed-seconds", type=float, default=1.0,
                    help="length of each mixed-load run through the scheduler (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import ga3c_synth as synth
    import paper_1611_06256_amd as g

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    N, T, A = args.agents, 5, 18
    import dataclasses
    desc = dataclasses.replace(g.SMALL_NET(A) if args.net == "small" else g.LARGE_NET(A), math=args.math)
    net = g.Ga3c(desc, max(N, 1024), N * T)
    net.params_init(synth.BASE_SEED)
    hp = g.HParams(clip_norm=40.0)

    seed = synth.BASE_SEED + 2
    frames_np = synth.rectangle_frames_tiled(seed, N * T).reshape(N, T, 4, 84, 84)
    tr = synth.trajectories(seed + 1, N, T, A)
    frames = torch.from_numpy(frames_np).cuda()
    # predict call t sees the frames of step t of every agent
    pframes = [frames[:, t].contiguous() for t in range(T)]
    actions = torch.from_numpy(tr["actions"]).cuda()
    rewards = torch.from_numpy(tr["rewards"]).cuda()
    dones = torch.from_numpy(tr["dones"]).cuda()
    uniforms = torch.from_numpy(synth.uniforms(seed + 3, N)).cuda()
    logits = torch.empty(N, A, device="cuda"); values = torch.empty(N, device="cuda")
    probs = torch.empty(N, A, device="cuda"); sampled = torch.empty(N, dtype=torch.int32, device="cuda")
    boot = torch.empty(N, device="cuda")
    stats = torch.zeros(8, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        # one prediction per frame: the value that closes a segment's returns, V(s_{t+t_max}), is what the agent is
        # told by the first prediction of its next segment (Sec. 4.1), so a segment costs t_max predictions, not
        # t_max + 1; with synthetic states the values of prediction 0 stand in for it
        for t in range(T):
            net.predict(pframes[t], uniforms=uniforms, logits=logits, values=boot if t == 0 else values, probs=probs,
                        actions=sampled, stream=stream)
        net.train_step(frames, actions, rewards, dones, boot, hp, stats=stats, stream=stream)

    def timed(fn, k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / k

    # The same work on two streams, as the predictor and trainer threads of Sec. 4.1 submit it: the predictions
    # of segment i run while the training step works on segment i - 1.  Three sets of bootstrap values, so the
    # predictions may run one segment ahead of training; events order writer and reader of each set.
    s_pred, s_train = torch.cuda.Stream(), torch.cuda.Stream()
    boots = [torch.zeros(N, device="cuda") for _ in range(3)]
    ev_pred = [torch.cuda.Event() for _ in range(3)]
    ev_train = [torch.cuda.Event() for _ in range(3)]
    for e in ev_pred + ev_train:
        e.record(stream)
    seg = [0]

    def step_two_streams():
        i = seg[0]; seg[0] += 1
        s_pred.wait_event(ev_train[i % 3])               # the training step that last read this set is done
        for t in range(T):
            net.predict(pframes[t], uniforms=uniforms, logits=logits, values=boots[i % 3] if t == 0 else values,
                        probs=probs, actions=sampled, stream=s_pred)
        ev_pred[i % 3].record(s_pred)
        s_train.wait_event(ev_pred[(i - 1) % 3])         # values written by the predictions of segment i - 1
        net.train_step(frames, actions, rewards, dones, boots[(i - 1) % 3], hp, stats=stats, stream=s_train)
        ev_train[(i - 1) % 3].record(s_train)

    for _ in range(args.warmup):
        step()
    sec_one = timed(step, args.steps)
    sec_two = None
    if args.streams == 2:
        for _ in range(args.warmup):
            step_two_streams()
        sec_two = timed(step_two_streams, args.steps)
    sec = sec_two if args.streams == 2 else sec_one
    frames_per_step = N * T

    # predict-only and train-only rates (same buffers)
    big = torch.from_numpy(synth.rectangle_frames_tiled(seed + 4, 1024)).cuda()
    bl = torch.empty(1024, A, device="cuda"); bv = torch.empty(1024, device="cuda")
    pred_fn = lambda: net.predict(big, logits=bl, values=bv, stream=stream)
    train_fn = lambda: net.train_step(frames, actions, rewards, dones, boot, hp, stats=stats, stream=stream)
    for _ in range(3):
        pred_fn(); train_fn()
    pred_sec = timed(pred_fn, max(args.steps, 20))
    train_sec = timed(train_fn, max(args.steps, 20))

    # per-stage times with HIP events recorded by the library on the same stream
    net.profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = net.profile_read()
    net.profile_enable(False)
    # conv1 runs as exact bf16x3 MFMA and is bound by fetching frames and storing activations
    hbm_stages = {"conv12_fwd", "conv1_fwd", "conv1_wgrad", "conv2_dgrad", "rmsprop", "sqnorm"}
    stages = []
    for name, p in prof.items():
        per_call_ms = p["ms"] / p["calls"]
        e = {"stage": name, "calls_per_step": p["calls"] / args.steps, "ms_per_call": round(per_call_ms, 5),
             "ms_per_step": round(p["ms"] / args.steps, 5)}
        if p["flop"] > 0:
            e["tflops"] = round(p["flop"] / (p["ms"] * 1e-3) / 1e12, 3)
        if p["bytes"] > 0:
            e["gbps"] = round(p["bytes"] / (p["ms"] * 1e-3) / 1e9, 2)
        if name in hbm_stages and p["bytes"] > 0:
            e["bound"] = "hbm"; e["frac"] = round(p["bytes"] / (p["ms"] * 1e-3) / PEAK_HBM, 4)
        elif p["flop"] > 0:
            e["bound"] = "mfma"; e["frac"] = round(p["flop"] / (p["ms"] * 1e-3) / PEAK_FP32_MFMA, 4)
        stages.append(e)
    stages.sort(key=lambda e: -e["ms_per_step"])
    dom = next(e for e in stages if "bound" in e)
    dp = prof[dom["stage"]]
    if dom["bound"] == "mfma":
        ach = dp["flop"] / (dp["ms"] * 1e-3) / 1e12
        roofline = {"kernel": dom["stage"], "bound": "mfma", "achieved": round(ach, 3), "peak": PEAK_FP32_MFMA / 1e12,
                    "unit": "TFLOP/s", "frac": round(ach * 1e12 / PEAK_FP32_MFMA, 4), "traffic": None,
                    "ms_per_launch": round(dp["ms"] / dp["calls"], 5)}
    else:
        ach = dp["bytes"] / (dp["ms"] * 1e-3) / 1e9
        roofline = {"kernel": dom["stage"], "bound": "hbm", "achieved": round(ach, 2), "peak": PEAK_HBM / 1e9,
                    "unit": "GB/s", "frac": round(ach * 1e9 / PEAK_HBM, 4), "traffic": None,
                    "ms_per_launch": round(dp["ms"] / dp["calls"], 5)}
    if dom["bound"] == "hbm" and dp["flop"] > 0:
        # the same kernel seen as a contraction: algorithmic flops of the layers' definitions against the fp32 matrix
        # peak (the split-bf16 arithmetic runs on the bf16 cores, so this can exceed 1)
        fl = dp["flop"] / (dp["ms"] * 1e-3)
        roofline["as_contraction"] = {"bound": "mfma", "achieved": round(fl / 1e12, 3), "peak": PEAK_FP32_MFMA / 1e12,
                                      "unit": "TFLOP/s", "frac": round(fl / PEAK_FP32_MFMA, 4)}
    if args.net == "small" and N == 512:
        launches = {"conv12_fwd": [(N, T), (N * T, 1)], "fc_fwd": [(N, T), (N * T, 1)], "heads_fwd": [(N, T)]}
        roofline["traffic"] = counter_traffic(dom["stage"], launches.get(dom["stage"], [(N * T, 1)]))
        roofline["algorithmic_bytes_per_launch"] = round(dp["bytes"] / dp["calls"]) if dp["bytes"] > 0 else None
    flop_step = sum(p["flop"] for p in prof.values()) / args.steps
    whole = {"tflops": round(flop_step / sec / 1e12, 3), "frac_fp32_mfma_peak": round(flop_step / sec / PEAK_FP32_MFMA, 4)}
    torch.cuda.synchronize()

    theta_np = net.params_get(0).cpu().numpy()
    out = {
        "metric": "frames/s through predict and train_step, balanced (PPS = TPS*t_max)",
        "value": round(frames_per_step / sec, 1), "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if args.math == 0 else "bf16", "data": "synthetic",
        "arithmetic": ("fp32 accuracy with fp32 accumulation: fp32 MFMA, or fp32 operands split exactly into three bf16 "
                       "terms on the bf16 MFMA (bytes are exact in bf16)") if args.math == 0 else
                      "operands of every contraction rounded to bfloat16, exact products, fp32 accumulation, fp32 parameters",
        "config": {"workload": f"configs[1]+[2]: {args.net} net, 18 actions; per step {T}x predict B={N} "
                               f"and 1 train_step {N} agents x t_max={T} = {N * T} frames, "
                               "clip 40; " + ("predictions and training on two streams" if args.streams == 2 else
                                              "one stream"), "agents": N, "t_max": T, "seed": seed, "streams": args.streams},
        "one_stream": {"value": round(frames_per_step / sec_one, 1), "ms_per_step": round(sec_one * 1e3, 4)},
        "two_streams": {"value": round(frames_per_step / sec_two, 1), "ms_per_step": round(sec_two * 1e3, 4)} if sec_two else None,
        "pps_predict_only": {"value": round(1024 / pred_sec, 1), "batch": 1024, "ms_per_call": round(pred_sec * 1e3, 4)},
        "tps_train_only": {"value": round(frames_per_step / train_sec, 1), "frames": frames_per_step,
                           "ms_per_call": round(train_sec * 1e3, 4), "paper_tps_batches_of_5": round(N / train_sec, 1)},
        "whole_step": whole,
        "roofline": roofline,
        "stages": stages,
    }

    if args.rmsprop_big:
        n = 1 << 28
        th = torch.zeros(n, device="cuda"); gg = torch.zeros(n, device="cuda"); dd = torch.ones(n, device="cuda")
        f = lambda: g.rmsprop_flat(th, gg, dd, 1.0, 3e-4, 0.99, 0.1, stream=stream)
        f(); f()
        s = timed(f, 10)
        out["rmsprop_2p28"] = {"gbps": round(20.0 * n / s / 1e9, 1), "frac_hbm_peak": round(20.0 * n / s / PEAK_HBM, 4),
                               "ms": round(s * 1e3, 4)}
        del th, gg, dd

    net.close()
    net = None
    if args.mixed_seconds > 0:
        # synthetic agents through the two-stream scheduler (bench_mixed.py): 256 agents with fixed caps, then adaptive caps
        from bench_mixed import run_mixed
        out["mixed_load"] = [run_mixed(args.net, think_us=0.0, seconds=args.mixed_seconds, dynamic=False),
                             run_mixed(args.net, think_us=0.0, seconds=2 * args.mixed_seconds, dynamic=True),
                             # enough agents to keep several batches in flight: what the whole queue system sustains
                             run_mixed(args.net, n_agents=2048, think_us=0.0, seconds=args.mixed_seconds, dynamic=False,
                                       predict_cap=1024, train_cap=2560),
                             # the same with 2 % of the actions ending an episode: updates on segments of unequal length
                             run_mixed(args.net, n_agents=2048, think_us=0.0, seconds=args.mixed_seconds, dynamic=False,
                                       predict_cap=1024, train_cap=2560, episode_end_prob=0.02)]

    if not args.no_cpu_baseline:
        import oracle as orc
        onet = orc.Net(conv=tuple(desc.conv), fc_units=desc.fc_units, n_actions=A, math=args.math)
        theta = theta_np.astype(np.float64)
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        t0 = time.perf_counter()
        cpu_steps = 0
        while cpu_steps < 1 or (time.perf_counter() - t0 < 10.0 and cpu_steps < 64):     # about 10 s of CPU work
            bo = None
            for t in range(T):
                out_t = orc.forward(onet, theta, frames_np[:, t])
                if t == 0:
                    bo = out_t["values"]
            orc.train_step(onet, theta, np.zeros_like(theta), frames_np, tr["actions"], tr["rewards"], tr["dones"], bo,
                           orc.HParams(clip_norm=40.0))
            cpu_steps += 1
        cpu_sec = (time.perf_counter() - t0) / cpu_steps
        out["cpu_baseline"] = {"value": round(frames_per_step / cpu_sec, 1), "unit": "frames/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"{cpu_steps} whole steps of the same workload ({cpu_sec:.2f} s each, fp64, OpenMP over frames)"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
