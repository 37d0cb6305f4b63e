#!/usr/bin/env python3
"""Benchmark of the GA3C hot path on one MI355X.

A step is one balanced pass of the whole path (Sec. 4.2 of the paper: in a
balanced configuration PPS ~ TPS * t_max): t_max = 5 prediction calls of N
frames each, one per action of every agent, followed by one training step on
the N agents x 5 frames those actions produced (the bootstrap value of a
segment is the value of the next segment's first prediction, so no sixth
prediction is needed).  N = 512 agents, the small network of Sec. 3.2 with 18
actions, synthetic game-like frames that are resident in HBM before the timed
region starts.  Four distinct sets of frames and trajectories (289 MB of
frames, more than the 256 MB last-level cache) take turns, so that a step
never finds its frames where the previous step left them.  By default the
step is submitted the way the paper's predictor and trainer threads do it
(Sec. 4.1): the five predictions on one stream, the training step (on the
segment the previous step predicted) on another, so that the two calls share
the GPU; `--streams 1` issues the six calls one after another (the default run
measures that too and reports both rates).

Timing: W warm-up steps, then TEN blocks of K steps each, every block
bracketed by torch.cuda.synchronize(); `ms_per_step` and `value` are the
median block, `spread` holds min / median / max.

Prints ONE JSON line.  `value` = frames per second through predict AND
train_step (each frame is predicted once and trained on once).  The line also
carries: predict-only and train-only rates; per-stage times (the execution
time of each stage's kernel between two HIP events that the runtime stamps at
the start and the end of that very dispatch, on the call's own stream: the
same figure a kernel trace shows, a one-stream pass); the roofline of the
dominant kernel; the
prediction sweep (batch 1 .. 1024); the larger network (predict 256, train
1280; fp32-grade and bfloat16-operand arithmetic); RMSProp on 2^28 parameters;
the queue system under synthetic agents (fixed caps against the Sec. 4.3
adjustment, small and large net, four think times); and the fp64 CPU oracle
timed on the same workload.

Roofline conventions.  FLOP = 2 per multiply-add of a layer's definition
("algorithmic").  Every contraction here executes on the bf16 matrix cores
(peak 2.5 PFLOP/s dense): with fp32-grade accuracy an fp32 operand is the exact
sum of three bf16 terms, so a layer costs 3 (bytes x fp32) or 6 (fp32 x fp32)
MFMAs per nominal one ("executed" FLOP); with --math 1 it costs one.  A stage's
`frac` is algorithmic FLOP/s over the bf16 peak; `executed_frac` counts the
MFMAs that actually run; both are at most 1.  The one fp32-MFMA kernel left
(conv weight gradients of layers 2 and 3) is priced against 157.3 TFLOP/s.
`fp32_equivalent_tflops` is the algorithmic rate again, for comparison with
an fp32-MFMA implementation; it is not a roofline fraction.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15     # MI355X dense bf16 matrix, FLOP/s
PEAK_FP32_MFMA = 157.3e12   # dense fp32 matrix
PEAK_HBM = 8.0e12           # B/s
TIMED_BLOCKS = 10

# HBM traffic per launch from hardware counters: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (two runs of
# `python3 bench.py --steps 3 --warmup 1 --streams 1 --no-cpu-baseline --only-step`), KiB per dispatch, small net,
# by frames in the launch.  Every read request on this chip is a 128-byte line while FETCH_SIZE prices it at 64
# bytes: on the streaming RMSProp kernel over 2^28 parameters (12 B read, 8 B written per parameter) the counters read
# 0.5000 and 1.0000 of the known bytes, hence the scale factors.  The summary is kept under profiles/.
FETCH_SCALE, WRITE_SCALE = 2.0, 1.0
COUNTER_KIB = {   # stage: {frames per launch: (FETCH_SIZE, WRITE_SIZE)}
    "conv12_fwd": {512: (7553.2, 5184.0), 1024: (14625.2, 10368.1), 2560: (35845.2, 89929.8)},   # 2560: training, keeps y1
    "fc_fwd": {512: (4153.5, 7168.0), 1024: (6649.5, 8192.0), 2560: (14425.5, 20480.5)},
    "heads_fwd": {512: (3761.5, 592.0), 1024: (4262.0, 1104.0)},
    "heads_train": {2560: (10529.0, 11960.4)},
    "conv1_wgrad": {2560: (67613.1, 4112.0)},
    "conv2_wgrad": {2560: (45157.9, 16450.1)},
    "conv2_dgrad": {2560: (45250.0, 64000.0)},
    "fc_wgrad": {2560: (19915.5, 20736.0)},
    "fc_dgrad": {2560: (25863.8, 26022.2)},
    "wgrad_reduce": {2560: (24263.6, 2728.5)},
    "rmsprop": {2560: (4064.8, 5496.2)},
}

# HIP kernel behind each stage of the small net's fast path, and the larger net's
KERNELS = {"conv12_fwd": "conv12_fused_fwd_kernel", "fc_fwd": "dense_gemm_bf16x6_kernel<2,2,2,2,k-major,k-major>",
           "fc_wgrad": "dense_gemm_bf16x6_kernel<2,2,2,2,row-major,row-major>",
           "fc_dgrad": "dense_gemm_bf16x6_kernel<4,2,2,2,k-major,row-major,mask>", "heads_fwd": "heads_fwd_kernel",
           "heads_train": "heads_train_kernel", "conv1_wgrad": "conv1_bf16x3_wgrad_kernel",
           "conv2_wgrad": "conv_wgrad_bf16x6_kernel", "conv3_wgrad": "conv_wgrad_s1_bf16x6_kernel",
           "conv2_dgrad": "conv_dgrad_bf16x6_kernel", "conv3_dgrad": "conv_fwd_bf16x6_kernel<dgrad>",
           "conv1_fwd": "conv1_bf16x3_fwd_kernel", "conv2_fwd": "conv_fwd_bf16x6_kernel", "conv3_fwd": "conv_fwd_bf16x6_kernel",
           "wgrad_reduce": "reduce_all_kernel", "rmsprop": "rmsprop_kernel", "predict_small": "predict_small_kernel"}
# bf16 MFMAs executed per nominal one with fp32-grade accuracy (operand split into three bf16 terms); "f32" = the
# stage runs on the fp32 matrix cores
TERMS = {"conv1_fwd": 3, "conv2_fwd": 6, "conv3_fwd": 6, "fc_fwd": 6, "fc_wgrad": 6, "fc_dgrad": 6, "conv1_wgrad": 3,
         "conv2_dgrad": 6, "conv3_dgrad": 6, "conv2_wgrad": 6, "conv3_wgrad": 6}
HBM_STAGES = {"rmsprop", "wgrad_reduce"}


def counter_traffic(stage, launches):
    """Mean HBM bytes per launch of a stage over `launches` = [(frames, count), ...]; None where not measured."""
    tab = COUNTER_KIB.get(stage)
    if not tab or any(b not in tab for b, _ in launches):
        return None
    tot = sum(n * (FETCH_SCALE * tab[b][0] + WRITE_SCALE * tab[b][1]) * 1024.0 for b, n in launches)
    return round(tot / sum(n for _, n in launches))


def spread(vals):
    return {"min": round(min(vals), 5), "median": round(statistics.median(vals), 5), "max": round(max(vals), 5)}


def rmsprop_2p28(g, torch, stream):
    """RMSProp (Eq. 3) on a buffer far larger than the caches: 2^28 parameters, 12 B read and 8 B written each."""
    n = 1 << 28
    th = torch.zeros(n, device="cuda"); gg = torch.zeros(n, device="cuda"); dd = torch.ones(n, device="cuda")
    f = lambda: g.rmsprop_flat(th, gg, dd, 1.0, 3e-4, 0.99, 0.1, stream=stream)
    f(); f()

    def blocks():
        out = []
        for _ in range(5):
            torch.cuda.synchronize(); t0 = time.perf_counter()
            for _ in range(5):
                f()
            torch.cuda.synchronize(); out.append((time.perf_counter() - t0) / 5)
        return out
    rs = blocks()
    s = statistics.median(rs)
    rec = {"kernel": "rmsprop_kernel", "bound": "hbm", "achieved": round(20.0 * n / s / 1e9, 1), "peak": PEAK_HBM / 1e9,
           "unit": "GB/s", "frac": round(20.0 * n / s / PEAK_HBM, 4), "ms": spread([x * 1e3 for x in rs]),
           "bytes_per_parameter": 20, "parameters": n}
    del th, gg, dd
    torch.cuda.empty_cache()
    return rec


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--agents", type=int, default=512)
    ap.add_argument("--net", choices=("small", "large"), default="small")
    ap.add_argument("--math", type=int, choices=(0, 1), default=0,
                    help="0: fp32 accuracy (default); 1: operands of every contraction rounded to bfloat16")
    ap.add_argument("--streams", type=int, choices=(1, 2), default=2,
                    help="2: predictions on one stream, training on another (predictor and trainer threads of "
                         "Sec. 4.1 share the GPU); 1: the six calls of a step one after another")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-step", action="store_true",
                    help="the step and its stages only: no sweep, larger net, big RMSProp or queue system (for profilers)")
    ap.add_argument("--only-rmsprop", action="store_true",
                    help="RMSProp over 2^28 parameters only (a kernel of known traffic: the calibration of the HBM counters)")
    ap.add_argument("--mixed-seconds", type=float, default=1.5,
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
    if args.only_rmsprop:
        print(json.dumps({"rmsprop_2p28": rmsprop_2p28(g, torch, torch.cuda.current_stream())}))
        return 0
    N, T, A = args.agents, 5, 18
    NSETS = 4
    desc = dataclasses.replace(g.SMALL_NET(A) if args.net == "small" else g.LARGE_NET(A), math=args.math)
    net = g.Ga3c(desc, max(N, 1024), N * T)
    net.params_init(synth.BASE_SEED)
    hp = g.HParams(clip_norm=40.0)
    stream = torch.cuda.current_stream()

    seed = synth.BASE_SEED + 2
    sets = []
    for k in range(NSETS):
        fr_np = synth.rectangle_frames_tiled(seed + 100 * k, N * T).reshape(N, T, 4, 84, 84)
        tr = synth.trajectories(seed + 100 * k + 1, N, T, A)
        fr = torch.from_numpy(fr_np).cuda()
        sets.append(dict(frames_np=fr_np, tr=tr, frames=fr,
                         # predict call t sees the frames of step t of every agent
                         pframes=[fr[:, t].contiguous() for t in range(T)],
                         actions=torch.from_numpy(tr["actions"]).cuda(), rewards=torch.from_numpy(tr["rewards"]).cuda(),
                         dones=torch.from_numpy(tr["dones"]).cuda()))
    uniforms = torch.from_numpy(synth.uniforms(seed + 3, N)).cuda()
    logits = torch.empty(N, A, device="cuda"); values = torch.empty(N, device="cuda")
    probs = torch.empty(N, A, device="cuda"); sampled = torch.empty(N, dtype=torch.int32, device="cuda")
    boot = torch.empty(N, device="cuda")
    stats = torch.zeros(8, device="cuda")
    count = [0]

    def step():
        # one prediction per frame: the value that closes a segment's returns, V(s_{t+t_max}), is what the agent is
        # told by the first prediction of its next segment (Sec. 4.1), so a segment costs t_max predictions, not
        # t_max + 1; with synthetic states the values of prediction 0 stand in for it
        d = sets[count[0] % NSETS]; count[0] += 1
        for t in range(T):
            net.predict(d["pframes"][t], uniforms=uniforms, logits=logits, values=boot if t == 0 else values, probs=probs,
                        actions=sampled, stream=stream)
        net.train_step(d["frames"], d["actions"], d["rewards"], d["dones"], boot, hp, stats=stats, stream=stream)

    def timed_blocks(fn, k, blocks=TIMED_BLOCKS):
        out = []
        for _ in range(blocks):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(k):
                fn()
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t0) / k)
        return out

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
        d, dprev = sets[i % NSETS], sets[(i - 1) % NSETS]
        s_pred.wait_event(ev_train[i % 3])               # the training step that last read this set is done
        for t in range(T):
            net.predict(d["pframes"][t], uniforms=uniforms, logits=logits, values=boots[i % 3] if t == 0 else values,
                        probs=probs, actions=sampled, stream=s_pred)
        ev_pred[i % 3].record(s_pred)
        s_train.wait_event(ev_pred[(i - 1) % 3])         # values written by the predictions of segment i - 1
        net.train_step(dprev["frames"], dprev["actions"], dprev["rewards"], dprev["dones"], boots[(i - 1) % 3], hp,
                       stats=stats, stream=s_train)
        ev_train[(i - 1) % 3].record(s_train)

    for _ in range(args.warmup):
        step()
    one = timed_blocks(step, args.steps)
    two = None
    if args.streams == 2:
        for _ in range(args.warmup):
            step_two_streams()
        two = timed_blocks(step_two_streams, args.steps)
    secs = two if args.streams == 2 else one
    sec = statistics.median(secs)
    frames_per_step = N * T

    # predict-only and train-only rates (the frame sets take turns here too)
    bigs = [torch.from_numpy(synth.rectangle_frames_tiled(seed + 4 + k, 1024)).cuda() for k in range(NSETS)]
    bl = torch.empty(1024, A, device="cuda"); bv = torch.empty(1024, device="cuda")
    pc, tc = [0], [0]

    def pred_fn():
        pc[0] += 1
        net.predict(bigs[pc[0] % NSETS], logits=bl, values=bv, stream=stream)

    def train_fn():
        tc[0] += 1
        d = sets[tc[0] % NSETS]
        net.train_step(d["frames"], d["actions"], d["rewards"], d["dones"], boot, hp, stats=stats, stream=stream)

    for _ in range(3):
        pred_fn(); train_fn()
    pred_secs = timed_blocks(pred_fn, max(args.steps, 20), 5)
    train_secs = timed_blocks(train_fn, max(args.steps, 20), 5)
    pred_sec, train_sec = statistics.median(pred_secs), statistics.median(train_secs)

    # per-stage times: an event pair per kernel launch, stamped at the dispatch's own start and end
    net.profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = net.profile_read()
    net.profile_enable(False)
    g0_flop = 2.0 * 400 * 16 * 256            # small net, per frame: conv1, conv2 (what the fused kernel's 3 and 6 terms apply to)
    g1_flop = 2.0 * 81 * 32 * 256
    stages = []
    for name, p in prof.items():
        t_s = p["ms"] * 1e-3
        e = {"stage": name, "kernel": KERNELS.get(name, name), "calls_per_step": p["calls"] / args.steps,
             "ms_per_call": round(p["ms"] / p["calls"], 5), "ms_per_step": round(p["ms"] / args.steps, 5)}
        if p["bytes"] > 0:
            e["algorithmic_gbps"] = round(p["bytes"] / t_s / 1e9, 2)
        if name in HBM_STAGES and p["bytes"] > 0:
            e.update(bound="hbm", peak=PEAK_HBM / 1e9, unit="GB/s", achieved=e["algorithmic_gbps"],
                     frac=round(p["bytes"] / t_s / PEAK_HBM, 4))
        elif p["flop"] > 0 and (name in TERMS or name == "conv12_fwd"):
            terms = 1 if args.math == 1 and TERMS.get(name) != "f32" else TERMS.get(name)
            alg = p["flop"] / t_s
            if terms == "f32":
                e.update(bound="mfma", dtype="f32", peak=PEAK_FP32_MFMA / 1e12, unit="TFLOP/s", achieved=round(alg / 1e12, 3),
                         frac=round(alg / PEAK_FP32_MFMA, 4), executed_frac=round(alg / PEAK_FP32_MFMA, 4))
            else:
                if name == "conv12_fwd":
                    executed = alg if args.math == 1 else alg * (3 * g0_flop + 6 * g1_flop) / (g0_flop + g1_flop)
                else:
                    executed = alg * terms
                e.update(bound="mfma", dtype="bf16", peak=PEAK_BF16_MFMA / 1e12, unit="TFLOP/s", achieved=round(alg / 1e12, 3),
                         frac=round(alg / PEAK_BF16_MFMA, 4), executed_tflops=round(executed / 1e12, 3),
                         executed_frac=round(executed / PEAK_BF16_MFMA, 4), fp32_equivalent_tflops=round(alg / 1e12, 3))
                if p["bytes"] > 0:
                    e["hbm_frac_by_algorithmic_bytes"] = round(p["bytes"] / t_s / PEAK_HBM, 4)
        else:
            e["bound"] = "latency"          # kilobytes of work per launch: the time is reported, not a fraction
        stages.append(e)
    stages.sort(key=lambda e: -e["ms_per_step"])
    dom = next(e for e in stages if e.get("bound") in ("mfma", "hbm"))
    dp = prof[dom["stage"]]
    roofline = {"kernel": dom["kernel"], "stage": dom["stage"], "bound": dom["bound"], "achieved": dom["achieved"],
                "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac"], "traffic": None,
                "ms_per_launch": round(dp["ms"] / dp["calls"], 5), "launches_per_step": dp["calls"] / args.steps}
    for k in ("dtype", "executed_tflops", "executed_frac", "fp32_equivalent_tflops", "hbm_frac_by_algorithmic_bytes"):
        if k in dom:
            roofline[k] = dom[k]
    if args.net == "small" and N == 512:
        launches = {"conv12_fwd": [(N, T), (N * T, 1)], "fc_fwd": [(N, T), (N * T, 1)], "heads_fwd": [(N, T)]}
        roofline["traffic"] = counter_traffic(dom["stage"], launches.get(dom["stage"], [(N * T, 1)]))
        roofline["algorithmic_bytes_per_launch"] = round(dp["bytes"] / dp["calls"]) if dp["bytes"] > 0 else None
    flop_step = sum(p["flop"] for p in prof.values()) / args.steps
    whole = {"algorithmic_tflops": round(flop_step / sec / 1e12, 3),
             "frac_of_bf16_mfma_peak": round(flop_step / sec / PEAK_BF16_MFMA, 4),
             "fp32_equivalent_tflops": round(flop_step / sec / 1e12, 3)}
    torch.cuda.synchronize()

    theta_np = net.params_get(0).cpu().numpy()
    out = {
        "metric": "frames/s through predict and train_step, balanced (PPS = TPS*t_max)",
        "value": round(frames_per_step / sec, 1), "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "timed_blocks": TIMED_BLOCKS,
        "ms_per_step": round(sec * 1e3, 4), "spread_ms_per_step": spread([s * 1e3 for s in secs]),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if args.math == 0 else "bf16", "data": "synthetic",
        "arithmetic": ("fp32 accuracy with fp32 accumulation: fp32 operands split exactly into three bf16 terms on the bf16 "
                       "MFMA (bytes are exact in bf16); one weight-gradient kernel on the fp32 MFMA") if args.math == 0 else
                      "operands of every contraction rounded to bfloat16, exact products, fp32 accumulation, fp32 parameters",
        "config": {"workload": f"configs[1]+[2]: {args.net} net, 18 actions; per step {T}x predict B={N} "
                               f"and 1 train_step {N} agents x t_max={T} = {N * T} frames, "
                               "clip 40; " + ("predictions and training on two streams" if args.streams == 2 else
                                              "one stream"), "agents": N, "t_max": T, "seed": seed, "streams": args.streams,
                   "frame_sets": NSETS, "frame_bytes_resident": NSETS * N * T * 4 * 84 * 84},
        "one_stream": {"value": round(frames_per_step / statistics.median(one), 1), "ms_per_step": spread([s * 1e3 for s in one])},
        "two_streams": {"value": round(frames_per_step / statistics.median(two), 1),
                        "ms_per_step": spread([s * 1e3 for s in two])} if two else None,
        "pps_predict_only": {"value": round(1024 / pred_sec, 1), "batch": 1024, "ms_per_call": spread([s * 1e3 for s in pred_secs])},
        "tps_train_only": {"value": round(frames_per_step / train_sec, 1), "frames": frames_per_step,
                           "ms_per_call": spread([s * 1e3 for s in train_secs]), "paper_tps_batches_of_5": round(N / train_sec, 1)},
        "whole_step": whole,
        "roofline": roofline,
        "stages": stages,
    }
    net.close()
    net = None

    if not args.only_step:
        # ---- prediction sweep, small net (config 1): calls back to back, 200 per batch size
        snet = g.Ga3c(dataclasses.replace(g.SMALL_NET(A), math=args.math), 1024, 0)
        snet.params_init(synth.BASE_SEED)
        sweep = []
        for B in [1 << i for i in range(11)]:
            fr = bigs[0][:B].contiguous()
            lg = torch.empty(B, A, device="cuda"); vl = torch.empty(B, device="cuda"); ac = torch.empty(B, dtype=torch.int32, device="cuda")
            fn = lambda: snet.predict(fr, uniforms=uniforms[:B] if B <= N else None, logits=lg, values=vl,
                                      actions=ac if B <= N else None, stream=stream)
            for _ in range(10):
                fn()
            s = statistics.median(timed_blocks(fn, 100, 3))
            sweep.append({"batch": B, "pps": round(B / s, 1), "us_per_call": round(s * 1e6, 2)})
        snet.close()
        out["predict_sweep_small_net"] = sweep

        # ---- the larger network (config 3): predict 256, train 256 x 5, both arithmetic variants
        large = []
        for m in (0, 1):
            ln = g.Ga3c(dataclasses.replace(g.LARGE_NET(A), math=m), 256, 1280)
            ln.params_init(synth.BASE_SEED)
            d = sets[0]
            lfr = d["frames"][:256].contiguous()
            pfr = lfr[:, 0].contiguous()
            lb = torch.empty(256, device="cuda"); ll = torch.empty(256, A, device="cuda")
            pf = lambda: ln.predict(pfr, logits=ll, values=lb, stream=stream)
            tf = lambda: ln.train_step(lfr, d["actions"][:256].contiguous(), d["rewards"][:256].contiguous(),
                                       d["dones"][:256].contiguous(), lb, hp, stream=stream)
            for _ in range(3):
                pf(); tf()
            ps = statistics.median(timed_blocks(pf, 50, 3)); ts = statistics.median(timed_blocks(tf, 20, 3))
            fwd_flop, train_flop = 18.7e6, 49.56e6           # per frame, from the layers' definitions
            large.append({"math": m, "dtype": "f32" if m == 0 else "bf16",
                          "predict_256": {"pps": round(256 / ps, 1), "us_per_call": round(ps * 1e6, 1),
                                          "algorithmic_tflops": round(256 * fwd_flop / ps / 1e12, 2),
                                          "frac_of_bf16_mfma_peak": round(256 * fwd_flop / ps / PEAK_BF16_MFMA, 4)},
                          "train_1280": {"tps_frames": round(1280 / ts, 1), "us_per_call": round(ts * 1e6, 1),
                                         "algorithmic_tflops": round(1280 * train_flop / ts / 1e12, 2),
                                         "frac_of_bf16_mfma_peak": round(1280 * train_flop / ts / PEAK_BF16_MFMA, 4)}})
            ln.close()
        out["large_net"] = large

        out["rmsprop_2p28"] = rmsprop_2p28(g, torch, stream)

    if args.mixed_seconds > 0 and not args.only_step:
        # synthetic agents through the two-stream scheduler (bench_mixed.py): 256 closed-loop agents; fixed caps
        # against the Sec. 4.3 adjustment started at 32 / 320, for four mean think times and both nets
        from bench_mixed import run_mixed
        runs = []
        for netk in ("small", "large"):
            for th_us in (0.0, 200.0, 2000.0, 20000.0):
                if netk == "large" and th_us not in (0.0, 200.0):
                    continue
                runs.append(run_mixed(netk, think_us=th_us, seconds=args.mixed_seconds, dynamic=False))
                runs.append(run_mixed(netk, think_us=th_us, seconds=2 * args.mixed_seconds, dynamic=True))
        # enough agents to keep several batches in flight: what the whole queue system sustains
        runs.append(run_mixed("small", n_agents=2048, think_us=0.0, seconds=args.mixed_seconds, dynamic=False,
                              predict_cap=1024, train_cap=2560))
        # the same with 2 % of the actions ending an episode: updates on segments of unequal length
        runs.append(run_mixed("small", n_agents=2048, think_us=0.0, seconds=args.mixed_seconds, dynamic=False,
                              predict_cap=1024, train_cap=2560, episode_end_prob=0.02))
        out["mixed_load"] = runs

    if not args.no_cpu_baseline:
        import oracle as orc
        onet = orc.Net(conv=tuple(desc.conv), fc_units=desc.fc_units, n_actions=A, math=args.math)
        theta = theta_np.astype(np.float64)
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        d = sets[0]
        t0 = time.perf_counter()
        cpu_steps = 0
        while cpu_steps < 1 or (time.perf_counter() - t0 < 10.0 and cpu_steps < 64):     # about 10 s of CPU work
            bo = None
            for t in range(T):
                out_t = orc.forward(onet, theta, d["frames_np"][:, t])
                if t == 0:
                    bo = out_t["values"]
            orc.train_step(onet, theta, np.zeros_like(theta), d["frames_np"], d["tr"]["actions"], d["tr"]["rewards"],
                           d["tr"]["dones"], bo, orc.HParams(clip_norm=40.0))
            cpu_steps += 1
        cpu_sec = (time.perf_counter() - t0) / cpu_steps
        out["cpu_baseline"] = {"value": round(frames_per_step / cpu_sec, 1), "unit": "frames/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"{cpu_steps} whole steps of the same workload ({cpu_sec:.2f} s each, fp64, OpenMP over frames)"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
