#!/usr/bin/env python3
"""Sweeps of the two calls on one MI355X, on seeded synthetic game-like frames:

  * prediction only, small net of Sec. 3.2 with 18 actions, batch 1, 2, 4, ... 1024:
    predictions/s with calls issued back to back, and the latency of a single call
    (median of 200 calls bracketed by HIP events, after 20 warm-up calls);
  * training only, the same net, N = 32, 128, 512 agents x t_max = 5, clip 40: trained frames/s;
  * the larger net (conv 32@8x8s4, 64@4x4s2, 64@3x3s1, fc 512): predict 256, train 256 x 5;
  * the paper's own larger networks (Sec. 5, "GPU utilization and DNN size": conv 32@8x8 with stride 4, 3, 2 or 1,
    conv 32@4x4s2, conv 64@4x4s2, fc 256, or 1024 for stride 1): predict 128, train 128 x 5 (128 agents is the
    paper's fastest setting).

Prints one JSON object.  `bench.py` remains the benchmark of record; this is the
table behind it.
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    args = ap.parse_args()

    import numpy as np
    import torch

    import ga3c_synth as synth
    import paper_1611_06256_amd as g

    if not torch.cuda.is_available():
        print("bench_sweep.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    A, T = 18, 5
    seed = synth.BASE_SEED + 1

    def back_to_back(fn, k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / k

    def single_call_latency(fn, k):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(k)]
        for a, b in ev:
            torch.cuda.synchronize()
            a.record(stream); fn(); b.record(stream)
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in ev])) * 1e3     # us

    def predict_rows(desc, batches):
        net = g.Ga3c(desc, max(batches), 0)
        net.params_init(seed)
        pool = torch.from_numpy(synth.rectangle_frames_tiled(seed, max(batches))).cuda()
        u = torch.from_numpy(synth.uniforms(seed + 1, max(batches))).cuda()
        rows = []
        for B in batches:
            fr = pool[:B].contiguous()
            lg = torch.empty(B, A, device="cuda"); vl = torch.empty(B, device="cuda")
            ac = torch.empty(B, dtype=torch.int32, device="cuda")
            fn = lambda: net.predict(fr, uniforms=u[:B], logits=lg, values=vl, actions=ac, stream=stream)
            for _ in range(args.warmup):
                fn()
            sec = back_to_back(fn, args.reps)
            lat = single_call_latency(fn, args.reps)
            rows.append({"batch": B, "pps": round(B / sec, 1), "us_per_call_back_to_back": round(sec * 1e6, 2),
                         "latency_us_median_events": round(lat, 2)})
        net.close()
        return rows

    def train_rows(desc, agents):
        net = g.Ga3c(desc, max(agents), max(agents) * T)
        net.params_init(seed)
        hp = g.HParams(clip_norm=40.0)
        rows = []
        for N in agents:
            fr = torch.from_numpy(synth.rectangle_frames_tiled(seed + 2, N * T).reshape(N, T, 4, 84, 84)).cuda()
            tr = synth.trajectories(seed + 3, N, T, A)
            ac = torch.from_numpy(tr["actions"]).cuda(); rw = torch.from_numpy(tr["rewards"]).cuda()
            dn = torch.from_numpy(tr["dones"]).cuda()
            boot = torch.empty(N, device="cuda")
            net.predict(fr[:, 0].contiguous(), values=boot, stream=stream)
            fn = lambda: net.train_step(fr, ac, rw, dn, boot, hp, stream=stream)
            for _ in range(max(3, args.warmup // 4)):
                fn()
            sec = back_to_back(fn, max(20, args.reps // 4))
            rows.append({"agents": N, "frames": N * T, "tps_frames": round(N * T / sec, 1),
                         "us_per_call": round(sec * 1e6, 2)})
        net.close()
        return rows

    out = {"data": "synthetic", "seed": seed, "n_gpus": 1, "dtype": "f32",
           "small_net_predict": predict_rows(g.SMALL_NET(A), [1 << i for i in range(11)]),
           "small_net_train": train_rows(g.SMALL_NET(A), [32, 128, 512]),
           "large_net_predict": predict_rows(g.LARGE_NET(A), [256]),
           "large_net_train": train_rows(g.LARGE_NET(A), [256])}
    family = []
    for stride in (4, 3, 2, 1):
        desc = g.NetDesc(in_c=4, in_h=84, in_w=84, conv=((32, 8, stride), (32, 4, 2), (64, 4, 2)),
                         fc_units=1024 if stride == 1 else 256, n_actions=A)
        family.append({"conv1_stride": stride, "predict": predict_rows(desc, [128])[0], "train": train_rows(desc, [128])[0]})
    out["paper_family"] = family
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
