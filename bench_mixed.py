#!/usr/bin/env python3
"""Steady-state mixed load on one GPU: synthetic agents feed the prediction
queue and the training queue of the scheduler (paper Sec. 4.1), whose batch
caps adapt every 1000 ticks (Sec. 4.3).

Each of the 256 agents is a closed loop: ask for an action, wait for it, "think"
for an exponentially distributed time (seeded; it stands in for the emulator
step), ask again; after t_max = 5 actions it hands in a 5-step trajectory whose
bootstrap is the value it was just told.  Frames are synthetic and sit in HBM.
Reports, per mean think time: predictions/s, trained frames/s, mean prediction
batch, mean training-queue length (the quantities of the paper's Fig. 4) and
the caps the adjustment ended with.  The driver loop is Python (numpy, one
ctypes call per batch of requests); its cost per tick is reported too.
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


def run_mixed(net_kind: str = "small", n_agents: int = 256, think_us: float = 0.0, seconds: float = 1.0,
              dynamic: bool = True, seed: int = 1615, predict_cap: int = 256, train_cap: int = 1280):
    import numpy as np
    import torch

    import ga3c_synth as synth
    import paper_1611_06256_amd as g

    T, A = 5, 18
    desc = g.SMALL_NET(A) if net_kind == "small" else g.LARGE_NET(A)
    net = g.Ga3c(desc, predict_cap, train_cap)
    net.params_init(seed)
    pool = torch.from_numpy(synth.rectangle_frames_tiled(seed, n_agents * T).reshape(n_agents, T, 4, 84, 84)).cuda()
    torch.cuda.synchronize()
    fb = 4 * 84 * 84
    base = pool.data_ptr()
    sched = g.Scheduler(net, g.HParams(clip_norm=40.0), t_max=T, predict_cap=predict_cap if not dynamic else 32, train_min=40,
                        train_cap=train_cap if not dynamic else 320, adjust_period=1000 if dynamic else 0, predict_cap_lo=1,
                        predict_cap_hi=predict_cap, train_cap_lo=40, train_cap_hi=train_cap, train_cap_step=40, seed=seed)
    rng = synth.rng(seed + 1)
    step = np.zeros(n_agents, np.int64)
    waiting = np.zeros(n_agents, bool)
    ready_at = np.zeros(n_agents)
    acts = np.zeros((n_agents, T), np.int32)
    ids = np.arange(n_agents, dtype=np.int32)
    t0 = time.perf_counter()
    ticks = 0
    while True:
        now = time.perf_counter() - t0
        if now > seconds:
            break
        go = (~waiting) & (ready_at <= now)
        if go.any():
            a = ids[go]
            sched.submit_predict_many(a, base + (a.astype(np.uint64) * T + (step[a] % T).astype(np.uint64)) * fb,
                                      rng.random(a.size, dtype=np.float32))
            waiting[a] = True
        sched.tick()
        ticks += 1
        a, action, value = sched.poll_arrays()
        if a.size:
            acts[a, step[a] % T] = action
            step[a] += 1
            waiting[a] = False
            ready_at[a] = now + (rng.exponential(think_us * 1e-6, a.size) if think_us > 0 else 0.0)
            done = a[step[a] % T == 0]
            if done.size:
                u = rng.random((done.size, T))
                rewards = np.where(u < 0.05, -1.0, np.where(u >= 0.95, 1.0, 0.0)).astype(np.float32)
                dones = (rng.random((done.size, T)) < 0.02).astype(np.uint8)
                # the bootstrap is the value of the newest state the agent knows
                vmap = dict(zip(a.tolist(), value.tolist()))
                sched.submit_trajectory_many(done, base + done.astype(np.uint64) * T * fb, acts[done], rewards, dones,
                                             np.array([vmap[int(i)] for i in done], np.float32))
    sched.drain()
    wall = time.perf_counter() - t0
    st = sched.stats()
    out = {"agents": n_agents, "think_us": think_us, "dynamic": dynamic, "seconds": round(wall, 3),
           "pps": round(st["predictions"] / wall, 1), "tps_frames": round(st["trained_frames"] / wall, 1),
           "mean_predict_batch": round(st["predictions"] / max(1, st["predict_batches"]), 2),
           "mean_train_batch_frames": round(st["trained_frames"] / max(1, st["train_batches"]), 1),
           "mean_train_queue": round(st["sum_train_queue"] / max(1, st["ticks"]), 2),
           "predict_cap": st["predict_cap"], "train_cap": st["train_cap"],
           "trials_accepted": st["trials_accepted"], "trials_rejected": st["trials_rejected"],
           "host_us_per_tick": round(wall / max(1, ticks) * 1e6, 1)}
    sched.close()
    net.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--net", choices=("small", "large"), default="small")
    ap.add_argument("--seconds", type=float, default=1.5)
    ap.add_argument("--think-us", type=float, nargs="*", default=[0.0, 200.0, 2000.0, 20000.0])
    args = ap.parse_args()
    rows = []
    for th in args.think_us:
        rows.append(run_mixed(args.net, think_us=th, seconds=args.seconds, dynamic=True))
    rows.append(run_mixed(args.net, think_us=0.0, seconds=args.seconds, dynamic=False))
    print(json.dumps({"metric": "mixed load, 256 synthetic agents, one GPU, two streams", "net": args.net,
                      "data": "synthetic", "runs": rows}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
