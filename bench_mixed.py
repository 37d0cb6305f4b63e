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

With --episode-end-prob p > 0 every action ends the agent's episode with
probability p: the agent then hands in the shorter segment at once, terminal
at its last step (Sec. 4.1), so updates run on segments of unequal length.
Every segment carries the version of the policy that chose its first action;
the scheduler reports the policy lag in updates (Sec. 4.2).  --min-batch-sweep
runs fixed caps with the minimum training batch set to 5, 10, 20, 40, 80, 160,
320 frames (the knob of Sec. 5.3), for the first two think times given.
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
              dynamic: bool = True, seed: int = 1615, predict_cap: int = 256, train_cap: int = 1280,
              train_min: int = 40, episode_end_prob: float = 0.0, adjust_period: int = 1000, trace: bool = False):
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
    sched = g.Scheduler(net, g.HParams(clip_norm=40.0), t_max=T, predict_cap=predict_cap if not dynamic else 32,
                        train_min=train_min,
                        train_cap=train_cap if not dynamic else 320, adjust_period=adjust_period if dynamic else 0, predict_cap_lo=1,
                        predict_cap_hi=predict_cap, train_cap_lo=max(40, train_min), train_cap_hi=train_cap, train_cap_step=40, seed=seed)
    rng = synth.rng(seed + 1)
    step = np.zeros(n_agents, np.int64)          # actions taken so far (picks the frame shown)
    seg_len = np.zeros(n_agents, np.int32)       # experiences gathered since the last hand-in
    seg_ver = np.zeros(n_agents, np.int64)       # version of the policy that chose the segment's first action
    waiting = np.zeros(n_agents, bool)
    ready_at = np.zeros(n_agents)
    acts = np.zeros((n_agents, T), np.int32)
    ids = np.arange(n_agents, dtype=np.int32)
    t0 = time.perf_counter()
    ticks = 0
    windows_seen = []
    half = None                                  # (time, trained frames, predictions) once half of the run is over
    while True:
        now = time.perf_counter() - t0
        if now > seconds:
            break
        if half is None and now > 0.5 * seconds:
            st = sched.stats()
            half = (now, st["trained_frames"], st["predictions"])
        go = (~waiting) & (ready_at <= now)
        if go.any():
            a = ids[go]
            sched.submit_predict_many(a, base + (a.astype(np.uint64) * T + (step[a] % T).astype(np.uint64)) * fb,
                                      rng.random(a.size, dtype=np.float32))
            waiting[a] = True
        sched.tick()
        ticks += 1
        if dynamic and ticks % adjust_period == 0:    # the window that just closed: its reading and the caps proposed next
            st = sched.stats()
            windows_seen.append((st["windows"], round(st["last_window_frames_per_s"]), st["predict_cap"], st["train_cap"],
                                 st["trials_accepted"], st["trials_rejected"], round(now, 4)))
        a, action, value, version = sched.poll_arrays(with_version=True)
        if a.size:
            first = seg_len[a] == 0
            seg_ver[a[first]] = version[first]
            acts[a, seg_len[a]] = action
            step[a] += 1
            seg_len[a] += 1
            waiting[a] = False
            ready_at[a] = now + (rng.exponential(think_us * 1e-6, a.size) if think_us > 0 else 0.0)
            ended = rng.random(a.size) < episode_end_prob if episode_end_prob > 0 else np.zeros(a.size, bool)
            hand = (seg_len[a] == T) | ended
            done = a[hand]
            if done.size:
                lens = seg_len[done].copy()
                u = rng.random((done.size, T))
                rewards = np.where(u < 0.05, -1.0, np.where(u >= 0.95, 1.0, 0.0)).astype(np.float32)
                dones = (rng.random((done.size, T)) < 0.02).astype(np.uint8)
                dones[np.flatnonzero(ended[hand]), lens[ended[hand]] - 1] = 1
                # the bootstrap is the value of the newest state the agent knows
                sched.submit_segment_many(done, base + done.astype(np.uint64) * T * fb, lens, acts[done], rewards, dones,
                                          value[hand], seg_ver[done])
                seg_len[done] = 0
    sched.drain()
    wall = time.perf_counter() - t0
    st = sched.stats()
    out = {"net": net_kind, "agents": n_agents, "think_us": think_us, "dynamic": dynamic, "seconds": round(wall, 3),
           "pps": round(st["predictions"] / wall, 1), "tps_frames": round(st["trained_frames"] / wall, 1),
           # the second half of the run on its own: what the adjustment has arrived at, without the climb
           "tps_frames_second_half": round((st["trained_frames"] - half[1]) / (wall - half[0]), 1) if half else None,
           "mean_predict_batch": round(st["predictions"] / max(1, st["predict_batches"]), 2),
           "mean_train_batch_frames": round(st["trained_frames"] / max(1, st["train_batches"]), 1),
           "mean_train_queue": round(st["sum_train_queue"] / max(1, st["ticks"]), 2),
           "predict_cap": st["predict_cap"], "train_cap": st["train_cap"],
           "trials_accepted": st["trials_accepted"], "trials_rejected": st["trials_rejected"],
           "windows": st["windows"], "last_change_window": st["last_change_window"],
           "seconds_to_last_change": round(wall * st["last_change_window"] / st["windows"], 3) if st["windows"] else None,
           "train_min": train_min, "episode_end_prob": episode_end_prob, "updates": st["train_batches"],
           "short_segments": st["short_segments"],
           "mean_policy_lag_updates": round(st["lag_sum"] / max(1, st["lag_count"]), 3), "max_policy_lag_updates": st["lag_max"],
           "host_us_per_tick": round(wall / max(1, ticks) * 1e6, 1)}
    if dynamic and half:
        # time to converge: the end of the first window whose reading reached 90 % of what the second half averages
        target = 0.9 * out["tps_frames_second_half"]
        out["seconds_to_90pct_of_second_half"] = next((w[6] for w in windows_seen if w[1] >= target), None)
    if trace:
        out["window_trace"] = windows_seen
    sched.close()
    net.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--net", choices=("small", "large"), default="small")
    ap.add_argument("--seconds", type=float, default=1.5)
    ap.add_argument("--think-us", type=float, nargs="*", default=[0.0, 200.0, 2000.0, 20000.0])
    ap.add_argument("--agents", type=int, default=256)
    ap.add_argument("--episode-end-prob", type=float, default=0.0)
    ap.add_argument("--min-batch-sweep", action="store_true")
    args = ap.parse_args()
    if args.min_batch_sweep:
        rows = [run_mixed(args.net, n_agents=args.agents, think_us=th, seconds=args.seconds, dynamic=False,
                          train_min=m, train_cap=max(1280, m), episode_end_prob=args.episode_end_prob)
                for th in args.think_us[:2] for m in (5, 10, 20, 40, 80, 160, 320)]
        print(json.dumps({"metric": "minimum training batch sweep (Sec. 5.3), synthetic agents, one GPU, two streams",
                          "net": args.net, "data": "synthetic", "runs": rows}))
        return 0
    rows = []
    for th in args.think_us:
        rows.append(run_mixed(args.net, n_agents=args.agents, think_us=th, seconds=args.seconds, dynamic=True,
                              episode_end_prob=args.episode_end_prob))
    rows.append(run_mixed(args.net, n_agents=args.agents, think_us=0.0, seconds=args.seconds, dynamic=False,
                          episode_end_prob=args.episode_end_prob))
    print(json.dumps({"metric": "mixed load, synthetic agents, one GPU, two streams", "net": args.net,
                      "data": "synthetic", "runs": rows}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
