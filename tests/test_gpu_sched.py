"""Queue-driven batching (paper Sec. 4.1, 4.3) on the GPU: what goes through
the scheduler's two streams must equal the same calls made directly."""
import numpy as np
import pytest

import ga3c_synth as synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    import paper_1611_06256_amd as g
    assert torch.cuda.is_available()
    return g


def setup(G, n_agents, T, seed, max_pred=64, max_train=320):
    import torch
    desc = G.SMALL_NET(6)
    nets = [G.Ga3c(desc, max_pred, max_train) for _ in range(2)]      # [0] behind the scheduler, [1] called directly
    theta = synth.perturbed_theta(seed, nets[0].offsets(), nets[0].n_params)
    for n in nets:
        n.params_set(torch.from_numpy(theta).cuda(), 0)
    frames = torch.from_numpy(synth.rectangle_frames(seed + 1, n_agents * T).reshape(n_agents, T, 4, 84, 84)).cuda()
    tr = synth.trajectories(seed + 2, n_agents, T, 6)
    u = synth.uniforms(seed + 3, n_agents * T).reshape(n_agents, T)
    torch.cuda.synchronize()
    return nets, frames, tr, u


def direct_predict(net, fr, u):
    import torch
    B = fr.shape[0]
    v = torch.empty(B, device="cuda"); p = torch.empty(B, 6, device="cuda")
    a = torch.empty(B, dtype=torch.int32, device="cuda")
    net.predict(fr, uniforms=torch.from_numpy(u).cuda(), values=v, probs=p, actions=a)
    torch.cuda.synchronize()
    return v.cpu().numpy(), p.cpu().numpy(), a.cpu().numpy()


def test_predictions_and_updates_match_direct_calls(G):
    import torch
    N, T = 24, 5
    (ns, nd), frames, tr, u = setup(G, N, T, 2024)
    hp = G.HParams(lr=1e-3, clip_norm=40.0)
    sched = G.Scheduler(ns, hp, t_max=T, predict_cap=16, train_min=40, train_cap=40)    # 8 agents per update
    got = {}
    step = 0
    # tick k: every agent asks for a prediction on its frame k; from tick 1 on, 8 agents hand in their trajectory
    for k in range(T):
        for a in range(N):
            sched.submit_predict(a, frames[a, k], float(u[a, k]))
        if k >= 1 and (k - 1) * 8 < N:
            for a in range((k - 1) * 8, min(k * 8, N)):
                sched.submit_trajectory(a, frames[a], tr["actions"][a], tr["rewards"][a], tr["dones"][a], 0.25 * a)
        # the prediction queue holds 24 requests, the cap is 16: a full batch goes out at once, the other 8 (less
        # than a full batch) when no earlier batch is in flight any more
        np_total, nt_total = 0, 0
        while True:
            p, t = sched.tick()
            np_total += p; nt_total += t
            if p == 0 and t == 0 and sched.stats()["predict_queue"] == 0:
                break
        assert np_total == N
        assert nt_total == (40 if k >= 1 and (k - 1) * 8 < N else 0)
        sched.drain()
        res = sched.poll()
        assert len(res) == N and sorted(r[0] for r in res) == list(range(N))
        # The same on the direct context, in the order the scheduler enqueued it: the first tick
        # sends 16 predictions and then the update, the second tick the other 8 predictions, which
        # therefore see the updated parameters (a prediction reads the last update enqueued before it).
        def check(agents):
            v, p_, a_ = direct_predict(nd, frames[agents, k].contiguous(), u[agents, k].copy())
            cdf = np.cumsum(p_.astype(np.float64), 1)
            by_agent = {r[0]: r for r in res}
            for i, agent in enumerate(agents):
                _, action, value = by_agent[agent]
                assert abs(value - v[i]) <= 1e-5 * max(1.0, abs(v[i])), (k, agent)
                if (np.abs(cdf[i] - u[agent, k]) > 1e-5).all():
                    assert action == a_[i], (k, agent)
        check(list(range(16)))
        if k >= 1 and (k - 1) * 8 < N:
            sl = slice((k - 1) * 8, k * 8)
            boot = torch.from_numpy((0.25 * np.arange(N)[sl]).astype(np.float32)).cuda()
            nd.train_step(frames[sl].contiguous(), torch.from_numpy(tr["actions"][sl]).cuda(),
                          torch.from_numpy(tr["rewards"][sl]).cuda(), torch.from_numpy(tr["dones"][sl]).cuda(), boot, hp)
            torch.cuda.synchronize()
            step += 1
        check(list(range(16, N)))
    assert step == 3
    # updates are deterministic: the parameters behind the scheduler equal the direct ones bit for bit
    np.testing.assert_array_equal(ns.params_get(0).cpu().numpy(), nd.params_get(0).cpu().numpy())
    np.testing.assert_array_equal(ns.params_get(1).cpu().numpy(), nd.params_get(1).cpu().numpy())
    st = sched.stats()
    assert st["predictions"] == N * T and st["trained_frames"] == 120 and st["train_batches"] == 3
    assert st["predict_queue"] == 0 and st["train_queue"] == 0
    sched.close(); ns.close(); nd.close()


def test_minimum_training_batch_and_caps(G):
    N, T = 12, 5
    (ns, nd), frames, tr, u = setup(G, N, T, 77)
    sched = G.Scheduler(ns, G.HParams(lr=0.0), t_max=T, predict_cap=4, train_min=40, train_cap=50)
    for a in range(7):                          # 35 frames: below the minimum, nothing is trained
        sched.submit_trajectory(a, frames[a], tr["actions"][a], tr["rewards"][a], tr["dones"][a], 0.0)
    assert sched.tick() == (0, 0)
    sched.submit_trajectory(7, frames[7], tr["actions"][7], tr["rewards"][7], tr["dones"][7], 0.0)
    assert sched.tick() == (0, 40)              # the minimum is reached: all 8 go (the cap would allow 10)
    for a in range(N):
        sched.submit_trajectory(a, frames[a], tr["actions"][a], tr["rewards"][a], tr["dones"][a], 0.0)
    assert sched.tick() == (0, 50)              # 12 wait, the cap lets 10 go
    assert sched.tick() == (0, 0)               # 2 are left: below the minimum again
    for a in range(N):
        sched.submit_predict(a, frames[a, 0], 0.5)
    assert [sched.tick()[0] for _ in range(4)] == [4, 4, 4, 0]
    sched.drain()
    assert len(sched.poll()) == N
    with pytest.raises(G.Ga3cError):
        sched.submit_trajectory(0, frames[0], np.full(5, 9, np.int32), tr["rewards"][0], tr["dones"][0], 0.0)
    with pytest.raises(G.Ga3cError):
        G.Scheduler(ns, G.HParams(), t_max=T, predict_cap=65)          # above the context's capacity
    sched.close(); ns.close(); nd.close()


def test_dynamic_adjustment_runs_within_bounds(G):
    N, T = 32, 5
    (ns, nd), frames, tr, u = setup(G, N, T, 99)
    sched = G.Scheduler(ns, G.HParams(lr=1e-4), t_max=T, predict_cap=8, train_min=40, train_cap=80, adjust_period=4,
                        predict_cap_lo=2, predict_cap_hi=64, train_cap_lo=40, train_cap_hi=160, train_cap_step=40, seed=3)
    polled, best = 0, 0.0
    for it in range(40):
        for a in range(N):
            sched.submit_predict(a, frames[a, it % T], float(u[a, it % T]))
            if it % 2 == 0:
                sched.submit_trajectory(a, frames[a], tr["actions"][a], tr["rewards"][a], tr["dones"][a], 0.0)
        for _ in range(3):
            sched.tick()
        polled += len(sched.poll())
        st = sched.stats()
        assert 2 <= st["predict_cap"] <= 64 and 40 <= st["train_cap"] <= 160
        best = max(best, st["last_window_frames_per_s"])
    while sched.stats()["predict_queue"] > 0 or sched.stats()["train_queue"] * T >= 40:
        sched.tick()
    sched.drain()
    polled += len(sched.poll())
    st = sched.stats()
    assert polled == st["predictions"] == 40 * N
    assert st["windows"] >= 25 and st["trials_accepted"] + st["trials_rejected"] >= 10     # a rejected trial costs a second window
    assert best > 0
    assert np.isfinite(ns.params_get(0).cpu().numpy()).all()
    sched.close(); ns.close(); nd.close()


def test_short_segments_and_policy_lag(G):
    # Sec. 4.1: an agent hands in fewer than t_max experiences when its episode ends; Sec. 4.2: the policy that acted
    # may be older than the parameters its experiences update.  Segments of mixed length go through the scheduler in
    # whole-segment batches under a frame cap; the parameters must equal those of the same ragged updates made
    # directly, and the lag statistics must count the updates issued between a prediction and its segment's update.
    import torch
    N, T = 12, 5
    (ns, nd), frames, tr, u = setup(G, N, T, 4242)
    seg = synth.ragged_segments(4243, N, T, 6, p_short=0.5)
    lens, start = seg["lengths"], seg["seg_start"]
    assert (lens < T).any() and (lens == T).any()
    hp = G.HParams(lr=1e-3, clip_norm=40.0)
    sched = G.Scheduler(ns, hp, t_max=T, predict_cap=64, train_min=1, train_cap=30)
    for a in range(N):
        sched.submit_predict(a, frames[a, 0], float(u[a, 0]))
    assert sched.tick() == (N, 0)
    sched.drain()
    ag, _, _, ver = sched.poll_arrays(with_version=True)
    assert sorted(ag) == list(range(N)) and (ver == 0).all()
    boot = (0.1 * np.arange(N)).astype(np.float32)
    for a in range(N):
        sl = slice(start[a], start[a + 1])
        sched.submit_segment(a, frames[a, :lens[a]], seg["actions"][sl], seg["rewards"][sl], seg["dones"][sl],
                             float(boot[a]), policy_version=int(ver[list(ag).index(a)]))
    with pytest.raises(G.Ga3cError):      # longer than t_max
        sched.submit_segment(0, frames[0], np.zeros(6, np.int32), np.zeros(6, np.float32), np.zeros(6, np.uint8), 0.0)
    # expected batches: whole segments, oldest first, while the frame count stays within the cap
    batches, cur, cnt = [], [], 0
    for a in range(N):
        if cur and cnt + lens[a] > 30:
            batches.append(cur); cur, cnt = [], 0
        cur.append(a); cnt += int(lens[a])
    batches.append(cur)
    assert len(batches) >= 2
    for k, b in enumerate(batches):
        nfr = int(sum(lens[a] for a in b))
        # a tick sends its prediction batch before its update: this prediction reads the parameters after k updates
        sched.submit_predict(b[0], frames[b[0], 1], 0.5)
        assert sched.tick() == (1, nfr)
        sched.drain()
        _, _, _, v = sched.poll_arrays(with_version=True)
        assert list(v) == [k]
        fr = torch.cat([frames[a, :lens[a]] for a in b]).contiguous()
        cat = lambda key: torch.from_numpy(np.concatenate([seg[key][start[a]:start[a + 1]] for a in b])).cuda()
        st_ = np.concatenate([[0], np.cumsum([lens[a] for a in b])]).astype(np.int32)
        if all(lens[a] == T for a in b):
            nd.train_step(fr.reshape(len(b), T, 4, 84, 84), cat("actions").reshape(len(b), T), cat("rewards").reshape(len(b), T),
                          cat("dones").reshape(len(b), T), torch.from_numpy(boot[b]).cuda(), hp)
        else:
            nd.train_step_ragged(fr, cat("actions"), cat("rewards"), cat("dones"), torch.from_numpy(st_).cuda(),
                                 torch.from_numpy(boot[b]).cuda(), hp)
        torch.cuda.synchronize()
    assert sched.tick() == (0, 0)
    np.testing.assert_array_equal(ns.params_get(0).cpu().numpy(), nd.params_get(0).cpu().numpy())
    np.testing.assert_array_equal(ns.params_get(1).cpu().numpy(), nd.params_get(1).cpu().numpy())
    st = sched.stats()
    assert st["train_batches"] == len(batches) and st["trained_frames"] == int(lens.sum())
    assert st["short_segments"] == int((lens < T).sum())
    # every segment was generated by version 0; batch k is update number k, so its segments lag by k updates
    assert st["lag_count"] == N and st["lag_max"] == len(batches) - 1
    assert st["lag_sum"] == sum(k * len(b) for k, b in enumerate(batches))
    sched.close(); ns.close(); nd.close()


def test_scheduler_host_code_is_clean_under_the_address_and_undefined_behaviour_sanitizers():
    # paper_1611_06256_amd/sched_sanitized (built beforehand by build.py / the entry point's build()) is the whole
    # library with its HOST code under ASan and UBSan plus tests/sched_sanitizer_driver.cpp: a closed loop of agents with
    # short segments, policy versions, the adjustment, the many-at-once calls and the error paths.  Any finding in the
    # queues, slot rings or staging buffers aborts it with a non-zero status.
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_1611_06256_amd", "sched_sanitized")
    if not os.path.exists(exe):
        pytest.skip("paper_1611_06256_amd/sched_sanitized is not built (python -m paper_1611_06256_amd.build sched_sanitized, or the entry point's build())")
    # (verify_asan_link_order=0: the environment may preload a library of its own; leaks are not looked for, the GPU
    # runtime keeps its own allocations until exit)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "0 problems" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
