"""The dynamic-adjustment rule (paper Sec. 4.3: change one knob at random by
one step, keep the change unless throughput dropped) on a synthetic
throughput model; host code only."""
import math

import pytest

import paper_1611_06256_amd as g


def model(p, t, p_star=64, t_star=640):
    """Concave in log2(p) and in t, maximal at (p_star, t_star)."""
    return 1e6 - 4e4 * (math.log2(p) - math.log2(p_star)) ** 2 - 0.5 * (t - t_star) ** 2


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("start", [(1, 40), (256, 1280), (8, 1000)])
def test_hill_climb_converges_and_stays_in_bounds(seed, start):
    tun = g.Tuner(1, 256, start[0], 40, 1280, 40, start[1], seed)
    p, t = start
    seen = []
    for _ in range(400):
        p, t = tun.report(model(p, t))
        assert 1 <= p <= 256 and 40 <= t <= 1280
        assert p & (p - 1) == 0 and (t - 40) % 40 == 0       # stays on the two ladders
        seen.append((p, t))
    st = tun.state()
    assert st["predict_cap"] in (32, 64, 128)                # argmax +- one step
    assert abs(st["train_cap"] - 640) <= 40
    assert st["accepted"] > 0 and st["rejected"] > 0
    # every proposal differs from the kept configuration in exactly one knob by one step
    kp, kt = st["predict_cap"], st["train_cap"]
    assert (p == kp) != (t == kt) or (p == kp and t == kt)


def test_same_seed_same_sequence():
    def run(seed):
        tun = g.Tuner(1, 256, 16, 40, 1280, 40, 200, seed)
        p, t, out = 16, 200, []
        for _ in range(100):
            p, t = tun.report(model(p, t))
            out.append((p, t))
        return out
    assert run(7) == run(7)
    assert run(7) != run(8)


def test_a_worse_trial_is_undone():
    tun = g.Tuner(1, 256, 64, 640, 640, 40, 640, 5)          # only the prediction cap can move
    p, t = tun.report(100.0)                                  # reference for (64, 640); first trial proposed
    assert t == 640 and p in (32, 128)
    p2, _ = tun.report(50.0)                                  # the trial was worse
    st = tun.state()
    assert st["predict_cap"] == 64 and st["rejected"] == 1 and st["accepted"] == 0
    assert p2 in (32, 128)
    tun.report(150.0)                                         # better: kept
    st = tun.state()
    assert st["predict_cap"] == p2 and st["accepted"] == 1


def test_bad_bounds_are_refused():
    with pytest.raises(g.Ga3cError):
        g.Tuner(4, 2, 3, 40, 1280, 40, 40, 0)
    with pytest.raises(g.Ga3cError):
        g.Tuner(1, 256, 512, 40, 1280, 40, 40, 0)
