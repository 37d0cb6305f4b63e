"""Seeded synthetic inputs for the GA3C hot path.

These stand in for Atari 2600 frames, actions, rewards and episode ends (the
paper's workload, Sec. 5: OpenAI Gym Atari games with action repeat 4), which
need an emulator that is not available.  The module holds no arithmetic of
the method: it only draws inputs.  Both the CPU oracle's tests and the HIP
library's tests feed on it, so that the two sides see identical data.

All draws come from ``numpy.random.Generator(PCG64(seed))``.
"""
from __future__ import annotations

from typing import Dict, Sequence, Tuple

import numpy as np

BASE_SEED = 1611


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def uniform_frames(seed: int, shape: Sequence[int]) -> np.ndarray:
    """iid uniform{0..255} bytes (the small parity configuration)."""
    return rng(seed).integers(0, 256, size=tuple(shape), dtype=np.uint8)


def rectangle_frames(seed: int, n: int, c: int = 4, h: int = 84, w: int = 84) -> np.ndarray:
    """Game-like stacks: a zero background, 3-12 axis-aligned rectangles of
    uniform intensity drawn in every plane with a small per-plane shift (as
    consecutive video frames would show), then 2 % salt noise per plane."""
    g = rng(seed)
    out = np.zeros((n, c, h, w), dtype=np.uint8)
    for b in range(n):
        k = int(g.integers(3, 13))
        for _ in range(k):
            y0 = int(g.integers(0, h - 2)); x0 = int(g.integers(0, w - 2))
            hh = int(g.integers(2, h - y0 + 1)); ww = int(g.integers(2, w - x0 + 1))
            hh = min(hh, 2 + int(g.integers(0, 30))); ww = min(ww, 2 + int(g.integers(0, 30)))
            val = int(g.integers(1, 256))
            for p in range(c):
                dy, dx = (int(v) for v in g.integers(-2, 3, size=2))
                ya, yb = np.clip([y0 + dy, y0 + dy + hh], 0, h)
                xa, xb = np.clip([x0 + dx, x0 + dx + ww], 0, w)
                out[b, p, ya:yb, xa:xb] = val
        salt = g.random((c, h, w)) < 0.02
        out[b][salt] = 255
    return out


def rectangle_frames_tiled(seed: int, n: int, base: int = 256, **kw) -> np.ndarray:
    """n rectangle frames made by drawing ``base`` distinct ones and repeating
    them with a seeded permutation (drawing tens of thousands one by one in
    Python would dominate a benchmark's set-up time)."""
    if n <= base:
        return rectangle_frames(seed, n, **kw)
    pool = rectangle_frames(seed, base, **kw)
    idx = rng(seed + 7).integers(0, base, size=n)
    return pool[idx]


def trajectories(seed: int, n_agents: int, t_max: int, n_actions: int) -> Dict[str, np.ndarray]:
    """actions uniform in [0,A); rewards in {-1,0,+1} w.p. .05/.90/.05;
    dones Bernoulli(0.02)."""
    g = rng(seed)
    actions = g.integers(0, n_actions, size=(n_agents, t_max), dtype=np.int32)
    u = g.random((n_agents, t_max))
    rewards = np.where(u < 0.05, -1.0, np.where(u >= 0.95, 1.0, 0.0)).astype(np.float32)
    dones = (g.random((n_agents, t_max)) < 0.02).astype(np.uint8)
    return {"actions": actions, "rewards": rewards, "dones": dones}


def ragged_segments(seed: int, n_segments: int, t_max: int, n_actions: int, p_short: float = 0.3) -> Dict[str, np.ndarray]:
    """Segments as the agents of Sec. 4.1 hand them in: t_max experiences, or fewer when the episode ended (then the
    last step is terminal).  A fraction p_short of the segments is short, with a length uniform in [1, t_max).
    Returns flat arrays over all frames plus seg_start [n_segments + 1] (int32) and the lengths."""
    g = rng(seed)
    short = g.random(n_segments) < p_short
    lengths = np.where(short & (t_max > 1), g.integers(1, max(t_max, 2), size=n_segments), t_max).astype(np.int32)
    seg_start = np.zeros(n_segments + 1, dtype=np.int32)
    np.cumsum(lengths, out=seg_start[1:])
    F = int(seg_start[-1])
    actions = g.integers(0, n_actions, size=F, dtype=np.int32)
    u = g.random(F)
    rewards = np.where(u < 0.05, -1.0, np.where(u >= 0.95, 1.0, 0.0)).astype(np.float32)
    dones = np.zeros(F, dtype=np.uint8)
    ends = seg_start[1:][lengths < t_max] - 1
    dones[ends] = 1
    return {"actions": actions, "rewards": rewards, "dones": dones, "seg_start": seg_start, "lengths": lengths}


def uniforms(seed: int, n: int) -> np.ndarray:
    """float32 uniforms in [0,1) handed to the sampler of both sides."""
    return rng(seed).random(n, dtype=np.float32)


def he_normal_theta(seed: int, tensors: Dict[str, Tuple[int, Tuple[int, ...]]], total: int) -> np.ndarray:
    """Flat float32 parameter vector: weights N(0, 2/fan_in), biases zero.
    ``tensors`` maps name -> (offset, shape); names ending in '.b' are biases."""
    g = rng(seed)
    theta = np.zeros(total, dtype=np.float32)
    for name, (off, shape) in tensors.items():
        if name.endswith(".b"):
            continue
        fan_in = int(np.prod(shape[1:]))
        n = int(np.prod(shape))
        theta[off:off + n] = (g.standard_normal(n) * np.sqrt(2.0 / fan_in)).astype(np.float32)
    return theta


def perturbed_theta(seed: int, tensors, total: int, bias_scale: float = 0.05) -> np.ndarray:
    """He-normal weights plus small non-zero biases, so that tests exercise
    the bias terms too."""
    theta = he_normal_theta(seed, tensors, total)
    g = rng(seed + 1)
    for name, (off, shape) in tensors.items():
        if name.endswith(".b"):
            n = int(np.prod(shape))
            theta[off:off + n] = (g.standard_normal(n) * bias_scale).astype(np.float32)
    return theta
