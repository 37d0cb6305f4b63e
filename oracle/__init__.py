"""ctypes front end of the fp64 CPU oracle (``ga3c_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  Nothing on the product path
may import it, and it imports nothing from the HIP package.

Every function marshals numpy arrays into the C routine of the same name and
does no arithmetic of its own (apart from slicing the flat parameter vector
into named views, which is bookkeeping).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ga3c_oracle.c")
_LIB = os.path.join(_HERE, "libga3c_oracle.so")
MAX_CONV = 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (C99, -O2, OpenMP).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Net(C.Structure):
    _fields_ = [
        ("in_c", C.c_int), ("in_h", C.c_int), ("in_w", C.c_int),
        ("n_conv", C.c_int),
        ("oc", C.c_int * MAX_CONV), ("k", C.c_int * MAX_CONV), ("stride", C.c_int * MAX_CONV),
        ("fc_units", C.c_int), ("n_actions", C.c_int), ("math", C.c_int),
    ]


class _HParams(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("gamma", "beta", "value_coef", "log_eps", "lr", "rms_decay", "rms_eps", "clip_norm")]


class _Stats(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("policy_loss", "value_loss", "entropy", "grad_norm", "clip_scale")]


@dataclass
class Net:
    """Network description: input C,H,W; conv layers (oc, k, stride); fc width; actions."""
    in_c: int = 4
    in_h: int = 84
    in_w: int = 84
    conv: Sequence[Tuple[int, int, int]] = ((16, 8, 4), (32, 4, 2))
    fc_units: int = 256
    n_actions: int = 6
    math: int = 0        # 1: operands of every contraction rounded to bfloat16

    def c(self) -> _Net:
        n = _Net()
        n.in_c, n.in_h, n.in_w = self.in_c, self.in_h, self.in_w
        n.n_conv = len(self.conv)
        for i, (oc, k, s) in enumerate(self.conv):
            n.oc[i], n.k[i], n.stride[i] = oc, k, s
        n.fc_units, n.n_actions = self.fc_units, self.n_actions
        n.math = self.math
        return n


@dataclass
class HParams:
    gamma: float = 0.99
    beta: float = 0.01
    value_coef: float = 1.0
    log_eps: float = 0.0
    lr: float = 3e-4
    rms_decay: float = 0.99
    rms_eps: float = 0.1
    clip_norm: float = 0.0

    def c(self) -> _HParams:
        return _HParams(self.gamma, self.beta, self.value_coef, self.log_eps,
                        self.lr, self.rms_decay, self.rms_eps, self.clip_norm)


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_param_count.restype = C.c_int64
        _lib.orc_acts_per_frame.restype = C.c_int64
        _lib.orc_grad_norm.restype = C.c_double
        _lib.orc_clip_scale.restype = C.c_double
        _lib.orc_clip_scale.argtypes = [C.c_double, C.c_double]
        _lib.orc_bf16_round.restype = C.c_double
        _lib.orc_bf16_round.argtypes = [C.c_double]
        _lib.orc_sample.argtypes = [C.c_void_p, C.c_int, C.c_double]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def param_count(net: Net) -> int:
    return int(lib().orc_param_count(C.byref(net.c())))


def acts_per_frame(net: Net) -> int:
    return int(lib().orc_acts_per_frame(C.byref(net.c())))


def offsets(net: Net) -> Dict[str, Tuple[int, Tuple[int, ...]]]:
    """Name -> (offset, shape) of every tensor in the flat parameter vector."""
    off = (C.c_int64 * (2 * MAX_CONV + 8))()
    n = lib().orc_offsets(C.byref(net.c()), off)
    o = [int(off[i]) for i in range(n)]
    out: Dict[str, Tuple[int, Tuple[int, ...]]] = {}
    c, h, w = net.in_c, net.in_h, net.in_w
    for l, (oc, k, s) in enumerate(net.conv):
        out[f"conv{l + 1}.W"] = (o[2 * l], (oc, c, k, k))
        out[f"conv{l + 1}.b"] = (o[2 * l + 1], (oc,))
        c, h, w = oc, (h - k) // s + 1, (w - k) // s + 1
    nb = 2 * len(net.conv)
    out["fc.W"] = (o[nb], (net.fc_units, c * h * w))
    out["fc.b"] = (o[nb + 1], (net.fc_units,))
    out["policy.W"] = (o[nb + 2], (net.n_actions, net.fc_units))
    out["policy.b"] = (o[nb + 3], (net.n_actions,))
    out["value.W"] = (o[nb + 4], (1, net.fc_units))
    out["value.b"] = (o[nb + 5], (1,))
    return out


def views(net: Net, flat: np.ndarray) -> Dict[str, np.ndarray]:
    """Named views into a flat parameter-sized vector (no copy)."""
    return {name: flat[o:o + int(np.prod(shape))].reshape(shape)
            for name, (o, shape) in offsets(net).items()}


def forward(net: Net, theta, frames: np.ndarray, want_acts: bool = False):
    """frames u8 [B,C,H,W] -> dict(logits [B,A], values [B], probs [B,A], acts [B,apf]?)."""
    theta = _f64(theta)
    frames = np.ascontiguousarray(frames, dtype=np.uint8)
    B, A = frames.shape[0], net.n_actions
    logits = np.zeros((B, A)); values = np.zeros(B); probs = np.zeros((B, A))
    acts = np.zeros((B, acts_per_frame(net))) if want_acts else None
    rc = lib().orc_forward(C.byref(net.c()), _p(theta), _p(frames), C.c_int(B),
                           _p(acts), _p(logits), _p(values), _p(probs))
    if rc != 0:
        raise MemoryError("orc_forward")
    out = {"logits": logits, "values": values, "probs": probs}
    if want_acts:
        out["acts"] = acts
    return out


def sample(probs: np.ndarray, uniforms: np.ndarray) -> np.ndarray:
    probs = _f64(probs)
    A = probs.shape[1]
    return np.array([lib().orc_sample(_p(probs[i]), A, float(uniforms[i]))
                     for i in range(probs.shape[0])], dtype=np.int32)


def returns(rewards, dones, bootstrap, gamma: float) -> np.ndarray:
    rewards = _f64(rewards)
    dones = np.ascontiguousarray(dones, dtype=np.uint8)
    N, T = rewards.shape
    boot = None if bootstrap is None else _f64(bootstrap)
    R = np.zeros((N, T))
    lib().orc_returns(_p(rewards), _p(dones), _p(boot), C.c_int(N), C.c_int(T),
                      C.c_double(gamma), _p(R))
    return R


def returns_ragged(rewards, dones, seg_start, bootstrap, gamma: float) -> np.ndarray:
    """Returns of segments of unequal length laid end to end: segment n is entries seg_start[n] .. seg_start[n+1]-1."""
    rewards = _f64(rewards).reshape(-1)
    dones = np.ascontiguousarray(dones, dtype=np.uint8).reshape(-1)
    seg = np.ascontiguousarray(seg_start, dtype=np.int32)
    N = seg.size - 1
    if N < 0 or (N >= 0 and (seg[0] != 0 or seg[-1] != rewards.size or np.any(np.diff(seg) < 0))):
        raise ValueError("seg_start must rise from 0 to the number of frames")
    boot = None if bootstrap is None else _f64(bootstrap)
    R = np.zeros(rewards.size)
    lib().orc_returns_ragged(_p(rewards), _p(dones), _p(seg), _p(boot), C.c_int(N), C.c_double(gamma), _p(R))
    return R


def loss_grad(logits, values, actions, R, beta: float, value_coef: float, log_eps: float):
    logits = _f64(logits); values = _f64(values); R = _f64(R).reshape(-1)
    actions = np.ascontiguousarray(actions, dtype=np.int32).reshape(-1)
    B, A = logits.shape
    dZ = np.zeros((B, A)); dV = np.zeros(B); sums = np.zeros(3)
    lib().orc_loss_grad(_p(logits), _p(values), _p(actions), _p(R), C.c_int(B), C.c_int(A),
                        C.c_double(beta), C.c_double(value_coef), C.c_double(log_eps),
                        _p(dZ), _p(dV), _p(sums))
    return dZ, dV, {"policy_loss": sums[0], "value_loss": sums[1], "entropy": sums[2]}


def backward(net: Net, theta, acts, dZ, dV) -> np.ndarray:
    theta = _f64(theta); acts = _f64(acts); dZ = _f64(dZ); dV = _f64(dV)
    grad = np.zeros(param_count(net))
    rc = lib().orc_backward(C.byref(net.c()), _p(theta), _p(acts), C.c_int(acts.shape[0]),
                            _p(dZ), _p(dV), _p(grad))
    if rc != 0:
        raise MemoryError("orc_backward")
    return grad


def conv_layer_forward(x, W, bias, stride: int, math: int = 0, xs: float = 1.0) -> np.ndarray:
    """One convolution layer + ReLU on x [B,C,H,W] (the stored input; xs = 255 for the first layer of math = 1)."""
    x = _f64(x); W = _f64(W); bias = _f64(bias)
    B, Cc, H, Wd = x.shape
    OC, _, K, _ = W.shape
    y = np.zeros((B, OC, (H - K) // stride + 1, (Wd - K) // stride + 1))
    lib().orc_conv_layer_forward(C.c_int(B), _p(x), C.c_int(Cc), C.c_int(H), C.c_int(Wd), _p(W), _p(bias), C.c_int(OC),
                                 C.c_int(K), C.c_int(stride), C.c_int(math), C.c_double(xs), _p(y))
    return y


def conv_layer_backward(x, W, stride: int, y, dy, math: int = 0, xs: float = 1.0, want_dx: bool = True):
    """Backward of one convolution layer: (gW, gb, dx).  dy is taken before the layer's ReLU mask (from y)."""
    x = _f64(x); W = _f64(W); y = _f64(y); dy = _f64(dy)
    B, Cc, H, Wd = x.shape
    OC, _, K, _ = W.shape
    gW = np.zeros(W.shape); gb = np.zeros(OC); dx = np.zeros(x.shape) if want_dx else None
    rc = lib().orc_conv_layer_backward(C.c_int(B), _p(x), C.c_int(Cc), C.c_int(H), C.c_int(Wd), _p(W), C.c_int(OC),
                                       C.c_int(K), C.c_int(stride), _p(y), _p(dy), C.c_int(math), C.c_double(xs),
                                       _p(gW), _p(gb), _p(dx))
    if rc != 0:
        raise MemoryError("orc_conv_layer_backward")
    return gW, gb, dx


def dense_forward(x, W, bias, relu: bool, math: int = 0) -> np.ndarray:
    """x [B,I], W [O,I], bias [O] -> [B,O]."""
    x = _f64(x); W = _f64(W); bias = _f64(bias)
    B, I = x.shape
    O = W.shape[0]
    y = np.zeros((B, O))
    lib().orc_dense_forward(C.c_int(B), _p(x), C.c_int64(I), _p(W), _p(bias), C.c_int(O), C.c_int(int(relu)),
                            C.c_int(math), _p(y))
    return y


def dense_backward(x, W, dy, math: int = 0, want_dx: bool = True):
    """Backward of a fully connected layer: (gW, gb, dx) for dy [B,O] = dL/d(pre-activation)."""
    x = _f64(x); W = _f64(W); dy = _f64(dy)
    B, I = x.shape
    O = W.shape[0]
    gW = np.zeros((O, I)); gb = np.zeros(O); dx = np.zeros((B, I)) if want_dx else None
    rc = lib().orc_dense_backward(C.c_int(B), _p(x), C.c_int64(I), _p(W), C.c_int(O), _p(dy), C.c_int(math),
                                  _p(gW), _p(gb), _p(dx))
    if rc != 0:
        raise MemoryError("orc_dense_backward")
    return gW, gb, dx


def bf16_round(values) -> np.ndarray:
    """Nearest bfloat16, ties to even, of every element (the rounding math = 1 applies to operands)."""
    L = lib()
    v = np.asarray(values, dtype=np.float64)
    return np.array([L.orc_bf16_round(float(x)) for x in v.reshape(-1)], dtype=np.float64).reshape(v.shape)


def grad_norm(grad) -> float:
    grad = _f64(grad)
    return float(lib().orc_grad_norm(_p(grad), C.c_int64(grad.size)))


def clip_scale(norm: float, c: float) -> float:
    return float(lib().orc_clip_scale(norm, c))


def rmsprop(theta, g, grad, scale: float, lr: float, alpha: float, eps: float):
    """Returns updated copies (theta', g')."""
    theta = _f64(theta).copy(); g = _f64(g).copy(); grad = _f64(grad)
    lib().orc_rmsprop(_p(theta), _p(g), _p(grad), C.c_int64(theta.size), C.c_double(scale),
                      C.c_double(lr), C.c_double(alpha), C.c_double(eps))
    return theta, g


def train_step(net: Net, theta, g, frames, actions, rewards, dones, bootstrap, hp: HParams):
    """One whole update.  frames u8 [N,T,C,H,W].  Returns a dict with updated
    theta, g, the unclipped summed gradient, stats and the intermediates."""
    theta = _f64(theta).copy(); g = _f64(g).copy()
    frames = np.ascontiguousarray(frames, dtype=np.uint8)
    N, T = frames.shape[0], frames.shape[1]
    actions = np.ascontiguousarray(actions, dtype=np.int32)
    rewards = _f64(rewards)
    dones = np.ascontiguousarray(dones, dtype=np.uint8)
    boot = None if bootstrap is None else _f64(bootstrap)
    A, B = net.n_actions, N * T
    grad = np.zeros(theta.size)
    R = np.zeros((N, T)); dZ = np.zeros((B, A)); dV = np.zeros(B)
    logits = np.zeros((B, A)); values = np.zeros(B)
    st = _Stats(); hpc = hp.c()
    rc = lib().orc_train_step(C.byref(net.c()), _p(theta), _p(g), _p(grad), _p(frames), _p(actions),
                              _p(rewards), _p(dones), _p(boot), C.c_int(N), C.c_int(T),
                              C.byref(hpc), C.byref(st), _p(R), _p(dZ), _p(dV), _p(logits), _p(values))
    if rc != 0:
        raise MemoryError("orc_train_step")
    return {"theta": theta, "g": g, "grad": grad, "R": R, "dZ": dZ, "dV": dV,
            "logits": logits, "values": values,
            "stats": {n: getattr(st, n) for n, _ in _Stats._fields_}}


def train_step_ragged(net: Net, theta, g, frames, actions, rewards, dones, seg_start, bootstrap, hp: HParams):
    """One whole update on segments of unequal length (Sec. 4.1): frames u8 [F,C,H,W], actions / rewards / dones [F],
    seg_start [N+1], bootstrap [N].  The steps of train_step in the same order, each through its own function:
    forward, returns, loss and head gradients, backward, norm, clip, RMSProp."""
    theta = _f64(theta); g = _f64(g)
    frames = np.ascontiguousarray(frames, dtype=np.uint8)
    actions = np.ascontiguousarray(actions, dtype=np.int32).reshape(-1)
    fw = forward(net, theta, frames, want_acts=True)
    logits, values, acts = fw["logits"], fw["values"], fw["acts"]
    R = returns_ragged(rewards, dones, seg_start, bootstrap, hp.gamma)
    dZ, dV, sums = loss_grad(logits, values, actions, R, hp.beta, hp.value_coef, hp.log_eps)
    grad = backward(net, theta, acts, dZ, dV)
    norm = grad_norm(grad)
    s = clip_scale(norm, hp.clip_norm)
    theta2, g2 = rmsprop(theta, g, grad, s, hp.lr, hp.rms_decay, hp.rms_eps)
    return {"theta": theta2, "g": g2, "grad": grad, "R": R, "dZ": dZ, "dV": dV, "logits": logits, "values": values,
            "stats": dict(sums, grad_norm=norm, clip_scale=s)}
