"""ctypes binding of libga3c.so.  Argument marshalling only.

torch is used for device memory and for the stream handle; tensors passed in
must live on the GPU, be contiguous and have the dtype the C ABI names.
There is no CPU fallback: without the compiled library, or without a GPU,
the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
MAX_CONV = 4


class Ga3cError(RuntimeError):
    pass


class _Conv(C.Structure):
    _fields_ = [("oc", C.c_int), ("k", C.c_int), ("stride", C.c_int)]


class _NetDesc(C.Structure):
    _fields_ = [("in_c", C.c_int), ("in_h", C.c_int), ("in_w", C.c_int), ("n_conv", C.c_int),
                ("conv", _Conv * MAX_CONV), ("fc_units", C.c_int), ("n_actions", C.c_int), ("math", C.c_int)]


class _HParams(C.Structure):
    _fields_ = [(n, C.c_float) for n in
                ("gamma", "beta", "value_coef", "log_eps", "lr", "rms_decay", "rms_eps", "clip_norm")]


class _SchedConfig(C.Structure):
    _fields_ = [("t_max", C.c_int), ("predict_cap", C.c_int), ("train_min", C.c_int), ("train_cap", C.c_int),
                ("adjust_period", C.c_int), ("predict_cap_lo", C.c_int), ("predict_cap_hi", C.c_int),
                ("train_cap_lo", C.c_int), ("train_cap_hi", C.c_int), ("train_cap_step", C.c_int),
                ("seed", C.c_uint64), ("hp", _HParams), ("adjust_margin", C.c_float)]


class Prediction(C.Structure):
    _fields_ = [("agent", C.c_int32), ("action", C.c_int32), ("value", C.c_float), ("policy_version", C.c_int32)]


class SchedStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in
                ("ticks", "predictions", "predict_batches", "trained_frames", "train_batches", "sum_predict_queue",
                 "sum_train_queue", "predict_queue", "train_queue", "trials_accepted", "trials_rejected")] + \
               [("predict_cap", C.c_int32), ("train_cap", C.c_int32), ("last_window_frames_per_s", C.c_double)] + \
               [(n, C.c_int64) for n in ("short_segments", "lag_sum", "lag_count", "lag_max", "windows",
                                         "last_change_window")]


class TrainStats(C.Structure):
    _fields_ = [("policy_loss", C.c_float), ("value_loss", C.c_float), ("entropy", C.c_float),
                ("grad_norm", C.c_float), ("clip_scale", C.c_float), ("nonfinite", C.c_int32)]


@dataclass
class NetDesc:
    in_c: int = 4
    in_h: int = 84
    in_w: int = 84
    conv: Sequence[Tuple[int, int, int]] = ((16, 8, 4), (32, 4, 2))
    fc_units: int = 256
    n_actions: int = 18
    math: int = 0

    def c(self) -> _NetDesc:
        d = _NetDesc()
        d.in_c, d.in_h, d.in_w, d.n_conv = self.in_c, self.in_h, self.in_w, len(self.conv)
        for i, (oc, k, s) in enumerate(self.conv):
            d.conv[i].oc, d.conv[i].k, d.conv[i].stride = oc, k, s
        d.fc_units, d.n_actions, d.math = self.fc_units, self.n_actions, self.math
        return d


def SMALL_NET(n_actions: int = 18) -> NetDesc:
    return NetDesc(n_actions=n_actions)


def LARGE_NET(n_actions: int = 18) -> NetDesc:
    return NetDesc(conv=((32, 8, 4), (64, 4, 2), (64, 3, 1)), fc_units=512, n_actions=n_actions)


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


def lib_path() -> str:
    return os.path.join(HERE, "libga3c.so")


_lib = None

EXPORTS = ("ga3c_create", "ga3c_destroy", "ga3c_params_count", "ga3c_params_offsets", "ga3c_params_init",
           "ga3c_params_get", "ga3c_params_set", "ga3c_predict", "ga3c_train_step", "ga3c_train_step_ragged",
           "ga3c_train_debug_get",
           "ga3c_rmsprop_flat", "ga3c_last_error", "ga3c_profile_enable", "ga3c_profile_read",
           "ga3c_use_generic_kernels", "ga3c_get_desc", "ga3c_predict_static",
           "ga3c_sched_create", "ga3c_sched_destroy", "ga3c_sched_submit_predict", "ga3c_sched_submit_trajectory",
           "ga3c_sched_submit_segment", "ga3c_sched_submit_segment_many",
           "ga3c_sched_submit_predict_many", "ga3c_sched_submit_trajectory_many",
           "ga3c_sched_tick", "ga3c_sched_poll", "ga3c_sched_drain", "ga3c_sched_get_stats", "ga3c_sched_last_error",
           "ga3c_tuner_create", "ga3c_tuner_report", "ga3c_tuner_state", "ga3c_tuner_destroy", "ga3c_tuner_set_margin",
           "ga3c_tuner_progress")


def load_library() -> C.CDLL:
    """Loads the built library; builds it first only if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build(True)
    lib = C.CDLL(path)
    vp, i32, u64, sz, f32 = C.c_void_p, C.c_int, C.c_uint64, C.c_size_t, C.c_float
    lib.ga3c_create.argtypes = [C.POINTER(_NetDesc), i32, i32, C.POINTER(vp)]
    lib.ga3c_destroy.argtypes = [vp]
    lib.ga3c_params_count.argtypes = [vp]
    lib.ga3c_params_count.restype = sz
    lib.ga3c_params_offsets.argtypes = [vp, C.POINTER(C.c_int64), i32]
    lib.ga3c_params_init.argtypes = [vp, u64, vp]
    lib.ga3c_params_get.argtypes = [vp, i32, vp, sz, vp]
    lib.ga3c_params_set.argtypes = [vp, i32, vp, sz, vp]
    lib.ga3c_predict.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.ga3c_train_step.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, C.POINTER(_HParams), vp, vp]
    lib.ga3c_train_step_ragged.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, C.POINTER(_HParams), vp, vp]
    lib.ga3c_train_debug_get.argtypes = [vp, i32, vp, sz, vp]
    lib.ga3c_predict_static.argtypes = [i32, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.ga3c_rmsprop_flat.argtypes = [vp, vp, vp, sz, f32, f32, f32, f32, vp]
    lib.ga3c_last_error.restype = C.c_char_p
    lib.ga3c_profile_enable.argtypes = [vp, i32]
    lib.ga3c_get_desc.argtypes = [vp, C.POINTER(_NetDesc), C.POINTER(i32), C.POINTER(i32)]
    lib.ga3c_sched_create.argtypes = [vp, C.POINTER(_SchedConfig), C.POINTER(vp)]
    lib.ga3c_sched_destroy.argtypes = [vp]
    lib.ga3c_sched_submit_predict.argtypes = [vp, i32, vp, f32]
    lib.ga3c_sched_submit_trajectory.argtypes = [vp, i32, vp, vp, vp, vp, f32]
    lib.ga3c_sched_submit_segment.argtypes = [vp, i32, vp, i32, vp, vp, vp, f32, C.c_int64]
    lib.ga3c_sched_submit_segment_many.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ga3c_sched_submit_predict_many.argtypes = [vp, i32, vp, vp, vp]
    lib.ga3c_sched_submit_trajectory_many.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
    lib.ga3c_sched_tick.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
    lib.ga3c_sched_poll.argtypes = [vp, C.POINTER(Prediction), i32]
    lib.ga3c_sched_drain.argtypes = [vp]
    lib.ga3c_sched_get_stats.argtypes = [vp, C.POINTER(SchedStats)]
    lib.ga3c_sched_last_error.restype = C.c_char_p
    lib.ga3c_tuner_create.argtypes = [i32, i32, i32, i32, i32, i32, i32, u64, C.POINTER(vp)]
    lib.ga3c_tuner_report.argtypes = [vp, C.c_double, C.POINTER(i32), C.POINTER(i32)]
    lib.ga3c_tuner_state.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.ga3c_tuner_destroy.argtypes = [vp]
    lib.ga3c_tuner_set_margin.argtypes = [vp, C.c_double]
    lib.ga3c_tuner_progress.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.ga3c_use_generic_kernels.argtypes = [vp, i32]
    lib.ga3c_profile_read.argtypes = [vp, C.c_char_p, sz]
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc < 0:
        raise Ga3cError(f"{what} failed ({rc}): {load_library().ga3c_last_error().decode()}")


def _ptr(t, dtype, what: str):
    """Device pointer of a tensor after checking device, dtype and layout."""
    import torch
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise Ga3cError(f"{what}: expected a GPU tensor")
    if t.dtype != dtype:
        raise Ga3cError(f"{what}: expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise Ga3cError(f"{what}: tensor must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


class Ga3c:
    """One network on the current GPU: ga3c_create .. ga3c_destroy."""

    def __init__(self, desc: NetDesc, max_predict_batch: int, max_train_frames: int):
        import torch
        if not torch.cuda.is_available():
            raise Ga3cError("no GPU visible: the HIP path has no CPU fallback")
        self._lib = load_library()
        self.desc = desc
        self._ctx = C.c_void_p()
        cd = desc.c()
        _check(self._lib.ga3c_create(C.byref(cd), max_predict_batch, max_train_frames, C.byref(self._ctx)),
               "ga3c_create")
        self.n_params = int(self._lib.ga3c_params_count(self._ctx))
        self.n_actions = desc.n_actions

    def close(self) -> None:
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self._lib.ga3c_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def offsets(self) -> Dict[str, Tuple[int, Tuple[int, ...]]]:
        """Name -> (offset, shape) of each tensor in the flat parameter vector."""
        off = (C.c_int64 * (2 * MAX_CONV + 7))()
        n = self._lib.ga3c_params_offsets(self._ctx, off, len(off))
        _check(n, "ga3c_params_offsets")
        o = [int(off[i]) for i in range(n)]
        d = self.desc
        out: Dict[str, Tuple[int, Tuple[int, ...]]] = {}
        c, h, w = d.in_c, d.in_h, d.in_w
        for l, (oc, k, s) in enumerate(d.conv):
            out[f"conv{l + 1}.W"] = (o[2 * l], (oc, c, k, k))
            out[f"conv{l + 1}.b"] = (o[2 * l + 1], (oc,))
            c, h, w = oc, (h - k) // s + 1, (w - k) // s + 1
        nb = 2 * len(d.conv)
        out["fc.W"] = (o[nb], (d.fc_units, c * h * w))
        out["fc.b"] = (o[nb + 1], (d.fc_units,))
        out["policy.W"] = (o[nb + 2], (d.n_actions, d.fc_units))
        out["policy.b"] = (o[nb + 3], (d.n_actions,))
        out["value.W"] = (o[nb + 4], (1, d.fc_units))
        out["value.b"] = (o[nb + 5], (1,))
        return out

    def params_init(self, seed: int, stream=None) -> None:
        _check(self._lib.ga3c_params_init(self._ctx, seed, _stream(stream)), "ga3c_params_init")

    def params_get(self, which: int = 0, out=None, stream=None):
        import torch
        if out is None:
            out = torch.empty(self.n_params, dtype=torch.float32, device="cuda")
        _check(self._lib.ga3c_params_get(self._ctx, which, _ptr(out, torch.float32, "out"), out.numel(),
                                         _stream(stream)), "ga3c_params_get")
        return out

    def params_set(self, src, which: int = 0, stream=None) -> None:
        import torch
        _check(self._lib.ga3c_params_set(self._ctx, which, _ptr(src, torch.float32, "src"), src.numel(),
                                         _stream(stream)), "ga3c_params_set")

    def predict(self, frames, uniforms=None, logits=None, values=None, probs=None, actions=None, stream=None):
        """frames u8 [B,C,H,W].  Output tensors that are passed in are filled."""
        import torch
        B = int(frames.shape[0])
        _check(self._lib.ga3c_predict(self._ctx, _ptr(frames, torch.uint8, "frames"), B,
                                      _ptr(uniforms, torch.float32, "uniforms"),
                                      _ptr(logits, torch.float32, "logits"), _ptr(values, torch.float32, "values"),
                                      _ptr(probs, torch.float32, "probs"), _ptr(actions, torch.int32, "actions"),
                                      _stream(stream)), "ga3c_predict")

    def train_step(self, frames, actions, rewards, dones, bootstrap, hp: HParams, stats=None, stream=None) -> None:
        """frames u8 [N,T,C,H,W]; actions i32, rewards f32, dones u8 [N,T]; bootstrap f32 [N] or None;
        stats: optional u8/any GPU tensor of at least 24 bytes that receives ga3c_train_stats."""
        import torch
        N, T = int(frames.shape[0]), int(frames.shape[1])
        hpc = hp.c()
        sp = None
        if stats is not None:
            if not stats.is_cuda or stats.numel() * stats.element_size() < C.sizeof(TrainStats):
                raise Ga3cError("stats: need a GPU tensor of at least 24 bytes")
            sp = C.c_void_p(stats.data_ptr())
        _check(self._lib.ga3c_train_step(self._ctx, _ptr(frames, torch.uint8, "frames"),
                                         _ptr(actions, torch.int32, "actions"), _ptr(rewards, torch.float32, "rewards"),
                                         _ptr(dones, torch.uint8, "dones"), _ptr(bootstrap, torch.float32, "bootstrap"),
                                         N, T, C.byref(hpc), sp, _stream(stream)), "ga3c_train_step")

    def train_step_ragged(self, frames, actions, rewards, dones, seg_start, bootstrap, hp: HParams, stats=None,
                          stream=None) -> None:
        """Segments of unequal length laid end to end: frames u8 [F,C,H,W]; actions i32, rewards f32, dones u8 [F];
        seg_start i32 [N+1] (GPU tensor); bootstrap f32 [N] or None."""
        import torch
        F, N = int(frames.shape[0]), int(seg_start.numel()) - 1
        if actions.numel() != F or rewards.numel() != F or dones.numel() != F or N < 0 or \
                (bootstrap is not None and bootstrap.numel() != N):
            raise Ga3cError("train_step_ragged: array sizes do not match the frame or segment count")
        hpc = hp.c()
        sp = None
        if stats is not None:
            if not stats.is_cuda or stats.numel() * stats.element_size() < C.sizeof(TrainStats):
                raise Ga3cError("stats: need a GPU tensor of at least 24 bytes")
            sp = C.c_void_p(stats.data_ptr())
        _check(self._lib.ga3c_train_step_ragged(
            self._ctx, _ptr(frames, torch.uint8, "frames"), _ptr(actions, torch.int32, "actions"),
            _ptr(rewards, torch.float32, "rewards"), _ptr(dones, torch.uint8, "dones"),
            _ptr(seg_start, torch.int32, "seg_start"), _ptr(bootstrap, torch.float32, "bootstrap"),
            N, F, C.byref(hpc), sp, _stream(stream)), "ga3c_train_step_ragged")

    def use_generic_kernels(self, on: bool) -> None:
        _check(self._lib.ga3c_use_generic_kernels(self._ctx, 1 if on else 0), "ga3c_use_generic_kernels")

    def profile_enable(self, on: bool) -> None:
        _check(self._lib.ga3c_profile_enable(self._ctx, 1 if on else 0), "ga3c_profile_enable")

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        """stage -> {calls, ms, flop, bytes} accumulated since the last read."""
        buf = C.create_string_buffer(1 << 16)
        _check(self._lib.ga3c_profile_read(self._ctx, buf, len(buf)), "ga3c_profile_read")
        out: Dict[str, Dict[str, float]] = {}
        for line in buf.value.decode().splitlines():
            name, calls, ms, flop, nbytes = line.split()
            out[name] = {"calls": int(calls), "ms": float(ms), "flop": float(flop), "bytes": float(nbytes)}
        return out

    def train_debug_get(self, which: int, out, stream=None):
        import torch
        _check(self._lib.ga3c_train_debug_get(self._ctx, which, _ptr(out, torch.float32, "out"), out.numel(),
                                              _stream(stream)), "ga3c_train_debug_get")
        return out


STATIC_MAX_FRAMES = 256        # GA3C_STATIC_MAX_FRAMES of include/ga3c.h


def predict_static(n_actions: int, math: int, theta, frames, uniforms=None, logits=None, values=None, probs=None,
                   actions=None, stream=None) -> None:
    """ga3c_predict_static: prediction of the Sec. 3.2 network from the caller's flat parameters, no context and no
    device allocation (at most STATIC_MAX_FRAMES frames)."""
    import torch
    lib = load_library()
    _check(lib.ga3c_predict_static(n_actions, math, _ptr(theta, torch.float32, "theta"), _ptr(frames, torch.uint8, "frames"),
                                   int(frames.shape[0]), _ptr(uniforms, torch.float32, "uniforms"),
                                   _ptr(logits, torch.float32, "logits"), _ptr(values, torch.float32, "values"),
                                   _ptr(probs, torch.float32, "probs"), _ptr(actions, torch.int32, "actions"),
                                   _stream(stream)), "ga3c_predict_static")


def _scheck(rc: int, what: str) -> int:
    if rc < 0:
        raise Ga3cError(f"{what} failed ({rc}): {load_library().ga3c_sched_last_error().decode()}")
    return rc


class Tuner:
    """The adjustment rule of the scheduler on its own (host only)."""

    def __init__(self, p_lo, p_hi, p0, t_lo, t_hi, t_step, t0, seed):
        self._lib = load_library()
        self._t = C.c_void_p()
        _scheck(self._lib.ga3c_tuner_create(p_lo, p_hi, p0, t_lo, t_hi, t_step, t0, seed, C.byref(self._t)),
                "ga3c_tuner_create")

    def report(self, throughput: float) -> Tuple[int, int]:
        p, t = C.c_int(), C.c_int()
        _scheck(self._lib.ga3c_tuner_report(self._t, throughput, C.byref(p), C.byref(t)), "ga3c_tuner_report")
        return p.value, t.value

    def set_margin(self, margin: float) -> None:
        _scheck(self._lib.ga3c_tuner_set_margin(self._t, margin), "ga3c_tuner_set_margin")

    def state(self):
        p, t, a, r, w, lc = C.c_int(), C.c_int(), C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
        _scheck(self._lib.ga3c_tuner_state(self._t, C.byref(p), C.byref(t), C.byref(a), C.byref(r)), "ga3c_tuner_state")
        _scheck(self._lib.ga3c_tuner_progress(self._t, C.byref(w), C.byref(lc)), "ga3c_tuner_progress")
        return {"predict_cap": p.value, "train_cap": t.value, "accepted": a.value, "rejected": r.value,
                "windows": w.value, "last_change_window": lc.value}

    def __del__(self):
        try:
            self._lib.ga3c_tuner_destroy(self._t)
        except Exception:
            pass


class Scheduler:
    """ga3c_sched_*: queues, two streams, batch caps and their adjustment."""

    def __init__(self, net: Ga3c, hp: HParams, t_max=5, predict_cap=256, train_min=40, train_cap=1280,
                 adjust_period=0, predict_cap_lo=1, predict_cap_hi=256, train_cap_lo=40, train_cap_hi=1280,
                 train_cap_step=40, seed=0, adjust_margin=0.0):
        self._lib = load_library()
        self._net = net
        cfg = _SchedConfig(t_max, predict_cap, train_min, train_cap, adjust_period, predict_cap_lo, predict_cap_hi,
                           train_cap_lo, train_cap_hi, train_cap_step, seed, hp.c(), adjust_margin)
        self._s = C.c_void_p()
        self.t_max = t_max
        _scheck(self._lib.ga3c_sched_create(net._ctx, C.byref(cfg), C.byref(self._s)), "ga3c_sched_create")

    def close(self):
        if self._s.value:
            self._lib.ga3c_sched_destroy(self._s)
            self._s = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def submit_predict(self, agent: int, frame, uniform: float) -> None:
        import torch
        _scheck(self._lib.ga3c_sched_submit_predict(self._s, agent, _ptr(frame, torch.uint8, "frame"), uniform),
                "ga3c_sched_submit_predict")

    def submit_trajectory(self, agent: int, frames, actions, rewards, dones, bootstrap: float) -> None:
        """frames: GPU u8 [t_max,C,H,W]; actions i32 / rewards f32 / dones u8: numpy arrays of t_max entries."""
        import numpy as np
        import torch
        a = np.ascontiguousarray(actions, dtype=np.int32); r = np.ascontiguousarray(rewards, dtype=np.float32)
        d = np.ascontiguousarray(dones, dtype=np.uint8)
        if a.size != self.t_max or r.size != self.t_max or d.size != self.t_max:
            raise Ga3cError("trajectory arrays must have t_max entries")
        _scheck(self._lib.ga3c_sched_submit_trajectory(self._s, agent, _ptr(frames, torch.uint8, "frames"),
                                                       a.ctypes.data_as(C.c_void_p), r.ctypes.data_as(C.c_void_p),
                                                       d.ctypes.data_as(C.c_void_p), bootstrap),
                "ga3c_sched_submit_trajectory")

    def submit_segment(self, agent: int, frames, actions, rewards, dones, bootstrap: float, policy_version: int = -1) -> None:
        """frames: GPU u8 [len,C,H,W] with 1 <= len <= t_max; actions / rewards / dones: numpy arrays of len entries;
        policy_version: the one that came with the prediction of the first action (-1 = not given)."""
        import numpy as np
        import torch
        a = np.ascontiguousarray(actions, dtype=np.int32); r = np.ascontiguousarray(rewards, dtype=np.float32)
        d = np.ascontiguousarray(dones, dtype=np.uint8)
        if r.size != a.size or d.size != a.size or int(frames.shape[0]) != a.size:
            raise Ga3cError("segment arrays and frames must have the same number of entries")
        _scheck(self._lib.ga3c_sched_submit_segment(self._s, agent, _ptr(frames, torch.uint8, "frames"), a.size,
                                                    a.ctypes.data_as(C.c_void_p), r.ctypes.data_as(C.c_void_p),
                                                    d.ctypes.data_as(C.c_void_p), bootstrap, policy_version),
                "ga3c_sched_submit_segment")

    def submit_predict_many(self, agents, frame_ptrs, uniforms) -> None:
        """agents i32 [n], frame_ptrs u64 [n] (device addresses), uniforms f32 [n]: numpy arrays."""
        import numpy as np
        a = np.ascontiguousarray(agents, dtype=np.int32); p = np.ascontiguousarray(frame_ptrs, dtype=np.uint64)
        u = np.ascontiguousarray(uniforms, dtype=np.float32)
        _scheck(self._lib.ga3c_sched_submit_predict_many(self._s, a.size, a.ctypes.data_as(C.c_void_p),
                                                         p.ctypes.data_as(C.c_void_p), u.ctypes.data_as(C.c_void_p)),
                "ga3c_sched_submit_predict_many")

    def submit_trajectory_many(self, agents, frame_ptrs, actions, rewards, dones, bootstrap) -> None:
        import numpy as np
        a = np.ascontiguousarray(agents, dtype=np.int32); p = np.ascontiguousarray(frame_ptrs, dtype=np.uint64)
        ac = np.ascontiguousarray(actions, dtype=np.int32); r = np.ascontiguousarray(rewards, dtype=np.float32)
        d = np.ascontiguousarray(dones, dtype=np.uint8); bo = np.ascontiguousarray(bootstrap, dtype=np.float32)
        if ac.size != a.size * self.t_max or r.size != ac.size or d.size != ac.size or bo.size != a.size:
            raise Ga3cError("trajectory arrays must be [n, t_max] and [n]")
        _scheck(self._lib.ga3c_sched_submit_trajectory_many(
            self._s, a.size, a.ctypes.data_as(C.c_void_p), p.ctypes.data_as(C.c_void_p),
            ac.ctypes.data_as(C.c_void_p), r.ctypes.data_as(C.c_void_p), d.ctypes.data_as(C.c_void_p),
            bo.ctypes.data_as(C.c_void_p)), "ga3c_sched_submit_trajectory_many")

    def submit_segment_many(self, agents, frame_ptrs, lens, actions, rewards, dones, bootstrap, policy_versions=None) -> None:
        """n segments at once: lens i32 [n]; actions / rewards / dones [n, t_max] (row i: the first lens[i] entries
        count); frame_ptrs u64 [n] (device addresses); policy_versions i64 [n] or None."""
        import numpy as np
        a = np.ascontiguousarray(agents, dtype=np.int32); p = np.ascontiguousarray(frame_ptrs, dtype=np.uint64)
        ln = np.ascontiguousarray(lens, dtype=np.int32)
        ac = np.ascontiguousarray(actions, dtype=np.int32); r = np.ascontiguousarray(rewards, dtype=np.float32)
        d = np.ascontiguousarray(dones, dtype=np.uint8); bo = np.ascontiguousarray(bootstrap, dtype=np.float32)
        pv = None if policy_versions is None else np.ascontiguousarray(policy_versions, dtype=np.int64)
        if ac.size != a.size * self.t_max or r.size != ac.size or d.size != ac.size or bo.size != a.size or \
                ln.size != a.size or p.size != a.size or (pv is not None and pv.size != a.size):
            raise Ga3cError("segment arrays must be [n, t_max] and [n]")
        _scheck(self._lib.ga3c_sched_submit_segment_many(
            self._s, a.size, a.ctypes.data_as(C.c_void_p), p.ctypes.data_as(C.c_void_p), ln.ctypes.data_as(C.c_void_p),
            ac.ctypes.data_as(C.c_void_p), r.ctypes.data_as(C.c_void_p), d.ctypes.data_as(C.c_void_p),
            bo.ctypes.data_as(C.c_void_p), None if pv is None else pv.ctypes.data_as(C.c_void_p)),
            "ga3c_sched_submit_segment_many")

    def poll_arrays(self, cap: int = 4096, with_version: bool = False):
        """Finished predictions as numpy arrays (agents, actions, values[, policy versions])."""
        import numpy as np
        buf = (Prediction * cap)()
        n = _scheck(self._lib.ga3c_sched_poll(self._s, buf, cap), "ga3c_sched_poll")
        rec = np.frombuffer(buf, dtype=np.dtype([("agent", "<i4"), ("action", "<i4"), ("value", "<f4"),
                                                 ("policy_version", "<i4")]), count=n)
        out = (rec["agent"].copy(), rec["action"].copy(), rec["value"].copy())
        return out + (rec["policy_version"].copy(),) if with_version else out

    def tick(self) -> Tuple[int, int]:
        p, t = C.c_int(), C.c_int()
        _scheck(self._lib.ga3c_sched_tick(self._s, C.byref(p), C.byref(t)), "ga3c_sched_tick")
        return p.value, t.value

    def poll(self, cap: int = 4096):
        buf = (Prediction * cap)()
        n = _scheck(self._lib.ga3c_sched_poll(self._s, buf, cap), "ga3c_sched_poll")
        return [(buf[i].agent, buf[i].action, buf[i].value) for i in range(n)]

    def drain(self) -> None:
        _scheck(self._lib.ga3c_sched_drain(self._s), "ga3c_sched_drain")

    def stats(self) -> Dict[str, float]:
        st = SchedStats()
        _scheck(self._lib.ga3c_sched_get_stats(self._s, C.byref(st)), "ga3c_sched_get_stats")
        return {n: getattr(st, n) for n, _ in SchedStats._fields_}


def rmsprop_flat(theta, g, grad, scale: float, lr: float, rms_decay: float, rms_eps: float, stream=None) -> None:
    import torch
    _check(load_library().ga3c_rmsprop_flat(_ptr(theta, torch.float32, "theta"), _ptr(g, torch.float32, "g"),
                                            _ptr(grad, torch.float32, "grad"), theta.numel(), scale, lr, rms_decay,
                                            rms_eps, _stream(stream)), "ga3c_rmsprop_flat")


def stats_from_tensor(t) -> Dict[str, float]:
    """Decode a ga3c_train_stats struct held in a (synchronised) GPU tensor."""
    raw = bytes(t.detach().cpu().numpy().tobytes()[:C.sizeof(TrainStats)])
    st = TrainStats.from_buffer_copy(raw)
    return {n: getattr(st, n) for n, _ in TrainStats._fields_}
