"""Compiles the HIP library for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libga3c.so")
SOURCES = [os.path.join(HERE, "csrc", "ga3c.hip"), os.path.join(HERE, "csrc", "sched.hip"),
           os.path.join(HERE, "csrc", "tuner.cpp")]
HEADERS = [os.path.join(HERE, "csrc", f) for f in ("gemm_mfma.hpp", "problems.hpp", "conv_frame.hpp", "dense_gemm.hpp",
                                                  "conv1_bf16x3.hpp", "dense_gemm_bf16x6.hpp", "conv2_bf16x6.hpp", "conv12_fused.hpp", "conv_fwd_bf16x6.hpp",
                                                  "conv_dgrad_bf16x6.hpp", "conv_wgrad_bf16x6.hpp", "conv_wgrad_s1_bf16x6.hpp", "sched_error.hpp", "launch.hpp")] + [
    os.path.join(os.path.dirname(HERE), "include", "ga3c.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
         # packed fp32 instructions stay off: the compiler must not form them
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True) -> str:
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        subprocess.check_call([hipcc] + FLAGS + ["-o", LIB] + SOURCES)
    return LIB


MICROBENCH = os.path.join(HERE, "microbench")


def build_microbench() -> str:
    """The standalone micro-benchmark program (csrc/microbench.hip): chip rates the kernel designs rest on."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    subprocess.check_call([hipcc] + flags + ["-o", MICROBENCH, os.path.join(HERE, "csrc", "microbench.hip")])
    return MICROBENCH


SCHED_SANITIZED = os.path.join(HERE, "sched_sanitized")


def build_sched_sanitized() -> str:
    """The whole library plus tests/sched_sanitizer_driver.cpp as one program whose HOST code is built with the
    address and undefined-behaviour sanitizers (device code is not instrumented); a GPU test runs it."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC", "-O3")] + [
        "-O1", "-g", "-fno-omit-frame-pointer", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
        "-Xarch_host", "-fno-sanitize-recover=all"]
    driver = os.path.join(os.path.dirname(HERE), "tests", "sched_sanitizer_driver.cpp")
    subprocess.check_call([hipcc] + flags + ["-o", SCHED_SANITIZED] + SOURCES + [driver])
    return SCHED_SANITIZED


if __name__ == "__main__":
    import sys
    what = sys.argv[1:]
    print(build_microbench() if what == ["microbench"] else build_sched_sanitized() if what == ["sched_sanitized"] else build(True))
