"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/ga3c.h declares, and refuses bad arguments before it
touches the device."""
import ctypes as C
import os
import re

import paper_1611_06256_amd as g
from paper_1611_06256_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ga3c.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ga3c_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = g.load_library()
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_header():
    assert C.sizeof(binding._NetDesc) == 4 * (4 + 3 * 4 + 3)
    assert C.sizeof(binding._HParams) == 32
    assert C.sizeof(binding.TrainStats) == 24


def test_bad_arguments_are_refused_without_a_device():
    lib = g.load_library()
    ctx = C.c_void_p()
    assert lib.ga3c_create(None, 1, 1, C.byref(ctx)) == -1
    assert b"null" in lib.ga3c_last_error()
    d = g.SMALL_NET(6).c()
    d.n_conv = 5
    assert lib.ga3c_create(C.byref(d), 1, 1, C.byref(ctx)) == -1 and not ctx.value
    d = g.SMALL_NET(64).c()
    assert lib.ga3c_create(C.byref(d), 1, 1, C.byref(ctx)) == -1
    d = g.NetDesc(in_h=6, in_w=6).c()          # 8x8 filter does not fit a 6x6 input
    assert lib.ga3c_create(C.byref(d), 1, 1, C.byref(ctx)) == -1
    assert b"conv layer 0" in lib.ga3c_last_error()
    d = g.SMALL_NET(6).c()
    assert lib.ga3c_create(C.byref(d), -1, 1, C.byref(ctx)) == -1
    d.math = 2                                  # 0 = fp32, 1 = bfloat16 operands; nothing else
    assert lib.ga3c_create(C.byref(d), 1, 1, C.byref(ctx)) == -1
    assert lib.ga3c_params_count(None) == 0
    assert lib.ga3c_destroy(None) == 0
    assert lib.ga3c_predict(None, None, 1, None, None, None, None, None, None) == -1
    assert lib.ga3c_params_init(None, 1, None) == -1
    assert lib.ga3c_rmsprop_flat(None, None, None, 4, 1.0, 1.0, 0.9, 0.1, None) == -1


def test_ticket_hand_off_model_is_race_free_and_the_sanitizer_sees_the_ordering_it_needs(tmp_path):
    # tests/ticket_model.cpp models the hand-off between the workgroups of a frame in the one-launch prediction
    # kernel with host threads; under the thread sanitizer the protocol as used (stores acknowledged, barrier,
    # ordered ticket) is clean over 200 launches, and the same model with the ordering at the ticket left out is
    # reported as a data race: the check is able to fail
    import subprocess
    exe = str(tmp_path / "ticket_model")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-pthread", "-o", exe,
                           os.path.join(ROOT, "tests", "ticket_model.cpp")])
    ok = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert ok.returncode == 0 and "ok 200" in ok.stdout, ok.stdout + ok.stderr
    assert "ThreadSanitizer" not in ok.stderr
    racy = subprocess.run([exe, "relaxed"], capture_output=True, text=True, timeout=300)
    assert racy.returncode != 0 and "data race" in racy.stderr


def test_benchmark_refuses_more_than_one_gpu():
    # this build is for one GPU: the benchmark says so instead of running a second rank
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
