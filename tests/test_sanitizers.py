"""CPU sanitizer tier: the library's host logic (pool.cpp, sched.cpp, window_plan.h) compiled as it is into a test
program (tests/native/host_trace.cpp) with AddressSanitizer + UndefinedBehaviorSanitizer, which replays random traces
against shadow models, and with ThreadSanitizer for two threads allocating and freeing on one pool.  Sanitizers cover
host code only: no GPU call is made, the pool's events are integers of the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_11729_amd", "csrc")
SRC = [os.path.join(ROOT, "tests", "native", "host_trace.cpp"), os.path.join(CSRC, "pool.cpp"), os.path.join(CSRC, "sched.cpp")]
INC = ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", "/opt/rocm/include", "-D__HIP_PLATFORM_AMD__"]


def build(tmp_path, name, san):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / name)
    # sched.cpp creates CU-masked streams through the HIP runtime: the program links it but never calls those entries
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", *san, *INC, *SRC, "-o", exe, "-pthread",
           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    return exe


def run(exe, *args, env_extra=None):
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)          # a sanitizer runtime must come first among the loaded libraries
    env.update(env_extra or {})
    r = subprocess.run([exe, *args], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    return r.stdout


def test_random_traces_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = build(tmp_path, "host_trace_asan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"])
    # leak checking stays on for the test's own objects; what the HIP runtime allocates at load time is not this code's
    out = run(exe, env_extra={"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1",
                              "LSAN_OPTIONS": "suppressions=" + os.path.join(ROOT, "tests", "native", "lsan.supp")})
    assert "traces ok" in out


def test_two_threads_on_one_pool_under_thread_sanitizer(tmp_path):
    exe = build(tmp_path, "host_trace_tsan", ["-fsanitize=thread"])
    out = run(exe, "threads", env_extra={"TSAN_OPTIONS": "halt_on_error=1"})
    assert "threads ok" in out
