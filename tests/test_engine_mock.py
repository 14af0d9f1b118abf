"""The library's host code -- window scheduler, transfer engine, training step, error paths --
compiled with g++ against a host-only stand-in for the HIP runtime (tests/mock_hip/: every stream a
thread, kernels that read their inputs and overwrite their outputs) and run on the CPU under the
address + undefined-behaviour sanitizers and under the thread sanitizer.

What this covers that the GPU tests cannot: an unfenced overlap of a layer copy with a layer
compute is a data race the thread sanitizer reports (a control run shows that it does); operand
extents beyond the arena or a blob are out-of-bounds accesses; leaks of events or bookkeeping on
the failure paths; and the i-th hipMemcpyAsync / kernel launch / event record / stream wait /
event creation failing mid-pass (every position of a pass): SP_ERR_HIP with a text naming the call,
the handle FAILED and still destroyable.  Details in tests/mock_hip/engine_mock_test.cpp.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2410_08791_amd", "csrc")
MOCK = os.path.join(ROOT, "tests", "mock_hip")
ENGINE_SOURCES = ["sp_host.hip", "sp_engine.hip", "sp_train.hip"]

pytestmark = pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")


def build(out, sanitize):
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", f"-fsanitize={sanitize}", "-Wall",
           "-Wno-unused-function", "-I", MOCK, "-I", CSRC, "-x", "c++"]
    if "undefined" in sanitize:
        cmd.append("-fno-sanitize-recover=undefined")
    cmd += [os.path.join(CSRC, f) for f in ENGINE_SOURCES]
    cmd += [os.path.join(MOCK, "mock_hip.cpp"), os.path.join(MOCK, "engine_mock_test.cpp"), "-lpthread", "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 0, r.stdout + r.stderr
    return out


def run(exe, *args, timeout=300):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", TSAN_OPTIONS="halt_on_error=0:exitcode=66",
               UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([exe, *args], capture_output=True, text=True, timeout=timeout, env=env)


def test_engine_under_address_and_undefined_sanitizers(tmp_path):
    exe = build(str(tmp_path / "engine_asan"), "address,undefined")
    r = run(exe)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "all checks passed" in r.stdout, out[-4000:]
    assert "ERROR: AddressSanitizer" not in out and "LeakSanitizer" not in out and "runtime error" not in out, out[-4000:]
    for line in ("ok forward windows arch 0", "ok forward windows arch 1", "ok training arch 0", "ok training arch 1",
                 "ok decode", "ok injected hipMemcpyAsync failures (forward)", "ok injected launch failures (training step)",
                 "ok injected event-creation failures"):
        assert line in r.stdout, line


def test_engine_under_thread_sanitizer_and_the_race_control(tmp_path):
    exe = build(str(tmp_path / "engine_tsan"), "thread")
    r = run(exe)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "all checks passed" in r.stdout, out[-4000:]
    assert "ThreadSanitizer" not in out, out[-4000:]
    # the control: an unfenced copy / compute pair IS reported by this build
    c = run(exe, "--control-race")
    assert "ThreadSanitizer: data race" in c.stderr and c.returncode == 66, (c.returncode, c.stderr[-2000:])
