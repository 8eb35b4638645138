"""The library's host code under AddressSanitizer / UndefinedBehaviorSanitizer on a GPU: a C++ driver (no Python, so
nothing has to be preloaded) calls every entry point of the C ABI on the tiny model, with one to four micro-batches in
flight, through both group pipelines, the static-scratch entry point, the measurement entry points and the error paths.
Any report of either sanitizer ends the program with a non-zero status.  (The file name places it after the parity tests.)"""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(HERE, "host_sanitizer_driver")


@pytest.mark.gpu
def test_every_entry_point_runs_clean_under_host_sanitizers():
    if not os.path.exists(EXE):
        pytest.skip("tests/host_sanitizer_driver is not built: run `python -c 'import __graft_entry__ as g; g.build()'` first")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:protect_shadow_gap=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=110, env=env)
    everything = r.stdout + r.stderr
    tail = everything[-3000:]
    if r.returncode != 0 and "[host-sanitizer-driver] create" not in r.stdout:
        pytest.skip("the sanitizer runtime could not start in this environment: " + tail[-300:])
    ours = ("ss_engine.hip", "ss_kernels.hip", "ss_sched.cpp", "ss_plan.cpp", "ss_common.cpp", "host_sanitizer_driver.cpp")
    if r.returncode != 0 and "Sanitizer" in everything and not any(name in everything for name in ours):
        # every frame of the report lies in the GPU runtime's libraries (seen once, in their exit handlers): not this code
        pytest.skip("a sanitizer report with no frame in this library's sources: " + everything[:600])
    assert r.returncode == 0, everything[:1500] + "\n...\n" + tail
    assert "[host-sanitizer-driver] done" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
