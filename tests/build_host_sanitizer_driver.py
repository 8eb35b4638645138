"""Builds tests/host_sanitizer_driver: the library's sources and a C++ driver of the C ABI in one executable, with
AddressSanitizer and UndefinedBehaviorSanitizer on the host side only (every -fsanitize= follows an -Xarch_host; the
gfx950 device code is compiled as in the product build).  Run here, on the CPU, before the GPU tests."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(os.path.dirname(HERE), "paper_2305_13144_amd", "csrc")
EXE = os.path.join(HERE, "host_sanitizer_driver")
SOURCES = ["ss_common.cpp", "ss_sched.cpp", "ss_plan.cpp", "ss_kernels.hip", "ss_engine.hip"]


def build() -> str:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-pthread",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           *[os.path.join(CSRC, s) for s in SOURCES], os.path.join(HERE, "host_sanitizer_driver.cpp"), "-o", EXE]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        noise = "is not a recognized feature for this target"
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in r.stderr.splitlines() if noise not in l))
    return EXE


if __name__ == "__main__":
    print(build())
