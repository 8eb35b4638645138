"""Compile the C oracle (test infrastructure) into two shared objects:

  libom_f64.so  arithmetic in double  (the parity reference)
  libom_f32.so  the same text with -DOM_REAL_FLOAT (plain fp32 evaluation; timed CPU baseline)

Plain gcc, no fast-math: the only reassociation allowed is the explicit
``omp simd reduction`` on the innermost dot product.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "om_model.c")
TARGETS = {"f64": ("libom_f64.so", []), "f32": ("libom_f32.so", ["-DOM_REAL_FLOAT"])}


def lib_path(kind: str) -> str:
    return os.path.join(HERE, TARGETS[kind][0])


def build(force: bool = True) -> None:
    for kind, (name, defs) in TARGETS.items():
        out = os.path.join(HERE, name)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        cmd = ["gcc", "-O2", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
               *defs, SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build()
    print("built", [lib_path(k) for k in TARGETS])
