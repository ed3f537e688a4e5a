"""Compile the C oracle twice: REAL=float (parity) and REAL=double (finite-difference checks)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gcn_oracle.c")
LIBS = {"f32": ("float", os.path.join(HERE, "liboracle_f32.so")),
        "f64": ("double", os.path.join(HERE, "liboracle_f64.so"))}


def build(force: bool = True) -> None:
    for real, out in LIBS.values():
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
               f"-DREAL={real}", SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build()
