"""Compile the CPU oracle (plain C) into two shared libraries: the float build
the parity tests use and a double build used as a shadow check."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rnnt_oracle.c")
FLAGS = ["-O2", "-ftree-vectorize", "-ffp-contract=off", "-fno-fast-math",
         "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"]


def lib_path(real: str) -> str:
    return os.path.join(HERE, f"librnnt_oracle_{'f32' if real == 'float' else 'f64'}.so")


def build(force: bool = False) -> None:
    for real in ("float", "double"):
        out = lib_path(real)
        if (not force and os.path.exists(out)
                and os.path.getmtime(out) >= os.path.getmtime(SRC)):
            continue
        cmd = ["gcc", *FLAGS, f"-DREAL={real}", SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build(force="--force" in sys.argv)
    print("built", lib_path("float"), lib_path("double"))
