"""Compile the HIP sources in csrc/ into librnnt_greedy.so for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
SOURCES = ["engine.hip", "decode.hip", "enc_proj.hip",
           "decode_f1.hip", "decode_f2.hip", "decode_f4.hip",
           "decode_l1.hip", "decode_l2.hip", "decode_l4.hip",
           "decode_f1b.hip", "decode_f2b.hip", "decode_f4b.hip",
           "decode_l1b.hip", "decode_l2b.hip", "decode_l4b.hip",
           "decode_f1e.hip", "decode_f2e.hip", "decode_f4e.hip",
           "decode_l1e.hip", "decode_l2e.hip", "decode_l4e.hip"]
LIB = os.path.join(HERE, "librnnt_greedy.so")
OBJ_DIR = os.path.join(HERE, "_build")
FLAGS = ((["-DRNNT_PROFILE"] if os.environ.get("RNNT_PROFILE") else []) +
         os.environ.get("RNNT_EXTRA_FLAGS", "").split() +
         ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-command-line-argument"])


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compile every source to an object (in parallel: the decode kernels are instantiated
    in several translation units for that reason) and link the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, os.cpu_count() or 1))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "rnnt_greedy.h"))
    return all(os.path.getmtime(d) <= t for d in deps)


if __name__ == "__main__":
    print(build(verbose=True))
