"""Compile the HIP sources in csrc/ into librnnt_greedy.so for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
SOURCES = ["engine.hip", "decode.hip", "enc_proj.hip", "probes.hip"]
# the decode kernel is instantiated in one unit per (loop nest, row groups, weight storage),
# all compiled from decode_inst.hip, so that the instances build in parallel
INSTANCES = [(nest, rg, wt) for wt in ("f32", "bf16", "fp8", "bf16a", "fp8a", "fp4a") for nest in ("f", "l")
             for rg in (1, 2, 4)] + [("s", 1, wt) for wt in ("f32", "bf16", "fp8", "bf16a", "fp8a", "fp4a")]
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

    def compile_one(job) -> str:
        src, name, defs = job
        obj = os.path.join(OBJ_DIR, name + ".o")
        cmd = ["hipcc", *FLAGS, *defs, "-c", os.path.join(CSRC, src), "-o", obj]
        if not defs:
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        # decode kernel instances: also ask for the register report and say so when an instance
        # uses scratch memory: spilled registers or a stack object cost time without failing a test
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        if r.returncode != 0:
            sys.stderr.write(r.stderr)
            raise subprocess.CalledProcessError(r.returncode, cmd)
        spilled = [ln for ln in r.stderr.splitlines() if "ScratchSize [bytes/lane]:" in ln
                   and not ln.rstrip().endswith(": 0 [-Rpass-analysis=kernel-resource-usage]")]
        if spilled:
            print(f"build.py: {name}: {len(spilled)} kernel instance(s) use scratch memory (a stack object or spilled registers)",
                  file=sys.stderr, flush=True)
        return obj

    jobs_ = [("decode_inst.hip", f"decode_{nest}{rg}_{wt}",
              [f"-DRNNT_INST_NEST={nest}", f"-DRNNT_INST_RG={rg}", f"-DRNNT_INST_WT={wt}"])
             for nest, rg, wt in INSTANCES]
    jobs_ += [(src, src.replace(".hip", ""), []) for src in SOURCES]
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, os.cpu_count() or 1))) as pool:
        objs = list(pool.map(compile_one, jobs_))
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
