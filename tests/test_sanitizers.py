"""AddressSanitizer + UndefinedBehaviorSanitizer passes over the CPU side: the oracle (all
schedules, follow mode, tight buffers; float and double builds) and the library's host-only
logic (stage planner, weight packer, e4m3 encoder).  Both are built here with gcc/g++ and run
as separate programs; a sanitizer report or a wrong result makes them exit non-zero.  No GPU."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
       "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(exe):
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert r.stdout.startswith("ok"), r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]


@pytest.mark.parametrize("real", ["float", "double"])
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path, real):
    exe = str(tmp_path / f"orc_san_{real}")
    subprocess.run(["gcc", *SAN, "-fopenmp", "-ffp-contract=off", f"-DREAL={real}",
                    "-I", os.path.join(ROOT, "oracle"),
                    os.path.join(ROOT, "oracle", "sanitize_driver.c"), "-o", exe, "-lm"],
                   check=True, capture_output=True)
    _run(exe)


def test_host_packer_and_planner_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_pack_check")
    subprocess.run(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
                    "-I", os.path.join(ROOT, "paper_2406_03791_amd", "csrc"),
                    os.path.join(ROOT, "tests", "host_pack_check.cpp"), "-o", exe],
                   check=True, capture_output=True)
    _run(exe)
