"""Builds libeggroll.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2511_16652_amd.build        # compile every translation unit and link

The shared object is placed next to this file; it is git-ignored but travels with the tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libeggroll.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
UNITS = ["api", "api_models", "api_noalloc", "k_decoder", "k_models", "k_noise", "k_project", "k_forward", "k_update", "k_int8", "k_update_i8", "k_gru_i8", "k_egg_model"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Wno-pass-failed", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the epilogues are long bodies inside fully unrolled loops over a lane's accumulator blocks: past the
         # default limit (16 K instructions) a "#pragma unroll" is dropped, the accumulator array is then
         # indexed dynamically and lives in scratch memory
         "-mllvm", "-pragma-unroll-threshold=200000"]


def _compile(unit: str) -> str:
    src = os.path.join(CSRC, unit + ".hip")
    obj = os.path.join(OBJDIR, unit + ".o")
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (unit, out))
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def build(jobs: int = 6) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, UNITS))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
