"""Build libocn.so: the HIP kernels and the C-ABI host library, for gfx950, in-tree.

    python -m paper_1810_08723_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libocn.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Floating-point contraction stays off: a*b+c must round twice, as in the definition of each
# operation.  Packed-FP32 instruction selection is switched off for the device pass.
COMMON = ["--offload-arch=gfx950", *os.environ.get("OCN_EXTRA_FLAGS", "").split(), "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]

SOURCES = (["api.cpp", "planner.cpp", "ew_launch.cpp", "red_launch.cpp", "ew_interp.hip", "index.hip"]
           + [f"ew_slice_{i}.hip" for i in range(8)] + [f"red_slice_{i}.hip" for i in range(4)]
           + [f"fred_slice_{i}.hip" for i in range(4)])


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *COMMON, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int | None = None) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(16, os.cpu_count() or 4)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
