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
# OCN_BUILD_TAG builds an experimental variant beside the library (with OCN_EXTRA_FLAGS)
_TAG = os.environ.get("OCN_BUILD_TAG", "")
OBJ = os.path.join(HERE, "_build" + ("_" + _TAG if _TAG else ""))
LIB = os.path.join(HERE, "libocn" + ("_" + _TAG if _TAG else "") + ".so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Floating-point contraction stays off: a*b+c must round twice, as in the definition of each
# operation.  Packed-FP32 instruction selection is switched off for the device pass.
COMMON = ["--offload-arch=gfx950", *os.environ.get("OCN_EXTRA_FLAGS", "").split(), "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]

SOURCES = (["api.cpp", "planner.cpp", "ew_launch.cpp", "red_launch.cpp", "ew_interp.hip", "ew_interleave.hip", "index.hip"]
           + [f"ew_slice_{i}.hip" for i in range(8)] + [f"red_slice_{i}.hip" for i in range(4)]
           + [f"fred_slice_{i}.hip" for i in range(4)])


def _stamp(src: str) -> str:
    """Fingerprint of everything an object depends on: its source, the files it includes and the
    flags."""
    import hashlib
    h = hashlib.sha256(" ".join(COMMON).encode())
    import re
    seen, todo = [], [os.path.join(CSRC, src)]
    while todo:                      # the files it includes with quotes, transitively
        path = os.path.normpath(todo.pop())
        if path in seen or not os.path.exists(path):
            continue
        seen.append(path)
        text = open(path, "rb").read()
        h.update(path.encode() + text)
        for inc in re.findall(rb'^\s*#\s*include\s+"([^"]+)"', text, flags=re.M):
            todo.append(os.path.join(os.path.dirname(path), inc.decode()))
    return h.hexdigest()


def _compile(src: str, force: bool = True) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    stamp_file, stamp = obj + ".stamp", _stamp(src)
    if not force and os.path.exists(obj) and os.path.exists(stamp_file) and open(stamp_file).read() == stamp:
        return obj
    cmd = [HIPCC, *COMMON, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    open(stamp_file, "w").write(stamp)
    return obj


def build(jobs: int | None = None, force: bool = True) -> str:
    """Compiles every source and links the library.  force=False recompiles only the objects
    whose source, headers or flags changed since they were last built."""
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(16, os.cpu_count() or 4)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda src: _compile(src, force), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--changed" not in sys.argv))
