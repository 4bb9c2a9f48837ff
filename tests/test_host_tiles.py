"""Builds (host only, no GPU) and runs the emulation of the tiled kernel's index arithmetic:
bounds of every access, each output written once, LDS slots and swizzle consistent."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_tiled_kernel_index_emulation(tmp_path):
    exe = tmp_path / "emulate_tiles"
    csrc = os.path.join(ROOT, "paper_1810_08723_amd", "csrc")
    cmd = [HIPCC, "--cuda-host-only", "-O1", "-std=c++17", "-Wno-unused-command-line-argument", "-o", str(exe),
           os.path.join(ROOT, "tests", "host", "emulate_tiles.hip"), os.path.join(csrc, "planner.cpp"),
           os.path.join(csrc, "ew_launch.cpp")]
    subprocess.run(cmd, check=True, capture_output=True)
    r = subprocess.run([str(exe), "6000"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:]
    assert r.stdout.startswith("ok:")
