"""The host-side layout code (stream offsets, tiling, the fused step's work list) built with
AddressSanitizer and UndefinedBehaviorSanitizer and driven with random layouts; the driver also
checks that tiles and work items cover the payload exactly once.  The XCD-aware order in which
workgroups take tiles is checked the same way: a permutation for every launch size."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_03644_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_layout_code_under_sanitizers(tmp_path):
    exe = str(tmp_path / "san_layout")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-I", CSRC,
           os.path.join(ROOT, "tests", "native", "san_layout.cpp"),
           os.path.join(CSRC, "layout.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_xcd_order_is_a_permutation(tmp_path):
    exe = str(tmp_path / "xcd_order_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-I", CSRC,
           os.path.join(ROOT, "tests", "native", "xcd_order_check.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok")
