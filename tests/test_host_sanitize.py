"""The host-only part of the library (the model planner of csrc/model.hip) compiled as plain C++ with the
library calls stubbed, under AddressSanitizer and UBSan: 2000 random models through create / describe /
step.  Needs g++ only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_model_planner_under_sanitizers(tmp_path):
    src = tmp_path / "model.cpp"
    text = open(os.path.join(ROOT, "paper_2602_02016_amd", "csrc", "model.hip")).read()
    src.write_text(text.replace('"../../include/dash.h"', '"dash.h"'))
    exe = tmp_path / "planner"
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "host", "planner_sanitize.cpp"), str(src), "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "sanitized planner ok" in r.stdout, (r.stdout[-500:], r.stderr[-2000:])


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_lds_layout_of_the_matmul_kernels(tmp_path):
    """csrc/lds_layout.h holds the index arithmetic both matmul kernels use for their direct loads and
    fragment reads.  tests/host/lds_layout_check.cpp emulates a whole operand slab with it on the host, for
    every tile size and both memory orders: every element lands once and where the MFMA operand reads expect
    it, nothing leaves the slab, no LDS bank conflicts.  Under AddressSanitizer and UBSan."""
    exe = tmp_path / "lds_layout_check"
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "paper_2602_02016_amd", "csrc"),
           os.path.join(ROOT, "tests", "host", "lds_layout_check.cpp"), "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "all layouts ok" in r.stdout, (r.stdout[-1500:], r.stderr[-2000:])
