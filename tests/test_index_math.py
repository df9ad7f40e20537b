"""The kernels' thread-number arithmetic at the 2^32 boundary, checked on the CPU.

`paper_1911_02079_amd/csrc/e4q_index.h` holds the functions the de-quantizers and the lookup kernels
use to turn a 64-bit thread number into (row, position) or (bag, word); they are host-callable, so
`tests/index_math_check.hip` is compiled with hipcc (no GPU needed) and run here.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC) and shutil.which("hipcc") is None, reason="hipcc not found")
def test_index_arithmetic_around_2_pow_32(tmp_path):
    exe = tmp_path / "index_math_check"
    cmd = [HIPCC if os.path.exists(HIPCC) else "hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17",
           "-Wno-unused-command-line-argument", os.path.join(ROOT, "tests", "index_math_check.hip"), "-o", str(exe)]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-2000:]
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-500:]
    assert "0 failures" in run.stdout
