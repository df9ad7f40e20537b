"""Builds libe4q.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_1911_02079_amd.build

hipcc cross-compiles without a GPU.  The flags matter for correctness, not only speed:
`-ffp-contract=off` (nothing is fused unless the source says fma) and correctly rounded
division are part of the arithmetic contract that makes results reproducible bit for bit;
packed-FP32 instruction selection is switched off.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libe4q.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

SOURCES = ["e4q_api.hip", "greedy_rpl_f32.hip", "greedy_rpl_f16.hip", "greedy_rpl_tail_f32.hip", "greedy_rpl_tail_f16.hip", "greedy_rpl_wide_f32.hip", "greedy_rpl_wide_f16.hip", "greedy_rpl_wide_tail_f32.hip", "greedy_rpl_wide_tail_f16.hip", "greedy_swl_f32_small.hip", "greedy_swl_f32_mid.hip",
           "greedy_swl_f32_big.hip", "greedy_swl_f16_small.hip", "greedy_swl_f16_mid.hip", "greedy_swl_f16_big.hip", "greedy_swl_any_f32.hip", "greedy_swl_any_f16.hip", "dequantize.hip", "kmeans16_f32.hip",
           "kmeans16_f16.hip", "kmeans16_tail_f32.hip", "kmeans16_tail_f16.hip", "kmeans16_misc.hip", "sls.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass does not know the AMDGPU feature name and says so; that is harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(jobs: int = 8) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(_compile, SOURCES))
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], check=True)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library())
