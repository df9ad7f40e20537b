"""bench.py's command line and the JSON line it prints.

CPU: more than one GPU is refused with a message; the help text lists the workloads.  GPU: a small workload
through the whole script (quantize + de-quantize steps, per-kernel HIP-event timings, roofline, oracle
baseline) and the keys of its one JSON line.
"""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def run_bench(*args, timeout=600):
    return subprocess.run([sys.executable, BENCH, *args], capture_output=True, text=True, timeout=timeout, cwd=ROOT)


def test_more_than_one_gpu_is_refused():
    res = run_bench("--gpus", "2")
    assert res.returncode != 0
    assert "one GPU" in (res.stdout + res.stderr)


def test_help_lists_the_workloads():
    res = run_bench("--help")
    assert res.returncode == 0
    for name in ("laplace_10M_x_128", "outlier_1M_x_64", "gaussian_10k_x_64", "batch_26_half_tables",
                 "mixture_2M_x_64_kmeans16", "lookup_10M_x_128_sls"):
        assert name in res.stdout


@pytest.mark.gpu
@pytest.mark.parametrize("args,kernel", [
    (["--workload", "gaussian_10k_x_64"], "greedy"),
    (["--workload", "mixture_2M_x_64_kmeans16", "--rows", "20000"], "kmeans16"),
    (["--workload", "lookup_10M_x_128_sls", "--rows", "50000"], "sls_fused"),
])
def test_json_line(args, kernel):
    res = run_bench(*args, "--steps", "3", "--warmup", "1")
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["value"] > 0 and d["ms_per_step"] > 0
    assert d["config"]["workload"] == args[1] and "model" not in d["config"]
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] in ("alu", "hbm") and 0 < roof["frac"] <= 1.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert any(kernel in name for name in d["kernels"])
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]


def test_committed_traffic_figures_are_present_and_plausible():
    """bench.py reports `roofline.traffic` from the counter summaries under profiles/ (counters cannot be read inside
    the timed run): the three default workloads' summaries must carry the figure, and it must lie between the
    algorithmic bytes per launch and the share of re-reads the design document accounts for."""
    import importlib.util

    spec = importlib.util.spec_from_file_location("bench_module", BENCH)
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    greedy = bench.read_traffic("greedy_rpl_kernel_laplace_10M_x_128_hbm_traffic.txt")
    assert greedy is not None and 1.0 <= greedy / (10_000_000 * 580) < 1.01       # every row read once, codes written once
    kmeans = bench.read_traffic("kmeans16_rpl_kernel_mixture_2M_x_64_kmeans16_hbm_traffic.txt")
    assert kmeans is not None and 1.0 <= kmeans / (2_000_000 * 320) < 1.01
    lookup = bench.read_traffic("sls_fused_w8_kernel_lookup_10M_x_128_sls_hbm_traffic.txt")
    algorithmic = 34_093_552 * 76 + (1 << 20) * 520
    assert lookup is not None and 2.0 < lookup / algorithmic < 3.0                 # 128-byte line fills on 68-byte records
