#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X, through libe4q's C ABI.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload laplace_10M_x_128]

Default workload (the one the headline metric is quoted on): row-wise greedy 4-bit quantization
of a seeded synthetic 10 M x 128 fp32 table, then de-quantization of the result.  One "step" is
one pass of the whole path over the table, which is already resident in HBM: the quantizer (row
load, min/max, Algorithm 1's search, encode + pack, binary16 scale/bias) followed by the
de-quantizer.  `--workload mixture_2M_x_64_kmeans16` times the codebook variant the same way;
`--workload lookup_10M_x_128_sls` times the 4-bit SparseLengthsSum lookup over the quantized
table (2^20 bags of 1..64 uniformly random rows; bound by HBM gathers);
`--workload batch_26_half_tables` times the batch entry point on 26 binary16 tables.  `--rows`,
`--dim`, `--n-bins`, `--ratio`, `--half`, `--nbits` vary the single-table workloads (for example `--ratio 0`
is plain min/max quantization, which is bound by HBM instead of VALU issue).

Prints ONE JSON line.  `value` is rows per second over whole steps; `kernels` gives each kernel's
own average duration from HIP events recorded on the launch stream inside the timed region;
`roofline` prices the dominant kernel (bound by plain fp32 VALU issue); `cpu_baseline` is the CPU
oracle timed on this machine's host cores on a bounded sample of the same table.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X: 256 CUs x 4 SIMDs at 2.4 GHz; a SIMD retires a wave64 binary32 add, multiply or multiply-add
# in 2 clocks (32 lanes per clock, measured with plain, non-packed instructions), which is the
# data-sheet 157.3 TFLOP/s at 2 flops per multiply-add.  One lane-op = one such operation on one lane.
# Rounding, clamping, compares, selects, conversions and binary64 operations retire at half that rate,
# so a kernel whose mix contains them cannot reach 1.0 of this peak.
PEAK_LANE_OPS = 256 * 4 * 32 * 2.4e9
PEAK_HBM_BYTES = 8.0e12

WORKLOADS = {
    # name: (method, generator, rows, dim, parameters)
    "gaussian_10k_x_64": ("greedy", "gaussian_table", 10_000, 64, {"n_bins": 200, "ratio": 0.16}),
    "outlier_1M_x_64": ("greedy", "outlier_table", 1_000_000, 64, {"n_bins": 200, "ratio": 0.16}),
    "laplace_10M_x_128": ("greedy", "laplace_offset_table", 10_000_000, 128, {"n_bins": 200, "ratio": 0.16}),
    "mixture_2M_x_64_kmeans16": ("kmeans16", "mixture_table", 2_000_000, 64, {"lloyd_iters": 20}),
    "batch_26_half_tables": ("greedy_batch", "batch_tables", 9_416_736, 0, {"n_bins": 100, "ratio": 0.16}),
    "lookup_10M_x_128_sls": ("sls", "laplace_offset_table", 10_000_000, 128, {"n_bags": 1 << 20, "max_len": 64}),
}


def greedy_lane_ops_per_row(dim: int, n_iter: int) -> int:
    """fp32 lane operations the method itself needs per row: 8 per element per scored range
    (subtract, multiply, round, clamp, fused multiply-add, subtract, multiply, add) for the
    1 + 2*n_iter ranges of Algorithm 1, 2 per element for min/max, 6 per element for the final
    encode and pack."""
    return (1 + 2 * n_iter) * dim * 8 + 2 * dim + 6 * dim


def kmeans_lane_ops_per_row(dim: int, iters: int) -> int:
    """Lane operations of the 16-means path per row: per element and Lloyd round 16 subtractions,
    8 three-input minimums, 15 compares, 15 index selects and one binary64 add (55); one more
    assignment pass against the rounded codebook (54 per element); 16 means per round (counted as
    one operation each); 2 per element for min/max."""
    return dim * (55 * iters + 54) + 16 * iters + 2 * dim


def read_traffic(name: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE runs); the
    summary under profiles/ carries a line `traffic_bytes_per_launch: <int>`."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(table_gpu, run_oracle, target_seconds: float = 12.0):
    """Times the CPU oracle (as it stands) on a prefix of the same table, rows partitioned over
    the host cores available to this process (16 at most)."""
    import numpy as np

    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    rows = table_gpu.shape[0]
    probe = np.ascontiguousarray(table_gpu[: min(rows, 2048)].cpu().numpy())
    t0 = time.perf_counter()
    run_oracle(probe)
    per_row = (time.perf_counter() - t0) / probe.shape[0]
    sample_rows = int(min(rows, 4_000_000, max(cores * 64, target_seconds * cores / per_row)))
    sample = np.ascontiguousarray(table_gpu[:sample_rows].cpu().numpy())
    bounds = [sample_rows * k // cores for k in range(cores + 1)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:  # ctypes releases the GIL inside the C call
        list(pool.map(lambda k: run_oracle(sample[bounds[k]:bounds[k + 1]]), range(cores)))
    dt = time.perf_counter() - t0
    return {"value": sample_rows / dt, "unit": "rows/s", "cores": cores, "kind": "oracle",
            "sample": f"first {sample_rows} rows of the same table, rows split over {cores} threads, "
                      f"{dt:.1f} s wall; single-thread probe {1e6 * per_row:.1f} us/row"}


def bench_sls(args, e4q, synth, torch, gen, rows, dim, params) -> int:
    """The lookup operator on the quantized table: one step = one e4q_sparse_lengths_sum call."""
    import numpy as np

    table = getattr(synth, gen)(rows, dim, device="cuda:0")
    codes, scale, bias = e4q.quantize_rowwise_greedy(table, 200, 0.16)
    del table
    n_bags = params["n_bags"]
    indices, offsets = synth.lookup_bags(rows, n_bags, 1, params["max_len"], device="cuda:0")
    n_lookups = indices.numel()
    out = torch.empty((n_bags, dim), dtype=torch.float32, device="cuda:0")
    pitch = args.row_pitch or e4q.fused_row_bytes(dim)
    fused = e4q.fuse_rows(codes, scale, bias, dim, pitch)  # one-off re-layout of the table, not timed
    run = lambda: e4q.sparse_lengths_sum_fused(fused, dim, indices, offsets, out=out)  # noqa: E731

    def side_timing(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    # context, outside the timed region: the same lookup from the three separate arrays, and from
    # records padded to one 128-byte line each
    three_ms = side_timing(lambda: e4q.sparse_lengths_sum(codes, scale, bias, dim, indices, offsets, out=out))
    line_pitch = (e4q.fused_row_bytes(dim) + 127) // 128 * 128   # whole 128-byte lines per record
    fused128 = e4q.fuse_rows(codes, scale, bias, dim, line_pitch)
    line_ms = side_timing(lambda: e4q.sparse_lengths_sum_fused(fused128, dim, indices, offsets, out=out))
    fuse_ms = side_timing(lambda: e4q.fuse_rows(codes, scale, bias, dim, pitch, out=fused))
    del fused128
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        evs[k][0].record()
        run()
        evs[k][1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    # per looked-up row: d/2 bytes of codes, 2 + 2 bytes of parameters, 8 bytes of index;
    # per bag: 4d bytes of output and 8 bytes of offset
    alg_bytes = n_lookups * (dim // 2 + 4 + indices.element_size()) + n_bags * (4 * dim + 8)
    sums = n_lookups * dim
    result = {
        "metric": "billion sums/sec (INT4 SparseLengthsSum)", "value": sums / (elapsed / args.steps) / 1e9,
        "unit": "G sums/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "rows": rows, "dim": dim, "n_bags": n_bags, "lookups": n_lookups,
                   "bag_lengths": f"uniform 1..{params['max_len']}", "index_dtype": "int64",
                   "row_pitch": pitch, "nontemporal_gathers": bool(args.sls_nontemporal),
                   "step": f"sparse_lengths_sum_fused over all bags, fused records {pitch} bytes apart resident in HBM "
                           f"({rows * pitch / 1e6:.1f} MB)"},
        "kernels": {"sls_fused_w8_kernel": {"avg_ms": ms, "lookups_per_s": n_lookups / (ms * 1e-3),
                                            "G_sums_per_s": sums / (ms * 1e-3) / 1e9, "row_pitch": pitch},
                    f"sls_fused_w8_kernel (row_pitch {line_pitch})": {"avg_ms": line_ms},
                    "sls_w8_kernel (separate codes / scale / bias arrays)": {"avg_ms": three_ms},
                    "fuse_rows_w_kernel": {"avg_ms": fuse_ms}},
        "roofline": {"kernel": "sls_fused_w8_kernel", "bound": "hbm", "achieved": alg_bytes / (ms * 1e-3) / 1e9,
                     "peak": PEAK_HBM_BYTES / 1e9, "unit": "GB/s", "frac": alg_bytes / (ms * 1e-3) / PEAK_HBM_BYTES,
                     "bytes_per_lookup": dim // 2 + 4 + indices.element_size(), "bytes_per_bag": 4 * dim + 8,
                     "traffic": read_traffic(f"sls_fused_w8_kernel_{args.workload}_hbm_traffic.txt")
                     if not (args.row_pitch or args.sls_nontemporal or args.rows or args.dim) else None},
    }
    if not args.no_cpu_baseline:
        import oracle

        cores = max(1, min(16, len(os.sched_getaffinity(0))))
        sample_bags = min(n_bags, 262_144)
        off = offsets[: sample_bags + 1].cpu().numpy()
        idx = indices[: int(off[-1])].cpu().numpy()
        used, inv = np.unique(idx, return_inverse=True)
        sub = torch.from_numpy(used).cuda()
        s_codes = codes[sub].cpu().numpy()
        s_scale = scale[sub].cpu().view(torch.int16).numpy().view(np.uint16)
        s_bias = bias[sub].cpu().view(torch.int16).numpy().view(np.uint16)
        inv = inv.astype(np.int64)
        bounds = [sample_bags * k // cores for k in range(cores + 1)]

        def part(k):
            o = off[bounds[k]:bounds[k + 1] + 1]
            return oracle.sparse_lengths_sum(s_codes, s_scale, s_bias, dim, inv[o[0]:o[-1]], o - o[0])

        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as pool:
            list(pool.map(part, range(cores)))
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": int(off[-1]) * dim / dt / 1e9, "unit": "G sums/s", "cores": cores,
                                  "kind": "oracle", "sample": f"first {sample_bags} bags ({int(off[-1])} lookups) over "
                                  f"the rows they touch, bags split over {cores} threads, {dt:.2f} s wall"}
    print(json.dumps(result), flush=True)
    return 0


def bench_batch(args, e4q, synth, torch, params) -> int:
    """26 binary16 tables through the batch entry point: one step = one e4q_quantize_rowwise_greedy_batch call."""
    n_bins, ratio = args.n_bins or params["n_bins"], (args.ratio if args.ratio >= 0 else params["ratio"])
    n_iter = e4q.greedy_iterations(n_bins, ratio)
    specs = synth.batch_specs()
    tables = synth.batch_tables(specs, device="cuda:0")
    outs = [e4q.alloc_outputs(t.shape[0], t.shape[1], "cuda:0") for t in tables]
    run = lambda: e4q.quantize_rowwise_greedy_batch(tables, n_bins, ratio, out=outs)  # noqa: E731
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        evs[k][0].record()
        run()
        evs[k][1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    rows = sum(s.rows for s in specs)
    ops = sum(greedy_lane_ops_per_row(s.dim, n_iter) * s.rows for s in specs)
    nbytes = sum((2 * s.dim + s.dim // 2 + 4) * s.rows for s in specs)
    result = {
        "metric": "rows quantized/sec (greedy 4-bit)", "value": rows / (elapsed / args.steps), "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * elapsed / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "tables": len(specs), "rows": rows, "input": "binary16",
                   "dims": sorted({s.dim for s in specs}), "n_bins": n_bins, "ratio": ratio,
                   "step": "quantize_rowwise_greedy_batch over all tables (grouped launches per dimension)"},
        "kernels": {"greedy_rpl_group_kernel (all launches of a step)": {"avg_ms": ms, "rows_per_s": rows / (ms * 1e-3)}},
        "roofline": {"kernel": "greedy_rpl_group_kernel", "bound": "alu", "achieved": ops / (ms * 1e-3) / 1e12,
                     "peak": PEAK_LANE_OPS / 1e12, "unit": "T lane-op/s (fp32 VALU: 256 CU x 128 lanes x 2.4 GHz = 157.3 TFLOP/s / 2)",
                     "frac": ops / (ms * 1e-3) / PEAK_LANE_OPS, "hbm_achieved_GBps": nbytes / (ms * 1e-3) / 1e9,
                     "traffic": None},
    }
    print(json.dumps(result), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="laplace_10M_x_128", choices=sorted(WORKLOADS))
    ap.add_argument("--rows", type=int, default=0, help="override the workload's row count")
    ap.add_argument("--dim", type=int, default=0, help="override the workload's embedding dimension")
    ap.add_argument("--n-bins", type=int, default=0, help="override b of Algorithm 1")
    ap.add_argument("--ratio", type=float, default=-1.0, help="override r of Algorithm 1 (0 = plain min/max)")
    ap.add_argument("--half", action="store_true", help="feed the table as binary16")
    ap.add_argument("--nbits", type=int, default=4, choices=[2, 4, 8], help="code width of the uniform quantizer")
    ap.add_argument("--layout", default="auto",
                    help="thread layout of the greedy search: auto (the library's cost model), rpl (one row per "
                         "lane), E,L (L lanes per row, E elements each) or E,L,twin (two such groups per row, one per candidate "
                         "range of a trip), through the greedy_layout diagnostic option")
    ap.add_argument("--workgroup-waves", type=int, default=0, choices=[0, 1, 4],
                    help="waves per workgroup of the row-per-lane kernels (greedy search, 16-means), through the "
                         "workgroup_waves diagnostic option; 0: the library chooses by the row count")
    ap.add_argument("--row-pitch", type=int, default=0,
                    help="lookup workload: bytes between fused records (default: the smallest record, d/2 + 4)")
    ap.add_argument("--sls-nontemporal", action="store_true", help="lookup workload: non-temporal record gathers")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy kernel three times, so that a "
                         "rocprofv3 --pmc run can scale FETCH_SIZE / WRITE_SIZE by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (rows shard with no "
              "communication; run one process per GPU on its own row range).", file=sys.stderr)
        return 2

    import torch

    import paper_1911_02079_amd as e4q
    from paper_1911_02079_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    e4q.binding.load_library()
    torch.cuda.set_device(0)
    e4q.set_option("greedy_layout", e4q.greedy_layout_value(args.layout))
    e4q.set_option("workgroup_waves", args.workgroup_waves)
    e4q.set_option("sls_nontemporal", 1 if args.sls_nontemporal else 0)
    method, gen, rows, dim, params = WORKLOADS[args.workload]
    if method == "sls":
        return bench_sls(args, e4q, synth, torch, gen, args.rows or rows, args.dim or dim, params)
    if method == "greedy_batch":
        return bench_batch(args, e4q, synth, torch, params)
    rows, dim = args.rows or rows, args.dim or dim
    params = dict(params)
    if args.n_bins:
        params["n_bins"] = args.n_bins
    if args.ratio >= 0:
        params["ratio"] = args.ratio

    table = getattr(synth, gen)(rows, dim, device="cuda:0")
    if args.half:
        table = table.half()
    xh = torch.empty((rows, dim), dtype=torch.float32, device=table.device)
    if method == "greedy":
        n_bins, ratio = params["n_bins"], params["ratio"]
        n_iter = e4q.greedy_iterations(n_bins, ratio)
        nbits = args.nbits
        out = e4q.alloc_outputs(rows, dim, table.device, nbits)
        quantize = lambda: e4q.quantize_rowwise_greedy(table, n_bins, ratio, nbits=nbits, out=out)  # noqa: E731
        dequantize = lambda: e4q.dequantize(out[0], out[1], out[2], dim, nbits=nbits, out=xh)  # noqa: E731
        quantize()  # the library reports which thread layout it ran with
        torch.cuda.synchronize()
        chosen = e4q.get_option("greedy_layout_chosen")
        rpl = chosen == 1
        layout = e4q.greedy_layout_name(chosen)
        q_name, dq_name = ("greedy_rpl_kernel" if rpl else "greedy_swl_kernel"), "dequantize_w4_kernel"
        ops_per_row = greedy_lane_ops_per_row(dim, n_iter)
        out_bytes_per_row = e4q.packed_bytes(dim, nbits) + 4
        model_cycles = e4q.greedy_layout_cost(rows, dim, n_iter, chosen) if n_iter > 0 else None
        config = {"n_bins": n_bins, "ratio": ratio, "candidate_ranges_per_row": 1 + 2 * n_iter, "nbits": nbits,
                  "layout": layout, "layout_forced": args.layout != "auto", "workgroup_waves": args.workgroup_waves or "auto",
                  "layout_model_us": None if model_cycles is None else model_cycles / 2.4e3,
                  "step": "quantize_rowwise_greedy + dequantize, table resident in HBM"}
        metric = f"rows quantized/sec (greedy {nbits}-bit)"

        def run_oracle(t):
            import oracle
            return oracle.quantize_rowwise_greedy(t, n_bins, ratio, nbits=nbits)
    else:
        iters = params["lloyd_iters"]
        out = (torch.empty((rows, (dim + 1) // 2), dtype=torch.uint8, device=table.device),
               torch.empty((rows, 16), dtype=torch.float16, device=table.device))
        quantize = lambda: e4q.quantize_rowwise_kmeans16(table, iters, out=out)  # noqa: E731
        dequantize = lambda: e4q.dequantize_codebook(out[0], out[1], dim, out=xh)  # noqa: E731
        q_name, dq_name = "kmeans16_rpl_kernel", "dequantize_codebook_w4_kernel"
        ops_per_row = kmeans_lane_ops_per_row(dim, iters)
        out_bytes_per_row = (dim + 1) // 2 + 32
        config = {"lloyd_iters": iters, "codebook_entries": 16, "nbits": 4,
                  "step": "quantize_rowwise_kmeans16 + dequantize_codebook, table resident in HBM"}
        metric = "rows quantized/sec (16-means codebook, 4-bit)"

        def run_oracle(t):
            import oracle
            return oracle.quantize_rowwise_kmeans16(t, iters)
    torch.cuda.synchronize()

    def step(events=None):
        if events is not None:
            events[0].record()
        quantize()
        if events is not None:
            events[1].record()
        dequantize()
        if events is not None:
            events[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # events live on torch's current stream, which is the stream handed to the library
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=table.device)  # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)  # one plain copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    q_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    dq_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
    q_bytes = (dim * table.element_size() + out_bytes_per_row) * rows
    dq_bytes = (out_bytes_per_row + 4 * dim) * rows
    achieved = ops_per_row * rows / (q_ms * 1e-3)
    result = {
        "metric": metric,
        "value": rows / (elapsed / args.steps),
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": dict({"workload": args.workload, "rows": rows, "dim": dim,
                        "input": "binary16" if args.half else "binary32"}, **config),
        "kernels": {
            q_name: {"avg_ms": q_ms, "rows_per_s": rows / (q_ms * 1e-3),
                     "algorithmic_GBps": q_bytes / (q_ms * 1e-3) / 1e9},
            dq_name: {"avg_ms": dq_ms, "algorithmic_GBps": dq_bytes / (dq_ms * 1e-3) / 1e9,
                      "frac_of_hbm_peak": dq_bytes / (dq_ms * 1e-3) / PEAK_HBM_BYTES},
        },
        "roofline": {
            "kernel": q_name, "bound": "alu", "achieved": achieved / 1e12,
            "peak": PEAK_LANE_OPS / 1e12, "unit": "T lane-op/s (fp32 VALU: 256 CU x 128 lanes x 2.4 GHz = 157.3 TFLOP/s / 2)",
            "frac": achieved / PEAK_LANE_OPS,
            "lane_ops_per_row": ops_per_row,
            "bytes_per_row": q_bytes // rows,
            "hbm_achieved_GBps": q_bytes / (q_ms * 1e-3) / 1e9,
            "hbm_frac": q_bytes / (q_ms * 1e-3) / PEAK_HBM_BYTES,
            "traffic": read_traffic(f"{q_name}_{args.workload}_hbm_traffic.txt")
            if not (args.rows or args.dim or args.n_bins or args.ratio >= 0 or args.half or args.nbits != 4
                    or args.layout != "auto") else None,
        },
    }
    if method == "greedy" and n_iter == 0:  # plain min/max: one pass over the data, bound by HBM
        result["roofline"].update({"bound": "hbm", "achieved": q_bytes / (q_ms * 1e-3) / 1e9, "peak": PEAK_HBM_BYTES / 1e9,
                                   "unit": "GB/s", "frac": q_bytes / (q_ms * 1e-3) / PEAK_HBM_BYTES})
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(table, run_oracle)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
