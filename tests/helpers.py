"""Helpers shared by the GPU tests (no quantization arithmetic here)."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np


def oracle_rows_in_parallel(oracle, table: np.ndarray, n_bins: int, ratio: float, threads: int = 0, nbits: int = 4):
    """The CPU oracle on a large table: rows split over host threads (the C call releases the GIL),
    results concatenated.  Rows are independent, so this is the oracle's result exactly."""
    threads = threads or max(1, min(16, len(os.sched_getaffinity(0))))
    rows = table.shape[0]
    bounds = [rows * k // threads for k in range(threads + 1)]
    with ThreadPoolExecutor(max_workers=threads) as pool:
        parts = list(pool.map(lambda k: oracle.quantize_rowwise_greedy(table[bounds[k]:bounds[k + 1]], n_bins, ratio, nbits=nbits),
                              range(threads)))
    return tuple(np.concatenate([p[i] for p in parts]) for i in range(3))


def f16_bits(t):
    """uint16 bit patterns of a float16 torch tensor, on the host."""
    import torch

    return t.cpu().view(torch.int16).numpy().view(np.uint16)


def oracle_kmeans_in_parallel(oracle, table: np.ndarray, lloyd_iters: int, threads: int = 0):
    """The codebook oracle on a large table, rows split over host threads."""
    threads = threads or max(1, min(16, len(os.sched_getaffinity(0))))
    rows = table.shape[0]
    bounds = [rows * k // threads for k in range(threads + 1)]
    with ThreadPoolExecutor(max_workers=threads) as pool:
        parts = list(pool.map(lambda k: oracle.quantize_rowwise_kmeans16(table[bounds[k]:bounds[k + 1]], lloyd_iters),
                              range(threads)))
    return tuple(np.concatenate([p[i] for p in parts]) for i in range(2))
