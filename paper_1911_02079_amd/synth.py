"""Seeded synthetic embedding tables.

This module only draws random inputs; it holds none of the quantization
arithmetic and is the one piece of code that both the HIP path's tests and the
CPU oracle's tests use.  The tables stand in for the trained recommendation
tables of the paper's experiments (Section 5: up to 50 M rows, embedding
dimension 8 to 128), which are not available here: same shapes, value
distributions chosen to exercise the clipping search (Gaussian rows, rows with
heavy-tailed outliers, Laplace rows with a per-row offset, a mixed batch of
half-precision tables, Gaussian-mixture rows for the codebook variant).

Every generator takes a `device` ("cpu" or "cuda") and a seed, draws with a
`torch.Generator` on that device, and returns a torch tensor on that device.
The CPU and GPU generators of torch produce different streams for one seed, so
a table is always drawn once and then shared (copied) between the two sides.
Large tables are drawn in row chunks so that temporaries stay small.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List

import numpy as np
import torch

BASE_SEED = 19110207
_CHUNK_ELEMS = 1 << 26  # 64 Mi elements of temporaries at a time


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _row_chunks(rows: int, dim: int):
    step = max(1, _CHUNK_ELEMS // max(dim, 1))
    for r0 in range(0, rows, step):
        yield r0, min(rows, r0 + step)


def _laplace(shape, scale, g: torch.Generator, device) -> torch.Tensor:
    """Laplace(0, scale) by inverse CDF from U(-1/2, 1/2); `scale` broadcasts."""
    u = torch.rand(shape, generator=g, device=device, dtype=torch.float32) - 0.5
    # clamp keeps log() finite when u hits -0.5 exactly
    mag = -torch.log(torch.clamp(1.0 - 2.0 * u.abs(), min=1e-30))
    return torch.sign(u) * mag * scale


def gaussian_table(rows: int = 10_000, dim: int = 64, sigma: float = 0.1, seed: int = BASE_SEED,
                   device="cpu", dtype=torch.float32) -> torch.Tensor:
    """Entries i.i.d. N(0, sigma^2) (sigma is the standard deviation)."""
    g = _gen(device, seed)
    out = torch.empty((rows, dim), device=device, dtype=dtype)
    for r0, r1 in _row_chunks(rows, dim):
        out[r0:r1] = (torch.randn((r1 - r0, dim), generator=g, device=device) * sigma).to(dtype)
    return out


def outlier_table(rows: int = 1_000_000, dim: int = 64, seed: int = BASE_SEED + 1, device="cpu",
                  outlier_frac: float = 0.02) -> torch.Tensor:
    """Row r is N(0, sigma_r^2) with sigma_r ~ LogNormal(ln 0.05, 0.5); each entry is replaced,
    independently with probability `outlier_frac`, by a Laplace(0, 10 sigma_r) draw."""
    g = _gen(device, seed)
    out = torch.empty((rows, dim), device=device, dtype=torch.float32)
    for r0, r1 in _row_chunks(rows, dim):
        n = r1 - r0
        sigma = 0.05 * torch.exp(0.5 * torch.randn((n, 1), generator=g, device=device))
        body = torch.randn((n, dim), generator=g, device=device) * sigma
        mask = torch.rand((n, dim), generator=g, device=device) < outlier_frac
        heavy = _laplace((n, dim), 10.0 * sigma, g, device)
        out[r0:r1] = torch.where(mask, heavy, body)
    return out


def laplace_offset_table(rows: int = 10_000_000, dim: int = 128, seed: int = BASE_SEED + 2,
                         device="cpu", b: float = 0.05, offset: float = 0.1) -> torch.Tensor:
    """Entries Laplace(0, b) plus a per-row offset ~ U(-offset, offset)."""
    g = _gen(device, seed)
    out = torch.empty((rows, dim), device=device, dtype=torch.float32)
    for r0, r1 in _row_chunks(rows, dim):
        n = r1 - r0
        mu = (torch.rand((n, 1), generator=g, device=device) * 2.0 - 1.0) * offset
        out[r0:r1] = _laplace((n, dim), b, g, device) + mu
    return out


@dataclass
class TableSpec:
    rows: int
    dim: int
    sigma: float
    seed: int


def batch_specs(n_tables: int = 26, seed: int = BASE_SEED + 3, min_rows: int = 1_000,
                max_rows: int = 5_000_000) -> List[TableSpec]:
    """Shapes of the mixed batch: rows log-uniform in [min_rows, max_rows], dim from
    {32, 64, 128}, per-table sigma ~ U(0.01, 0.2).  Drawn with NumPy on the host so that the
    shapes are the same wherever the tables themselves are drawn."""
    rs = np.random.RandomState(seed)
    specs = []
    for t in range(n_tables):
        rows = int(round(math.exp(rs.uniform(math.log(min_rows), math.log(max_rows)))))
        dim = int(rs.choice([32, 64, 128]))
        sigma = float(rs.uniform(0.01, 0.2))
        specs.append(TableSpec(rows=rows, dim=dim, sigma=sigma, seed=seed + 1000 + t))
    return specs


def batch_tables(specs: List[TableSpec], device="cpu") -> List[torch.Tensor]:
    """Half-precision N(0, sigma_t^2) tables for `specs`."""
    return [gaussian_table(s.rows, s.dim, s.sigma, s.seed, device, torch.float16) for s in specs]


def mixture_table(rows: int = 2_000_000, dim: int = 64, seed: int = BASE_SEED + 4, device="cpu",
                  n_comp: int = 3, sigma: float = 0.02, mean_range: float = 0.3) -> torch.Tensor:
    """Each row draws `n_comp` component means ~ U(-mean_range, mean_range); each entry picks a
    component uniformly and adds N(0, sigma^2)."""
    g = _gen(device, seed)
    out = torch.empty((rows, dim), device=device, dtype=torch.float32)
    for r0, r1 in _row_chunks(rows, dim):
        n = r1 - r0
        means = (torch.rand((n, n_comp), generator=g, device=device) * 2.0 - 1.0) * mean_range
        comp = torch.randint(0, n_comp, (n, dim), generator=g, device=device)
        out[r0:r1] = torch.gather(means, 1, comp) + torch.randn((n, dim), generator=g, device=device) * sigma
    return out


def lookup_bags(rows: int, n_bags: int = 1 << 20, min_len: int = 1, max_len: int = 64, seed: int = BASE_SEED + 5,
                device="cpu", index_dtype=torch.int64):
    """Index stream of a pooled embedding lookup: bag lengths uniform in [min_len, max_len], row
    numbers uniform over the table (no locality: the cache non-resident case of the paper's
    Table 1).  Returns (indices [sum of lengths], offsets int64 [n_bags + 1])."""
    g = _gen(device, seed)
    lengths = torch.randint(min_len, max_len + 1, (n_bags,), generator=g, device=device)
    offsets = torch.zeros(n_bags + 1, dtype=torch.int64, device=device)
    offsets[1:] = torch.cumsum(lengths, 0)
    total = int(offsets[-1])
    indices = torch.randint(0, rows, (total,), generator=g, device=device).to(index_dtype)
    return indices, offsets
