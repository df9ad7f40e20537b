"""Algorithm 1, Eq. 1 and Eq. 2 of arXiv 1911.02079 in exact rational arithmetic.

A pin for the oracle that shares nothing with it: Python `Fraction`s, no rounding
anywhere except the round() of Eq. 1 itself, and the while-loop of Algorithm 1
with its own stopping test (evaluated exactly).  On inputs built so that every
floating-point operation of the oracle is exact (integer lattices, see
`lattice_row`), oracle and this file must agree on the returned range, on the
loss and on every non-tie code.
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np

HALF = Fraction(1, 2)


def round_half_even(v: Fraction) -> int:
    fl = math.floor(v)
    rem = v - fl
    if rem > HALF:
        return fl + 1
    if rem < HALF:
        return fl
    return fl if fl % 2 == 0 else fl + 1


def quantize(X, xmin: Fraction, xmax: Fraction, nbits: int = 4):
    """x_int of Eq. 1 for each x clipped to [xmin, xmax]; also flags exact rounding ties."""
    levels = 2 ** nbits - 1
    scale = (xmax - xmin) / levels
    codes, ties = [], []
    for x in X:
        if scale == 0:
            codes.append(0)
            ties.append(False)
            continue
        xc = min(max(x, xmin), xmax)
        t = (xc - xmin) / scale
        codes.append(round_half_even(t))
        ties.append((t - math.floor(t)) == HALF)
    return codes, ties, scale


def loss(X, xmin: Fraction, xmax: Fraction, nbits: int = 4) -> Fraction:
    """Eq. 2: squared l2 distance between X and its quantize->dequantize image."""
    codes, _, scale = quantize(X, xmin, xmax, nbits)
    return sum(((x - (scale * q + xmin)) ** 2 for x, q in zip(X, codes)), Fraction(0))


def greedy(X, b: int, r: Fraction, literal: bool = False, nbits: int = 4):
    """Algorithm 1.  `literal=False` stores the pair (cur_min, cur_max) with every improvement;
    `literal=True` updates only the bound that moved, as the printed listing does.
    Returns (xmin, xmax, loss, n_trips, largest loss evaluated)."""
    X = [Fraction(x) for x in X]
    xmin = cur_min = min(X)
    xmax = cur_max = max(X)
    best = loss(X, xmin, xmax, nbits)
    stepsize = (xmax - xmin) / b
    min_steps = b * (1 - r) * stepsize
    trips, biggest = 0, best
    while cur_min + min_steps < cur_max:
        trips += 1
        loss_l = loss(X, cur_min + stepsize, cur_max, nbits)
        loss_r = loss(X, cur_min, cur_max - stepsize, nbits)
        biggest = max(biggest, loss_l, loss_r)
        if loss_l < loss_r:
            cur_min = cur_min + stepsize
            if loss_l < best:
                best, xmin = loss_l, cur_min
                if not literal:
                    xmax = cur_max
        else:
            cur_max = cur_max - stepsize
            if loss_r < best:
                best, xmax = loss_r, cur_max
                if not literal:
                    xmin = cur_min
    return xmin, xmax, best, trips, biggest


def lattice_row(rng: np.random.Generator, d: int, b: int, shift: int = 0, outliers: int = 2,
                levels: int = 15) -> np.ndarray:
    """Integer-valued row whose range is exactly levels*b*2^shift (levels = 2^n - 1), centred near zero.

    Then stepsize = 15*2^shift, every candidate bound is an integer, every candidate scale
    (b - i - j)*2^shift is an integer with at most 11 significant bits, and all errors are
    integers: binary16 storage of scale and bias and every binary32 operation of the loss are
    exact as long as the losses stay below 2^24 (the caller checks that)."""
    unit = 1 << shift
    span = levels * b * unit
    lo = -(span // 2 // unit) * unit
    hi = lo + span
    # bulk of the row in the inner part of the range, a few points out at the ends
    inner_lo, inner_hi = lo + span // 4, hi - span // 4
    x = rng.integers(inner_lo // unit, inner_hi // unit + 1, size=d) * unit
    pos = rng.permutation(d)
    x[pos[0]], x[pos[1]] = lo, hi
    for k in range(outliers):
        if 2 + k < d:
            x[pos[2 + k]] = rng.integers(lo // unit, hi // unit + 1) * unit
    return x.astype(np.int64)


def bell_lattice_row(rng: np.random.Generator, d: int, b: int) -> np.ndarray:
    """Integer row with range exactly 15*b whose values cluster around the middle (rounded normal
    draws): the loss along the greedy path is bumpy there, which is what separates the two
    bookkeeping readings of Algorithm 1."""
    span = 15 * b
    lo = -(span // 2)
    x = np.clip(np.rint(rng.standard_normal(d) * span / 6).astype(np.int64), lo, lo + span)
    x[0], x[1] = lo, lo + span
    return x
