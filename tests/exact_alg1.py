"""Algorithm 1, Eq. 1 and Eq. 2 of arXiv 1911.02079 in exact rational arithmetic.

A pin for the oracle that shares nothing with it: Python `Fraction`s, no rounding
anywhere except the round() of Eq. 1 itself, and Algorithm 1's search written as a
walk over integer lattice coordinates with its stopping test evaluated exactly.  On inputs built so that every
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
    """The search of Algorithm 1 as a walk on the lattice of clipping ranges.

    Node (i, j) is the range [lowest + i*w, highest - j*w] with w = (highest - lowest)/b, so its
    width is (b - i - j)*w.  The walk starts at (0, 0) and, while the width of the node it stands
    on still exceeds b*(1 - r)*w (Algorithm 1's stopping test, here stated on the width and
    evaluated exactly; a row of equal values has w = 0 and never moves), scores the two
    neighbours (i + 1, j) and (i, j + 1) with Eq. 2 and steps to the one whose error is strictly
    smaller, to (i, j + 1) on a tie.  The answer is the node with the smallest error met, the
    earliest one among equals.  `literal=True` keeps the printed bookkeeping instead: an
    improvement found by raising the lower bound records only i, one found by lowering the
    upper bound records only j, and the answer combines the two records.
    Returns (xmin, xmax, error of the best node, moves made, largest error evaluated)."""
    X = [Fraction(x) for x in X]
    lowest, highest = min(X), max(X)
    w = (highest - lowest) / b

    def node_error(i, j):
        return loss(X, lowest + i * w, highest - j * w, nbits)

    i = j = 0
    keep_i = keep_j = 0
    smallest = largest = node_error(0, 0)
    moves = 0
    while (b - i - j) * w > b * (1 - r) * w:
        moves += 1
        up, down = node_error(i + 1, j), node_error(i, j + 1)
        largest = max(largest, up, down)
        if up < down:
            i += 1
            if up < smallest:
                smallest, keep_i = up, i
                if not literal:
                    keep_j = j
        else:
            j += 1
            if down < smallest:
                smallest, keep_j = down, j
                if not literal:
                    keep_i = i
    return lowest + keep_i * w, highest - keep_j * w, smallest, moves, largest


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
