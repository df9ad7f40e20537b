"""Second, separately written implementation of the oracle's greedy path in NumPy float32.

TEST INFRASTRUCTURE ONLY.  It exists so that a slip in the C oracle (an index, a
swapped operand, the hand-written binary16 conversion) shows up as a bit
difference on small tables: binary16 rounding here is NumPy's `astype(float16)`,
the fused multiply-add is emulated exactly in float64 (the product of a 4-bit
integer and a binary16 value plus a binary16 value is exact in float64), and the
loops are Python loops.  Slow: use on a few hundred rows at most.

Follows Eq. 1, Eq. 2 and Algorithm 1 of arXiv 1911.02079 with the same readings
as the C file (parameters rounded to binary16 before scoring, reciprocal
multiply, round-half-even, adjacent-pair summation tree, joint best tracking,
ceil(b*r) trips).
"""
from __future__ import annotations

import math

import numpy as np

F32 = np.float32


def _stored(lo: F32, hi: F32, qmax: float = 15.0):
    scale32 = F32(F32(hi - lo) / F32(qmax))
    return F32(np.float16(scale32)), F32(np.float16(lo))


def _codes_f32(x: np.ndarray, scale: F32, bias: F32, qmax: float = 15.0) -> np.ndarray:
    if scale == 0:
        return np.zeros_like(x)
    inv = F32(F32(1.0) / scale)
    t = ((x - bias).astype(F32) * inv).astype(F32)
    return np.clip(np.rint(t), F32(0), F32(qmax)).astype(F32)


def _pair_tree(s: np.ndarray) -> F32:
    p = 1
    while p < s.size:
        p *= 2
    v = np.zeros(p, dtype=F32)
    v[: s.size] = s
    while v.size > 1:
        v = (v[0::2] + v[1::2]).astype(F32)
    return F32(v[0])


def loss(x: np.ndarray, lo: F32, hi: F32, qmax: float = 15.0) -> F32:
    scale, bias = _stored(lo, hi, qmax)
    q = _codes_f32(x, scale, bias, qmax)
    # fmaf(q, scale, bias): q*scale + bias is exact in float64, one rounding to float32
    xh = (q.astype(np.float64) * np.float64(scale) + np.float64(bias)).astype(F32)
    e = (x - xh).astype(F32)
    return _pair_tree((e * e).astype(F32))


def greedy_row(x: np.ndarray, n_bins: int, ratio: float, literal_alg1: bool = False, qmax: float = 15.0):
    x = x.astype(F32)
    lo0, hi0 = F32(x.min()) + F32(0), F32(x.max()) + F32(0)   # a zero bound is +0 whichever zeros the row holds
    if lo0 == hi0:
        return lo0, hi0, F32(0), 0, 0
    br = float(n_bins) * float(F32(ratio))
    n_iter = int(min(max(math.ceil(br - br * 2.0 ** -22), 0), n_bins - 1))
    step = F32(F32(hi0 - lo0) / F32(n_bins))
    cur_lo, cur_hi, i, j = lo0, hi0, 0, 0
    best = [lo0, hi0, loss(x, lo0, hi0, qmax), 0, 0]
    for _ in range(n_iter):
        nlo, nhi = F32(cur_lo + step), F32(cur_hi - step)
        ll, lr = loss(x, nlo, cur_hi, qmax), loss(x, cur_lo, nhi, qmax)
        if ll < lr:
            cur_lo, i = nlo, i + 1
            if ll < best[2]:
                best[2], best[0], best[3] = ll, cur_lo, i
                if not literal_alg1:
                    best[1], best[4] = cur_hi, j
        else:
            cur_hi, j = nhi, j + 1
            if lr < best[2]:
                best[2], best[1], best[4] = lr, cur_hi, j
                if not literal_alg1:
                    best[0], best[3] = cur_lo, i
    return tuple(best)


def quantize_rowwise_greedy(table: np.ndarray, n_bins: int = 200, ratio: float = 0.16,
                            literal_alg1: bool = False, nbits: int = 4):
    rows, dim = table.shape
    qmax, per = float(2 ** nbits - 1), 8 // nbits
    nbytes = (dim + per - 1) // per
    codes = np.zeros((rows, nbytes), dtype=np.uint8)
    scale_bits = np.zeros(rows, dtype=np.uint16)
    bias_bits = np.zeros(rows, dtype=np.uint16)
    losses = np.zeros(rows, dtype=F32)
    ij = np.zeros((rows, 2), dtype=np.int32)
    for r in range(rows):
        x = table[r].astype(F32)
        lo, hi, l, i, j = greedy_row(x, n_bins, ratio, literal_alg1, qmax)
        scale, bias = _stored(lo, hi, qmax)
        scale_bits[r] = np.float16(scale).view(np.uint16)
        bias_bits[r] = np.float16(bias).view(np.uint16)
        q = np.zeros(nbytes * per, dtype=np.uint8)
        q[:dim] = _codes_f32(x, scale, bias, qmax).astype(np.uint8)
        for s_ in range(per):
            codes[r] |= q[s_::per] << (s_ * nbits)
        losses[r], ij[r, 0], ij[r, 1] = l, i, j
    return codes, scale_bits, bias_bits, losses, ij
