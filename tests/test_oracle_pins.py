"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without the GPU.

Each test states which plausible mistake in `oracle/e4q_oracle.c` it would catch.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import exact_alg1 as ex

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16_bits_to_f64(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def true_loss_f64(oracle, table, codes, scale_bits, bias_bits):
    """Eq. 2 per row, re-measured in float64 from the emitted artefacts only."""
    xh = oracle.dequantize(codes, scale_bits, bias_bits, table.shape[1]).astype(np.float64)
    return ((table.astype(np.float64) - xh) ** 2).sum(axis=1)


# ----------------------------------------------------------------------------------------------
# binary16 conversion: the oracle's hand-written routine against NumPy's (an independent one).
# Catches: wrong tie rule, wrong subnormal shift, overflow handling.
# ----------------------------------------------------------------------------------------------
def test_f16_to_f32_all_bit_patterns(oracle_lib):
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle_lib.f16_bits_to_f32(bits)
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f32_to_f16_rne_against_numpy(oracle_lib):
    rng = np.random.default_rng(1)
    vals = [0.0, -0.0, 1.0, 65504.0, 65519.99, 65520.0, 70000.0, 1e-8, 2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), np.float32(1)),
            2.0 ** -24, 3 * 2.0 ** -25, 6.1e-5, 6.097e-5, np.inf, -np.inf]
    # every midpoint between neighbouring binary16 values (ties) and its float32 neighbours
    h = np.arange(0, 0x7BFF, 37, dtype=np.uint16).view(np.float16).astype(np.float64)
    hn = (np.arange(0, 0x7BFF, 37, dtype=np.uint16) + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((h + hn) / 2).astype(np.float32)
    vals = np.concatenate([np.array(vals, dtype=np.float32), mid, np.nextafter(mid, np.float32(0)),
                           np.nextafter(mid, np.float32(np.inf)), -mid,
                           (rng.standard_normal(4000) * 10.0 ** rng.uniform(-9, 5, 4000)).astype(np.float32)])
    got = oracle_lib.f32_to_f16_bits(vals)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)


# ----------------------------------------------------------------------------------------------
# P1. Eq. 1 on a row that already lies on a 16-point evenly spaced grid: codes are the grid
# indices, scale and bias are the grid's, dequantize returns the row bit for bit, loss is 0 and
# the greedy search (strict '<') keeps min/max.
# Catches: 2^n instead of 2^n - 1, swapped nibbles, bias/scale swapped, off-by-one clamp.
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("lo,s", [(-0.5, 0.0625), (3.0, 0.25), (-8.0, 1.0), (0.0, 2.0 ** -10)])
@pytest.mark.parametrize("dim", [16, 23, 64])
def test_exact_grid_is_reproduced(oracle_lib, lo, s, dim):
    rng = np.random.default_rng(dim)
    k = rng.integers(0, 16, size=(50, dim))
    k[:, 0], k[:, 1] = 0, 15
    k = rng.permuted(k, axis=1)
    table = (lo + k * s).astype(np.float32)
    codes, sc, bi, loss, ij = oracle_lib.quantize_rowwise_greedy(table, 200, 0.16, return_search=True)
    assert np.array_equal(oracle_lib.unpack_codes(codes, dim), k.astype(np.uint8))
    assert np.all(f16_bits_to_f64(sc) == s) and np.all(f16_bits_to_f64(bi) == lo)
    assert np.array_equal(oracle_lib.dequantize(codes, sc, bi, dim), table)
    assert np.all(loss == 0) and np.all(ij == 0)
    if dim % 2:  # the missing last nibble packs as 0
        assert np.all(codes[:, -1] >> 4 == 0)


def test_rounding_ties_go_to_even(oracle_lib):
    """round() in Eq. 1 is read as round-half-to-even.  Values exactly halfway between grid
    points of a power-of-two grid (everything exact in binary32) must take the even code."""
    k = np.arange(15)
    row = np.concatenate([[0.0, 15.0], k + 0.5]).astype(np.float32) * np.float32(0.125) - np.float32(2.0)
    codes, sc, bi = oracle_lib.quantize_rowwise_greedy(row[None, :], 200, 0.0)
    q = oracle_lib.unpack_codes(codes, row.size)[0]
    assert q[:2].tolist() == [0, 15]
    assert q[2:].tolist() == [int(np.rint(v + 0.5)) for v in k]  # 0.5->0, 1.5->2, 2.5->2, ...
    assert q[2:].tolist() == [0, 2, 2, 4, 4, 6, 6, 8, 8, 10, 10, 12, 12, 14, 14]


def test_nibble_order_and_row_bytes(oracle_lib):
    # element 0 -> low nibble of byte 0, element 1 -> high nibble
    row = np.arange(16, dtype=np.float32)[None, :]
    codes, sc, bi = oracle_lib.quantize_rowwise_greedy(row, 200, 0.0)
    assert codes.tolist() == [[0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]]
    assert codes.dtype == np.uint8 and sc.dtype == np.uint16 and bi.dtype == np.uint16


def test_table3_size_column(oracle_lib):
    """Bytes per row d/2 + 4 (packed codes + binary16 scale and bias) against the model-size
    percentages printed in Table 3 for GREEDY (FP16); the table's figures are truncated to two
    decimals and include the non-embedding 0.01 % of the model, hence the 0.011 allowance."""
    lines = [l.split() for l in open(os.path.join(GOLDEN, "table3_greedy_fp16_size_percent.txt"))
             if l.strip() and not l.startswith("#")]
    for d, pct in lines:
        d, pct = int(d), float(pct)
        table = np.random.default_rng(d).standard_normal((7, d)).astype(np.float32)
        codes, sc, bi = oracle_lib.quantize_rowwise_greedy(table)
        out_bytes = codes.nbytes + sc.nbytes + bi.nbytes
        assert out_bytes == 7 * (d // 2 + 4)
        assert abs(100.0 * out_bytes / table.nbytes - pct) <= 0.011


# ----------------------------------------------------------------------------------------------
# P7. With r = 0 the result is plain min/max affine quantization (ASYM, Section 2).  Checked
# against the real-number definition evaluated in float64: same codes away from rounding ties,
# and every reconstruction error within half a step (+ the binary16 rounding of the parameters).
# Catches: clipping applied when none is asked for, wrong rounding function (floor/trunc).
# ----------------------------------------------------------------------------------------------
def test_ratio_zero_is_textbook_minmax(oracle_lib):
    from paper_1911_02079_amd import synth

    table = synth.gaussian_table(300, 48, seed=5).numpy()
    codes, sc, bi, loss, ij = oracle_lib.quantize_rowwise_greedy(table, 200, 0.0, return_search=True)
    assert np.all(ij == 0)
    x = table.astype(np.float64)
    lo, hi = x.min(1, keepdims=True), x.max(1, keepdims=True)
    scale, bias = f16_bits_to_f64(sc)[:, None], f16_bits_to_f64(bi)[:, None]
    # stored parameters are the binary16 roundings of (max-min)/15 and min
    assert np.allclose(scale, (hi - lo) / 15, rtol=2.0 ** -11)
    assert np.allclose(bias, lo, rtol=2.0 ** -11)
    t = (x - bias) / scale
    q = oracle_lib.unpack_codes(codes, 48).astype(np.float64)
    near_tie = np.abs(t - np.floor(t) - 0.5) < 1e-4
    want = np.clip(np.rint(t), 0, 15)
    assert np.array_equal(q[~near_tie], want[~near_tie])
    assert np.all(np.abs(q - want) <= 1)
    xh = oracle_lib.dequantize(codes, sc, bi, 48).astype(np.float64)
    inside = (t >= 0) & (t <= 15)
    assert np.all(np.abs(x - xh)[inside] <= 0.5 * scale.repeat(48, 1)[inside] * (1 + 1e-5))
    # the search's float32 loss is the float64 loss of the artefacts up to float32 rounding
    assert np.allclose(loss, ((x - xh) ** 2).sum(1), rtol=1e-5)


def test_uniform_noise_model_sanity(oracle_lib):
    """For smooth data the error of min/max quantization is close to step^2/12 per element."""
    rng = np.random.default_rng(3)
    table = rng.uniform(-1, 1, size=(400, 128)).astype(np.float32)
    codes, sc, bi = oracle_lib.quantize_rowwise_greedy(table, 200, 0.0)
    mse = true_loss_f64(oracle_lib, table, codes, sc, bi) / 128
    model = f16_bits_to_f64(sc) ** 2 / 12
    assert 0.85 < np.mean(mse / model) < 1.15


# ----------------------------------------------------------------------------------------------
# P2 / P4. Greedy keeps the best of a set that contains min/max, and a longer search extends the
# same path: its loss never exceeds ASYM's and never increases with r.
# Catches: best-so-far not initialised with the starting loss, '>' for '<', literal bookkeeping.
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("maker", ["gauss", "outlier", "laplace"])
def test_never_worse_than_minmax_and_monotone_in_r(oracle_lib, maker):
    from paper_1911_02079_amd import synth

    table = {"gauss": lambda: synth.gaussian_table(400, 64, seed=11),
             "outlier": lambda: synth.outlier_table(400, 64, seed=12),
             "laplace": lambda: synth.laplace_offset_table(400, 128, seed=13)}[maker]().numpy()
    prev = None
    for r in [0.0, 0.05, 0.16, 0.3, 0.5]:
        codes, sc, bi, loss, ij = oracle_lib.quantize_rowwise_greedy(table, 200, r, return_search=True)
        assert np.all(ij.sum(1) <= oracle_lib.n_iter(200, r))
        if prev is not None:
            assert np.all(loss <= prev[0])  # exact, in the search's own arithmetic
            assert np.all(true_loss_f64(oracle_lib, table, codes, sc, bi) <= prev[1] * (1 + 1e-6))
        if r == 0.0:
            asym = (loss.copy(), true_loss_f64(oracle_lib, table, codes, sc, bi))
        prev = (loss, true_loss_f64(oracle_lib, table, codes, sc, bi))
        assert np.all(loss <= asym[0])
    # clipping must actually pay on these inputs (the paper's Table 2 shows an 8-13 % gain of
    # GREEDY over ASYM in normalized l2 on trained tables; synthetic rows give the same order)
    gain = 1 - np.sqrt(prev[1].sum() / asym[1].sum())
    assert gain > 0.05


def test_n_iter_is_ceil_b_times_r(oracle_lib):
    assert oracle_lib.n_iter(200, 0.16) == 32      # defaults of Algorithm 1
    assert oracle_lib.n_iter(100, 0.16) == 16
    assert oracle_lib.n_iter(1000, 0.5) == 500     # "GREEDY (opt)" of Fig. 1
    assert oracle_lib.n_iter(200, 0.0) == 0
    assert oracle_lib.n_iter(7, 0.5) == 4
    assert oracle_lib.n_iter(3, 0.999) == 2        # never more than b - 1 (range stays positive)


# ----------------------------------------------------------------------------------------------
# P3. Brute force over the whole (i, j) grid on tiny rows.
# Catches: a search that leaves the grid, a loss that is not Eq. 2, wrong step size.
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dim,b,r", [(4, 10, 0.5), (8, 20, 0.4), (16, 12, 0.9), (5, 16, 0.25)])
def test_brute_force_on_tiny_rows(oracle_lib, dim, b, r):
    rng = np.random.default_rng(dim * 100 + b)
    table = rng.standard_normal((60, dim)).astype(np.float32)
    table[::3] = rng.laplace(size=(20, dim)).astype(np.float32)
    n_it = oracle_lib.n_iter(b, r)
    codes, sc, bi, loss, ij = oracle_lib.quantize_rowwise_greedy(table, b, r, return_search=True)
    hit = 0
    for k in range(table.shape[0]):
        x = table[k]
        bl, bi_, bj_ = oracle_lib.brute_force_row(x, b, n_it)
        asym = oracle_lib.range_loss(x, x.min(), x.max())
        assert bl <= loss[k] <= asym
        # the greedy answer is a grid point and its loss is the loss of that grid point
        i, j = ij[k]
        assert i + j <= n_it
        step = np.float32((x.max() - x.min()) / np.float32(b))
        lo, hi = np.float32(x.min()), np.float32(x.max())
        for _ in range(i):
            lo = np.float32(lo + step)
        for _ in range(j):
            hi = np.float32(hi - step)
        assert oracle_lib.range_loss(x, lo, hi) == loss[k]
        assert sc[k] == np.float16(np.float32(hi - lo) / np.float32(15)).view(np.uint16)
        assert bi[k] == np.float16(lo).view(np.uint16)
        hit += bl == loss[k]
    assert hit >= 10  # the greedy path finds the grid optimum on a fair share of rows


# ----------------------------------------------------------------------------------------------
# Exact rational re-execution of Algorithm 1 on integer lattices (every float op exact there).
# Catches: wrong trip count (the while test of Algorithm 1 is evaluated exactly on that side),
# tie handling (strict '<': ties move the upper bound, keep the earlier best), a dropped term.
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dim,b,r,shift", [(8, 20, Fraction(2, 5), 0), (16, 200, Fraction(4, 25), 0),
                                           (16, 200, Fraction(4, 25), 3), (12, 50, Fraction(1, 2), 1),
                                           (7, 9, Fraction(1, 3), 2)])
@pytest.mark.parametrize("literal", [False, True])
def test_against_exact_rational_algorithm1(oracle_lib, dim, b, r, shift, literal):
    rng = np.random.default_rng(dim + b + shift)
    rows = [ex.lattice_row(rng, dim, b, shift) for _ in range(12)]
    table = np.stack(rows).astype(np.float32)
    codes, sc, bi, loss, ij = oracle_lib.quantize_rowwise_greedy(
        table, b, float(r), literal_alg1=literal, return_search=True)
    q = oracle_lib.unpack_codes(codes, dim)
    checked = 0
    for k, x in enumerate(rows):
        xmin, xmax, best, trips, biggest = ex.greedy([int(v) for v in x], b, r, literal)
        assert trips == oracle_lib.n_iter(b, float(r)) == math.ceil(b * r)
        assert biggest < 2 ** 24  # precondition: float32 sums were exact
        lo0, hi0 = int(x.min()), int(x.max())
        step = Fraction(hi0 - lo0, b)
        assert xmin == lo0 + ij[k, 0] * step and xmax == hi0 - ij[k, 1] * step
        assert Fraction(float(f16_bits_to_f64(bi[k]))) == xmin
        assert Fraction(float(f16_bits_to_f64(sc[k]))) == (xmax - xmin) / 15
        assert Fraction(float(loss[k])) == best
        want, ties, _ = ex.quantize([Fraction(int(v)) for v in x], xmin, xmax)
        for e in range(dim):
            if not ties[e]:
                assert q[k, e] == want[e]
                checked += 1
            else:
                assert abs(int(q[k, e]) - want[e]) <= 1
    assert checked > dim * len(rows) // 2


def test_literal_and_joint_bookkeeping_can_differ(oracle_lib):
    """The printed listing updates only the bound that moved; found by search, a row where that
    returns a pair whose own loss was never evaluated.  The oracle's default (joint) result must
    be the exact-arithmetic joint result, and the literal switch the exact literal one."""
    rng = np.random.default_rng(7)
    found = 0
    b, r = 200, Fraction(4, 25)
    for _ in range(60):
        x = ex.bell_lattice_row(rng, 16, b)
        a = ex.greedy([int(v) for v in x], b, r, literal=False)
        l = ex.greedy([int(v) for v in x], b, r, literal=True)
        assert a[4] < 2 ** 24
        if (a[0], a[1]) == (l[0], l[1]):
            continue
        found += 1
        t = x[None, :].astype(np.float32)
        for lit, want in ((False, a), (True, l)):
            _, sc, bi, _, _ = oracle_lib.quantize_rowwise_greedy(t, b, 0.16, literal_alg1=lit, return_search=True)
            assert Fraction(float(f16_bits_to_f64(bi[0]))) == want[0]
            assert Fraction(float(f16_bits_to_f64(sc[0]))) == (want[1] - want[0]) / 15
        # joint tracking returns a pair whose own loss is the best loss seen
        assert ex.loss([Fraction(int(v)) for v in x], a[0], a[1]) == a[2]
        if found >= 5:
            break
    assert found >= 1


# ----------------------------------------------------------------------------------------------
# P5. Scaling a row by a power of two scales scale and bias by it and leaves the codes alone
# (every operation of the method commutes with an exact scaling).
# Catches: an absolute epsilon or threshold hidden anywhere in the path.
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("k", [-6, -1, 3, 8])
def test_power_of_two_equivariance(oracle_lib, k):
    from paper_1911_02079_amd import synth

    table = synth.outlier_table(200, 32, seed=21).numpy()
    c0, s0, b0 = oracle_lib.quantize_rowwise_greedy(table)
    c1, s1, b1 = oracle_lib.quantize_rowwise_greedy((table * np.float32(2.0 ** k)).astype(np.float32))
    assert np.array_equal(c0, c1)
    normal = (np.abs(f16_bits_to_f64(s0)) * 2.0 ** min(k, 0) > 2.0 ** -14) & \
             (np.abs(f16_bits_to_f64(b0)) * 2.0 ** min(k, 0) > 2.0 ** -14)
    assert normal.mean() > 0.9
    assert np.array_equal(f16_bits_to_f64(s1)[normal], f16_bits_to_f64(s0)[normal] * 2.0 ** k)
    assert np.array_equal(f16_bits_to_f64(b1)[normal], f16_bits_to_f64(b0)[normal] * 2.0 ** k)


# ----------------------------------------------------------------------------------------------
# P6. Code range, extremes, degenerate rows.
# ----------------------------------------------------------------------------------------------
def test_code_range_and_extremes(oracle_lib):
    from paper_1911_02079_amd import synth

    table = synth.laplace_offset_table(500, 128, seed=31).numpy()
    codes, sc, bi = oracle_lib.quantize_rowwise_greedy(table)
    q = oracle_lib.unpack_codes(codes, 128)
    assert q.max() <= 15
    rows = np.arange(500)
    assert np.all(q[rows, table.argmin(1)] == 0) and np.all(q[rows, table.argmax(1)] == 15)


def test_constant_and_tiny_range_rows(oracle_lib):
    table = np.zeros((4, 10), dtype=np.float32)
    table[1] = 0.375
    table[2] = -7.0
    table[3] = 1.0
    table[3, 4] = np.float32(1.0) + np.float32(2.0 ** -23)  # range far below binary16 resolution
    codes, sc, bi, loss, ij = oracle_lib.quantize_rowwise_greedy(table, return_search=True)
    assert np.all(codes == 0) and np.all(sc == 0) and np.all(ij[:3] == 0)
    # row 3: every candidate stores the same (scale 0, bias 1.0) and so has the same loss; the
    # strict '<' of Algorithm 1 keeps the first one, the untouched min/max
    assert loss[3] > 0 and np.all(ij[3] == 0)
    assert np.array_equal(f16_bits_to_f64(bi), [0.0, 0.375, -7.0, 1.0])
    assert np.array_equal(oracle_lib.dequantize(codes, sc, bi, 10)[:3], table[:3])


def test_zero_bounds_are_positive_zero(oracle_lib):
    """-0 = +0, so "min X" does not say which zero a zero minimum is when a row holds both (Algorithm 1,
    lines 1-2, is silent): a zero bound is +0, wherever the zeros stand in the row.  Pinned on the stored
    bits: bias 0x0000, never 0x8000, and scale +0 for rows of nothing but zeros; the codes and the
    de-quantized values do not depend on the order of the zeros either."""
    nz, pz = np.float32(-0.0), np.float32(0.0)
    rows = np.array([
        [nz, pz, 1.0, 0.5, pz, nz, 0.25, 1.0],      # minimum zero, -0 first
        [pz, nz, 1.0, 0.5, nz, pz, 0.25, 1.0],      # the same numbers, +0 first
        [nz, nz, nz, nz, nz, nz, nz, nz],           # nothing but -0
        [nz, pz, nz, pz, nz, pz, nz, pz],           # zeros of both signs only
        [-1.0, nz, pz, -0.5, nz, -0.25, pz, -1.0],  # maximum zero
        [-1.0, pz, nz, -0.5, pz, -0.25, nz, -1.0],
    ], dtype=np.float32)
    for ratio in (0.0, 0.3):
        codes, sc, bi = oracle_lib.quantize_rowwise_greedy(rows, 20, ratio)[:3]
        assert np.array_equal(bi[:4], [0, 0, 0, 0])
        assert np.array_equal(sc[2:4], [0, 0])
        assert np.array_equal(codes[0], codes[1]) and sc[0] == sc[1]
        assert np.array_equal(codes[4], codes[5]) and sc[4] == sc[5] and bi[4] == bi[5]
        assert np.all(codes[2:4] == 0)
        xh = oracle_lib.dequantize(codes, sc, bi, 8)
        assert np.array_equal(xh[0], xh[1]) and np.array_equal(xh[4], xh[5])
        assert not np.signbit(xh[2:4]).any()


def test_summation_is_the_adjacent_pair_tree(oracle_lib):
    """Squared errors are summed by a balanced tree over index-adjacent pairs.  Built so that
    errors are known integers with squares near 2^24: then other orders (left to right,
    pairing k with k + d/2) give different float32 sums, and only the adjacent-pair tree
    matches."""
    rng = np.random.default_rng(0)
    d, scale = 64, 8192.0
    seen_other_orders_differ = False
    for _ in range(20):
        q = rng.integers(0, 16, d)
        q[0], q[1] = 0, 15
        e = rng.integers(-4000, 4001, d)
        e[0] = e[1] = 0
        x = (q * scale + e).astype(np.float32)
        s = (e.astype(np.float64) ** 2).astype(np.float32)

        def adjacent(v):
            v = v.copy()
            while v.size > 1:
                v = (v[0::2] + v[1::2]).astype(np.float32)
            return float(v[0])

        def halves(v):
            v = v.copy()
            while v.size > 1:
                h = v.size // 2
                v = (v[:h] + v[h:]).astype(np.float32)
            return float(v[0])

        def serial(v):
            acc = np.float32(0)
            for t in v:
                acc = np.float32(acc + t)
            return float(acc)

        got = oracle_lib.range_loss(x, 0.0, 15 * scale)
        assert got == adjacent(s)
        seen_other_orders_differ |= (halves(s) != got) or (serial(s) != got)
    assert seen_other_orders_differ
    # a row whose length is not a power of two is padded with zeros, which changes nothing
    x = np.concatenate([x[:40]])
    x[0], x[1] = 0.0, 15 * scale
    e40 = (x.astype(np.float64) - np.rint(x.astype(np.float64) / scale) * scale)
    s40 = np.zeros(64, dtype=np.float32)
    s40[:40] = (e40 ** 2).astype(np.float32)
    assert oracle_lib.range_loss(x, 0.0, 15 * scale) == adjacent(s40)


# ----------------------------------------------------------------------------------------------
# The separately written NumPy implementation agrees with the C oracle bit for bit.
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dim,b,r,literal", [(64, 200, 0.16, False), (24, 100, 0.16, False),
                                             (7, 30, 0.5, True), (128, 40, 0.3, False)])
def test_numpy_twin_bit_identical(oracle_lib, dim, b, r, literal):
    from oracle import numpy_twin
    from paper_1911_02079_amd import synth

    table = synth.outlier_table(24, dim, seed=40 + dim).numpy()
    table[3] = 0.25  # constant row
    got = oracle_lib.quantize_rowwise_greedy(table, b, r, literal_alg1=literal, return_search=True)
    want = numpy_twin.quantize_rowwise_greedy(table, b, r, literal_alg1=literal)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    # binary16 input is widened exactly
    t16 = table.astype(np.float16)
    got = oracle_lib.quantize_rowwise_greedy(t16, b, r, literal_alg1=literal, return_search=True)
    want = numpy_twin.quantize_rowwise_greedy(t16.astype(np.float32), b, r, literal_alg1=literal)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)


# ----------------------------------------------------------------------------------------------
# binary16 tables: widening is exact, so a binary16 table must give what the same values give as a
# binary32 table (NumPy's conversion feeds the binary32 side, which the pins above cover).
# Catches: binary16 rows read at the wrong pitch or offset, bit patterns read as integers.
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dim", [8, 37, 64, 128])
def test_binary16_tables_are_widened_exactly(oracle_lib, dim):
    from paper_1911_02079_amd import synth

    t16 = synth.outlier_table(40, dim, seed=70 + dim).numpy().astype(np.float16)
    t16[0, 0], t16[1, 1], t16[2, 2] = np.float16(6e-8), np.float16(-0.0), np.float16(-3e-6)
    got = oracle_lib.quantize_rowwise_greedy(t16, 200, 0.16, return_search=True)
    want = oracle_lib.quantize_rowwise_greedy(t16.astype(np.float32), 200, 0.16, return_search=True)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    assert len(np.unique(got[0])) > 8
    # and the exact-grid pin from a binary16 table: codes are the grid indices
    k = np.concatenate([np.arange(16), np.random.default_rng(dim).integers(0, 16, max(dim - 16, 0))])[None, :]
    grid = (-0.5 + k * 0.0625).astype(np.float16)
    codes, sc, bi = oracle_lib.quantize_rowwise_greedy(grid, 200, 0.16)
    assert np.array_equal(oracle_lib.unpack_codes(codes, k.shape[1])[:, : k.shape[1]], k.astype(np.uint8))
    assert f16_bits_to_f64(sc)[0] == 0.0625 and f16_bits_to_f64(bi)[0] == -0.5


# ----------------------------------------------------------------------------------------------
# Other bit widths through the same code: n = 8 is the paper's ASYM-8BITS baseline (Section 5),
# n = 2 the next power of two down.  2^n - 1 levels, 8/n codes per byte, lowest bits first.
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("nbits", [2, 8])
def test_other_bit_widths_exact_grid_and_packing(oracle_lib, nbits):
    levels = 2 ** nbits
    rng = np.random.default_rng(nbits)
    dim = 37
    k = rng.integers(0, levels, size=(20, dim))
    k[:, 0], k[:, 1] = 0, levels - 1
    k = rng.permuted(k, axis=1)
    lo, s = -2.0, 2.0 ** -6
    table = (lo + k * s).astype(np.float32)
    codes, sc, bi, loss, ij = oracle_lib.quantize_rowwise_greedy(table, 200, 0.16, return_search=True, nbits=nbits)
    per = 8 // nbits
    assert codes.shape == (20, (dim + per - 1) // per)
    assert np.array_equal(oracle_lib.unpack_codes(codes, dim, nbits), k.astype(np.uint8))
    assert np.all(f16_bits_to_f64(sc) == s) and np.all(f16_bits_to_f64(bi) == lo)
    assert np.array_equal(oracle_lib.dequantize(codes, sc, bi, dim, nbits), table)
    assert np.all(loss == 0) and np.all(ij == 0)
    # the byte layout, written out: first element in the lowest bits
    row = (np.arange(8) % levels).astype(np.float32)[None, :]
    row[0, 0], row[0, 7] = 0, levels - 1
    c, _, _ = oracle_lib.quantize_rowwise_greedy(row, 200, 0.0, nbits=nbits)
    q = row[0].astype(np.int64)
    if nbits == 8:
        assert c[0].tolist() == q.tolist()
    else:
        assert c[0].tolist() == [int(q[0] | q[1] << 2 | q[2] << 4 | q[3] << 6), int(q[4] | q[5] << 2 | q[6] << 4 | q[7] << 6)]


@pytest.mark.parametrize("nbits,b", [(2, 40), (8, 8)])
@pytest.mark.parametrize("literal", [False, True])
def test_other_bit_widths_against_exact_rational_algorithm1(oracle_lib, nbits, b, literal):
    levels = 2 ** nbits - 1
    rng = np.random.default_rng(nbits * 10 + b)
    r = Fraction(1, 4)
    rows = [ex.lattice_row(rng, 12, b, 0, levels=levels) for _ in range(10)]
    table = np.stack(rows).astype(np.float32)
    codes, sc, bi, loss, ij = oracle_lib.quantize_rowwise_greedy(table, b, float(r), literal_alg1=literal,
                                                                 return_search=True, nbits=nbits)
    q = oracle_lib.unpack_codes(codes, 12, nbits)
    for k, x in enumerate(rows):
        xmin, xmax, best, trips, biggest = ex.greedy([int(v) for v in x], b, r, literal, nbits)
        assert trips == oracle_lib.n_iter(b, float(r)) and biggest < 2 ** 24
        assert Fraction(float(f16_bits_to_f64(bi[k]))) == xmin
        assert Fraction(float(f16_bits_to_f64(sc[k]))) == (xmax - xmin) / levels
        assert Fraction(float(loss[k])) == best
        want, ties, _ = ex.quantize([Fraction(int(v)) for v in x], xmin, xmax, nbits)
        assert all(t or int(a) == w for a, w, t in zip(q[k], want, ties))


@pytest.mark.parametrize("nbits", [2, 8])
def test_other_bit_widths_invariants_and_twin(oracle_lib, nbits):
    from oracle import numpy_twin
    from paper_1911_02079_amd import synth

    table = synth.outlier_table(40, 24, seed=60 + nbits).numpy()
    got = oracle_lib.quantize_rowwise_greedy(table, 50, 0.3, return_search=True, nbits=nbits)
    want = numpy_twin.quantize_rowwise_greedy(table, 50, 0.3, nbits=nbits)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    asym = oracle_lib.quantize_rowwise_greedy(table, 50, 0.0, return_search=True, nbits=nbits)
    assert np.all(got[3] <= asym[3])
    assert oracle_lib.unpack_codes(got[0], 24, nbits).max() <= 2 ** nbits - 1
    for k in range(10):
        bl, _, _ = oracle_lib.brute_force_row(table[k], 50, oracle_lib.n_iter(50, 0.3), nbits)
        assert bl <= got[3][k]


def test_eight_bit_minmax_error_is_seventeen_times_smaller(oracle_lib):
    """Uniform-noise model: the step of n-bit min/max quantization is range/(2^n - 1), so the 8-bit
    error is 15/255 of the 4-bit one (Table 2: ASYM-8BITS 0.0026-0.0040 against ASYM 0.0445-0.0678)."""
    rng = np.random.default_rng(8)
    table = rng.uniform(-1, 1, size=(300, 128)).astype(np.float32)
    e = {}
    for nbits in (4, 8):
        codes, sc, bi = oracle_lib.quantize_rowwise_greedy(table, 200, 0.0, nbits=nbits)
        xh = oracle_lib.dequantize(codes, sc, bi, 128, nbits).astype(np.float64)
        e[nbits] = np.sqrt(((table - xh) ** 2).sum())
    assert 15.5 < e[4] / e[8] < 18.5
