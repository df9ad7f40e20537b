"""Pins for the codebook (row-wise 16-means) part of the CPU oracle."""
import os

import numpy as np
import pytest

import exact_lloyd

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16_to_f64(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def objective(x, centres):
    """Lloyd's objective: sum over values of the squared distance to the nearest centre (float64)."""
    d = (x[:, :, None].astype(np.float64) - centres[:, None, :].astype(np.float64)) ** 2
    return d.min(axis=2).sum(axis=1)


def test_populated_16_point_grid_is_a_fixed_point(oracle_lib):
    """Every grid point of min + k*step occupied: each cluster holds copies of one value, the means
    are those values, nothing moves; codebook, indices and reconstruction are exact.
    Catches: 16 instead of 15 grid intervals, off-by-one in the index, swapped nibbles."""
    rng = np.random.default_rng(0)
    for lo, s, dim in [(-2.0, 0.25, 64), (0.5, 2.0 ** -6, 33), (-8.0, 1.0, 128)]:
        k = np.concatenate([np.arange(16), rng.integers(0, 16, dim - 16)])
        k = np.stack([rng.permutation(k) for _ in range(20)])
        table = (lo + k * s).astype(np.float32)
        idx, cb, c32 = oracle_lib.quantize_rowwise_kmeans16(table, 20, return_centres=True)
        assert np.array_equal(oracle_lib.unpack_codes(idx, dim), k.astype(np.uint8))
        assert np.all(f16_to_f64(cb) == lo + np.arange(16) * s)
        assert np.array_equal(oracle_lib.dequantize_codebook(idx, cb, dim), table)
        if dim % 2:
            assert np.all(idx[:, -1] >> 4 == 0)


def test_equal_distances_take_the_lower_index(oracle_lib):
    """Zero Lloyd rounds: the codebook is the min/max grid itself; a value exactly halfway between
    two grid points goes to the lower one.  Catches '<=' in the nearest-centre scan."""
    grid = np.arange(16) * 0.25 - 2.0
    mids = (np.arange(15) + 0.5) * 0.25 - 2.0
    row = np.concatenate([grid, mids, [0.0]]).astype(np.float32)[None, :]
    idx, cb = oracle_lib.quantize_rowwise_kmeans16(row, 0)
    q = oracle_lib.unpack_codes(idx, 32)[0]
    assert q[:16].tolist() == list(range(16))
    assert q[16:31].tolist() == list(range(15))
    assert np.all(f16_to_f64(cb)[0] == grid)


def test_small_dimensions_are_lossless_up_to_binary16(oracle_lib):
    """dim <= 16: every value is its own codebook entry (Table 2 prints loss 0 for d = 8 and 16)."""
    rng = np.random.default_rng(1)
    for dim in (1, 5, 8, 15, 16):
        table = rng.standard_normal((30, dim)).astype(np.float32)
        idx, cb = oracle_lib.quantize_rowwise_kmeans16(table, 20)
        assert np.array_equal(oracle_lib.unpack_codes(idx, dim), np.tile(np.arange(dim, dtype=np.uint8), (30, 1)))
        want = table.astype(np.float16).astype(np.float32)
        assert np.array_equal(oracle_lib.dequantize_codebook(idx, cb, dim), want)
        assert np.all(cb[:, dim:] == 0)


def test_table3_codebook_size_column(oracle_lib):
    """d/2 bytes of indices + 16 binary16 codebook entries per row against the KMEANS (FP16) sizes
    printed in Table 3."""
    for line in open(os.path.join(GOLDEN, "table3_kmeans_fp16_size_percent.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        d, pct = int(line.split()[0]), float(line.split()[1])
        table = np.random.default_rng(d).standard_normal((5, d)).astype(np.float32)
        idx, cb = oracle_lib.quantize_rowwise_kmeans16(table, 2)
        assert idx.nbytes + cb.nbytes == 5 * (d // 2 + 32)
        assert abs(100.0 * (idx.nbytes + cb.nbytes) / table.nbytes - pct) <= 0.011


@pytest.mark.parametrize("maker", ["mixture", "gauss", "outlier"])
def test_lloyd_objective_never_increases(oracle_lib, maker):
    """Each Lloyd round can only lower the objective; round 0 is the min/max (ASYM) grid, so the
    codebook is never worse than uniform min/max quantization with unrounded parameters.
    Catches: a wrong update (median, sum without division), an assignment that is not the nearest."""
    from paper_1911_02079_amd import synth

    table = {"mixture": lambda: synth.mixture_table(150, 64, seed=3),
             "gauss": lambda: synth.gaussian_table(150, 128, seed=4),
             "outlier": lambda: synth.outlier_table(150, 40, seed=5)}[maker]().numpy()
    prev = None
    for rounds in range(0, 21):
        _, _, c32 = oracle_lib.quantize_rowwise_kmeans16(table, rounds, return_centres=True)
        j = objective(table, c32)
        if prev is not None:
            assert np.all(j <= prev * (1 + 1e-6) + 1e-12)
        else:
            first = j
        prev = j
    assert prev.sum() < 0.85 * first.sum()  # clustering pays (Table 2: 0.0578 vs 0.0678 normalized l2 at d = 128)


def test_emitted_indices_are_nearest_in_the_stored_codebook(oracle_lib):
    """Indices refer to the binary16 codebook that is actually stored: each is the first entry at
    minimal distance (binary32).  Catches: indices taken from the unrounded centres."""
    from paper_1911_02079_amd import synth

    table = synth.mixture_table(300, 64, seed=8).numpy()
    idx, cb = oracle_lib.quantize_rowwise_kmeans16(table, 20)
    q = oracle_lib.unpack_codes(idx, 64)
    book = cb.view(np.float16).astype(np.float32)
    dist = np.abs(table[:, :, None] - book[:, None, :]).astype(np.float32)
    assert np.array_equal(q, dist.argmin(axis=2).astype(np.uint8))  # argmin returns the first minimum
    moved = (book != synth.mixture_table(300, 64, seed=8).numpy().min(1, keepdims=True)).any()
    assert moved


@pytest.mark.parametrize("dim,m,rounds", [(24, 5, 1), (32, 7, 3), (48, 5, 20), (64, 9, 7)])
def test_against_exact_rational_lloyd(oracle_lib, dim, m, rounds):
    """Integer rows with range 15*m: the oracle's float decisions must equal the exact ones, so
    centres agree to binary32 rounding and labels agree exactly (rows with an exact tie between
    two different centres are left out).  Catches: wrong number of rounds, empty clusters moved,
    wrong initial grid, wrong mean."""
    rng = np.random.default_rng(dim + rounds)
    used = 0
    for _ in range(40):
        x = rng.integers(0, 15 * m + 1, dim)
        x[0], x[1] = 0, 15 * m
        x = x - (15 * m) // 2
        centres, labels, tie = exact_lloyd.lloyd(x, rounds)
        if tie:
            continue
        used += 1
        idx, cb, c32 = oracle_lib.quantize_rowwise_kmeans16(x[None, :].astype(np.float32), rounds, return_centres=True)
        want = np.array([float(c) for c in centres])
        assert np.allclose(c32[0].astype(np.float64), want, rtol=2.0 ** -23, atol=0)
        # labels are taken against the binary16 codebook; compare where rounding cannot matter:
        # recompute the exact nearest entry of the stored codebook
        book = cb.view(np.float16).astype(np.float64)[0]
        q = oracle_lib.unpack_codes(idx, dim)[0]
        for e in range(dim):
            d = np.abs(float(x[e]) - book)
            assert q[e] == int(np.argmin(d)) or np.isclose(d[q[e]], d.min(), rtol=1e-6)
    assert used >= 10


def test_against_scikit_learn_lloyd(oracle_lib):
    """A library routine for the special case it covers: scikit-learn's Lloyd iterations started
    from the same grid, on rows where no cluster runs empty (scikit-learn relocates empty
    clusters, this method keeps them)."""
    sklearn_cluster = pytest.importorskip("sklearn.cluster")
    rng = np.random.default_rng(11)
    table = rng.uniform(-1, 1, size=(12, 256)).astype(np.float32)
    _, _, c32 = oracle_lib.quantize_rowwise_kmeans16(table, 20, return_centres=True)
    compared = 0
    for r in range(table.shape[0]):
        x = table[r].astype(np.float64).reshape(-1, 1)
        lo, hi = float(table[r].min()), float(table[r].max())
        init = (lo + np.arange(16) * (hi - lo) / 15).reshape(-1, 1)
        km = sklearn_cluster.KMeans(n_clusters=16, init=init, n_init=1, max_iter=20, tol=0.0, algorithm="lloyd").fit(x)
        if len(np.unique(km.labels_)) < 16:
            continue
        compared += 1
        assert np.allclose(c32[r], km.cluster_centers_[:, 0], rtol=1e-5, atol=1e-6)
    assert compared >= 8


def test_optimal_1d_clustering_is_a_lower_bound(oracle_lib):
    """The exact optimum of 1-D 16-means (dynamic programme over the sorted values) bounds Lloyd's
    result from below, and Lloyd from the grid gets within a factor of it on easy rows."""
    from paper_1911_02079_amd import synth

    table = synth.mixture_table(25, 40, seed=21).numpy()
    _, _, c32 = oracle_lib.quantize_rowwise_kmeans16(table, 20, return_centres=True)
    got = objective(table, c32)
    for r in range(table.shape[0]):
        xs = np.sort(table[r].astype(np.float64))
        n = xs.size
        p1, p2 = np.concatenate([[0], np.cumsum(xs)]), np.concatenate([[0], np.cumsum(xs ** 2)])

        def sse(i, j):  # cost of one cluster xs[i:j]
            s, s2, c = p1[j] - p1[i], p2[j] - p2[i], j - i
            return max(s2 - s * s / c, 0.0)

        best = np.full((17, n + 1), np.inf)
        best[0, 0] = 0.0
        for k in range(1, 17):
            for j in range(k, n + 1):
                best[k, j] = min(best[k - 1, i] + sse(i, j) for i in range(k - 1, j))
        opt = best[16, n]
        assert got[r] >= opt * (1 - 1e-6) - 1e-12
        assert got[r] <= 50 * opt + 1e-6


def test_binary16_tables_are_widened_exactly(oracle_lib):
    """A binary16 table must give what the same values give as a binary32 table: widening is exact
    (NumPy's own conversion feeds the binary32 side, which every other pin covers), so codebook,
    indices and unrounded centres are equal bit for bit, for clustered rows and for dim <= 16.
    Catches: a binary16 row read at the wrong stride or offset, bit patterns read as integers,
    a widening that is not the IEEE one."""
    from paper_1911_02079_amd import synth

    for dim, seed in [(64, 31), (33, 32), (128, 33), (16, 34), (7, 35)]:
        t16 = synth.mixture_table(60, dim, seed=seed).numpy().astype(np.float16)
        # subnormals and both zeros belong to binary16 too
        t16[0, 0], t16[1, 1 % dim], t16[2, 2 % dim] = np.float16(6e-8), np.float16(-0.0), np.float16(-3e-6)
        got = oracle_lib.quantize_rowwise_kmeans16(t16, 20, return_centres=True)
        want = oracle_lib.quantize_rowwise_kmeans16(t16.astype(np.float32), 20, return_centres=True)
        for g, w in zip(got, want):
            assert np.array_equal(g, w)
        assert dim <= 16 or len(np.unique(got[0])) > 16  # the table is not degenerate


def test_populated_grid_fixed_point_from_binary16(oracle_lib):
    """The fixed-point pin again with the table handed over as binary16 (every grid value below is
    exact in binary16): exact codebook, indices and reconstruction."""
    rng = np.random.default_rng(5)
    for lo, s, dim in [(-2.0, 0.25, 64), (0.5, 2.0 ** -6, 33), (-8.0, 1.0, 128)]:
        k = np.concatenate([np.arange(16), rng.integers(0, 16, dim - 16)])
        k = np.stack([rng.permutation(k) for _ in range(20)])
        table = (lo + k * s).astype(np.float16)
        assert np.all(table.astype(np.float64) == lo + k * s)
        idx, cb = oracle_lib.quantize_rowwise_kmeans16(table, 20)
        assert np.array_equal(oracle_lib.unpack_codes(idx, dim), k.astype(np.uint8))
        assert np.all(f16_to_f64(cb) == lo + np.arange(16) * s)
        assert np.array_equal(oracle_lib.dequantize_codebook(idx, cb, dim), table.astype(np.float32))


@pytest.mark.parametrize("dim,m,rounds", [(24, 5, 2), (48, 7, 20)])
def test_exact_rational_lloyd_from_binary16(oracle_lib, dim, m, rounds):
    """Exact rational Lloyd rounds on small integer rows (exact in binary16) handed over as binary16."""
    rng = np.random.default_rng(100 + dim)
    used = 0
    for _ in range(30):
        x = rng.integers(0, 15 * m + 1, dim)
        x[0], x[1] = 0, 15 * m
        x = x - (15 * m) // 2
        centres, _, tie = exact_lloyd.lloyd(x, rounds)
        if tie:
            continue
        used += 1
        _, _, c32 = oracle_lib.quantize_rowwise_kmeans16(x[None, :].astype(np.float16), rounds, return_centres=True)
        want = np.array([float(c) for c in centres])
        assert np.allclose(c32[0].astype(np.float64), want, rtol=2.0 ** -23, atol=0)
    assert used >= 8
