"""Pins for the 4-bit SparseLengthsSum part of the CPU oracle (Section 4 of the paper)."""
import numpy as np
import pytest
import scipy.sparse as sp


def random_bags(rng, rows, n_bags, max_len, out_of_range=0):
    lengths = rng.integers(0, max_len + 1, n_bags)
    lengths[rng.integers(0, n_bags, max(1, n_bags // 10))] = 0  # some empty bags
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    indices = rng.integers(0, rows, int(offsets[-1])).astype(np.int64)
    if out_of_range and indices.size:
        bad = rng.integers(0, indices.size, out_of_range)
        indices[bad[::2]] = rows + rng.integers(0, 5, bad[::2].size)
        indices[bad[1::2]] = -1 - rng.integers(0, 5, bad[1::2].size)
    return indices, offsets


def incidence(indices, offsets, rows):
    """Sparse n_bags x rows matrix of index multiplicities (out-of-range indices dropped)."""
    n_bags = offsets.size - 1
    bag_of = np.repeat(np.arange(n_bags), np.diff(offsets))
    ok = (indices >= 0) & (indices < rows)
    return sp.csr_matrix((np.ones(ok.sum()), (bag_of[ok], indices[ok])), shape=(n_bags, rows))


def f16(x):
    return np.asarray(x, dtype=np.float16).view(np.uint16)


@pytest.mark.parametrize("dim", [8, 13, 64])
def test_integer_tables_against_exact_incidence_product(oracle_lib, dim):
    """scale 1 or 2 and integer bias: every de-quantized value is a small integer, every sum is
    exact, and the result must equal (incidence matrix) x (de-quantized table) computed by a sparse
    library product.  Catches wrong nibble, wrong row, bags shifted by one, dropped bias."""
    rng = np.random.default_rng(dim)
    rows = 500
    q = rng.integers(0, 16, (rows, dim)).astype(np.uint8)
    qp = np.concatenate([q, np.zeros((rows, dim % 2), np.uint8)], axis=1)
    codes = (qp[:, 0::2] | (qp[:, 1::2] << 4)).astype(np.uint8)
    scale = rng.choice([1.0, 2.0], rows)
    bias = rng.integers(-20, 20, rows).astype(np.float64)
    table = q * scale[:, None] + bias[:, None]
    indices, offsets = random_bags(rng, rows, 300, 40, out_of_range=30)
    got = oracle_lib.sparse_lengths_sum(codes, f16(scale), f16(bias), dim, indices, offsets)
    want = incidence(indices, offsets, rows) @ table
    assert np.array_equal(got.astype(np.float64), want)
    assert np.all(got[np.diff(offsets) == 0] == 0)


def test_float_tables_against_float64_product(oracle_lib):
    from paper_1911_02079_amd import synth

    rng = np.random.default_rng(5)
    t = synth.gaussian_table(2000, 32, 0.1, seed=9).numpy()
    codes, sc, bi = oracle_lib.quantize_rowwise_greedy(t)
    xh = oracle_lib.dequantize(codes, sc, bi, 32).astype(np.float64)
    indices, offsets = random_bags(rng, 2000, 400, 100)
    got = oracle_lib.sparse_lengths_sum(codes, sc, bi, 32, indices, offsets)
    want = incidence(indices, offsets, 2000) @ xh
    scale_of_sum = incidence(indices, offsets, 2000) @ np.abs(xh)
    assert np.all(np.abs(got - want) <= 1e-6 * scale_of_sum + 1e-12)


def test_single_index_bags_reproduce_the_dequantizer(oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(300, 24, seed=3).numpy()
    codes, sc, bi = oracle_lib.quantize_rowwise_greedy(t)
    perm = np.random.default_rng(1).permutation(300).astype(np.int64)
    got = oracle_lib.sparse_lengths_sum(codes, sc, bi, 24, perm, np.arange(301, dtype=np.int64))
    assert np.array_equal(got, oracle_lib.dequantize(codes, sc, bi, 24)[perm])


def test_accumulation_runs_left_to_right(oracle_lib):
    """Row 0 de-quantizes to 491520 (ulp 1/32), row 1 to 1/128.  Adding four small values one at a
    time to the large one changes nothing; adding the large one last keeps their sum."""
    codes = np.array([[0xFF], [0x11]], dtype=np.uint8)          # dim 2: codes (15, 15) and (1, 1)
    sc, bi = f16([32768.0, 2.0 ** -7]), f16([0.0, 0.0])
    offsets = np.array([0, 5, 10], dtype=np.int64)
    indices = np.array([0, 1, 1, 1, 1, 1, 1, 1, 1, 0], dtype=np.int64)
    got = oracle_lib.sparse_lengths_sum(codes, sc, bi, 2, indices, offsets)
    assert got[0].tolist() == [491520.0, 491520.0]
    assert got[1].tolist() == [491520.03125, 491520.03125]


def test_empty_inputs(oracle_lib):
    codes = np.zeros((3, 4), dtype=np.uint8)
    sc, bi = f16([1, 1, 1]), f16([0, 0, 0])
    out = oracle_lib.sparse_lengths_sum(codes, sc, bi, 8, np.zeros(0, np.int64), np.zeros(1, np.int64))
    assert out.shape == (0, 8)
    out = oracle_lib.sparse_lengths_sum(codes, sc, bi, 8, np.zeros(0, np.int64), np.zeros(5, np.int64))
    assert out.shape == (4, 8) and np.all(out == 0)


def test_fused_records_hold_codes_then_scale_then_bias(oracle_lib):
    """The fused lookup record, byte by byte, on a hand-written example (little-endian binary16)."""
    codes = np.array([[0x10, 0x32, 0x54], [0xAB, 0xCD, 0xEF]], dtype=np.uint8)   # dim 5 or 6: 3 code bytes
    sc, bi = f16([1.0, 0.5]), f16([-2.0, 3.0])        # 0x3C00, 0x3800 / 0xC000, 0x4200
    got = oracle_lib.fuse_rows(codes, sc, bi, 6, 10)
    assert got.tolist() == [[0x10, 0x32, 0x54, 0, 0x00, 0x3C, 0x00, 0xC0, 0, 0],
                            [0xAB, 0xCD, 0xEF, 0, 0x00, 0x38, 0x00, 0x42, 0, 0]]
    with pytest.raises(ValueError):
        oracle_lib.fuse_rows(codes, sc, bi, 6, 7)      # too small
    with pytest.raises(ValueError):
        oracle_lib.fuse_rows(codes, sc, bi, 6, 9)      # odd
    # and the codes / parameters can be read back from where the layout says they are
    rng = np.random.default_rng(0)
    c = rng.integers(0, 256, (50, 32)).astype(np.uint8)
    s, b = rng.integers(0, 0x7BFF, 50).astype(np.uint16), rng.integers(0, 0x7BFF, 50).astype(np.uint16)
    rec = oracle_lib.fuse_rows(c, s, b, 64, 68)
    assert np.array_equal(rec[:, :32], c)
    assert np.array_equal(rec[:, 32:34].copy().view(np.uint16)[:, 0], s)
    assert np.array_equal(rec[:, 34:36].copy().view(np.uint16)[:, 0], b)
