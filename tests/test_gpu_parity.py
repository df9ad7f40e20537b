"""GPU parity: libe4q (through its C ABI, via the ctypes binding) against the CPU oracle,
element by element on the same seeded inputs.

Bar (integer outputs): packed codes, scale bits and bias bits are compared for exact equality
on every row -- both sides follow the same binary32 operation sequence, so any difference is a
bug, not noise.  The relative per-row l2 error (float64, from the emitted artefacts) is also
compared at 1e-5, which is the stated tolerance for the floating-point side.
"""
import sys

import numpy as np
import pytest
import torch

from helpers import f16_bits

pytestmark = pytest.mark.gpu

L2_RTOL = 1e-5


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def e4q():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1911_02079_amd as pkg

    pkg.binding.load_library()  # fails loudly if libe4q.so is missing
    return pkg


def row_l2(table_f32, xh):
    return ((table_f32.astype(np.float64) - xh.astype(np.float64)) ** 2).sum(axis=1)


def compare_with_oracle(e4q, oracle, table_gpu, n_bins, ratio, label):
    """Quantize on the GPU and on the CPU, compare everything; returns the GPU outputs."""
    say(f"{label}: shape={tuple(table_gpu.shape)} dtype={table_gpu.dtype} b={n_bins} r={ratio}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(table_gpu, n_bins, ratio)
    torch.cuda.synchronize()
    host = table_gpu.cpu().numpy()
    o_codes, o_scale, o_bias = oracle.quantize_rowwise_greedy(np.ascontiguousarray(host), n_bins, ratio)
    g_codes = codes.cpu().numpy()
    g_scale = scale.cpu().view(torch.int16).numpy().view(np.uint16)
    g_bias = bias.cpu().view(torch.int16).numpy().view(np.uint16)
    bad_rows = np.flatnonzero((g_codes != o_codes).any(axis=1) | (g_scale != o_scale) | (g_bias != o_bias))
    assert bad_rows.size == 0, f"{label}: {bad_rows.size} rows differ, first {bad_rows[:5]}"
    # floating-point side of the bar: per-row l2 error of the artefacts, and the dequantizer itself
    dim = host.shape[1]
    xh_gpu = e4q.dequantize(codes, scale, bias, dim)
    torch.cuda.synchronize()
    xh_gpu = xh_gpu.cpu().numpy()
    xh_cpu = oracle.dequantize(o_codes, o_scale, o_bias, dim)
    assert np.array_equal(xh_gpu.view(np.uint32), xh_cpu.view(np.uint32)), f"{label}: dequantize differs"
    f32 = host.astype(np.float32)
    lg, lc = row_l2(f32, xh_gpu), row_l2(f32, xh_cpu)
    assert np.all(np.abs(lg - lc) <= L2_RTOL * np.maximum(lc, 1e-300))
    return codes, scale, bias


# --------------------------------------------------------------------------------------------
# The paper-shaped workloads at sizes the oracle finishes in seconds (several tiles + ragged tail)
# --------------------------------------------------------------------------------------------
def test_config1_gaussian_10k_x_64(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.gaussian_table(10_000, 64, 0.1, device="cuda")
    compare_with_oracle(e4q, oracle_lib, t, 200, 0.16, "config1")


def test_config2_outlier_rows(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(50_003, 64, device="cuda")
    compare_with_oracle(e4q, oracle_lib, t, 200, 0.16, "config2-reduced")


def test_config3_laplace_offset_rows(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.laplace_offset_table(30_011, 128, device="cuda")
    compare_with_oracle(e4q, oracle_lib, t, 200, 0.16, "config3-reduced")


def test_config4_batch_of_half_tables(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    specs = synth.batch_specs(26, max_rows=20_000, min_rows=100)
    tables = synth.batch_tables(specs, device="cuda")
    say(f"config4-reduced: {len(tables)} fp16 tables, rows {[s.rows for s in specs]}")
    outs = e4q.quantize_rowwise_greedy_batch(tables, 100, 0.16)
    torch.cuda.synchronize()
    for k, (t, (codes, scale, bias)) in enumerate(zip(tables, outs)):
        o_codes, o_scale, o_bias = oracle_lib.quantize_rowwise_greedy(t.cpu().numpy(), 100, 0.16)
        assert np.array_equal(codes.cpu().numpy(), o_codes), f"table {k}"
        assert np.array_equal(scale.cpu().view(torch.int16).numpy().view(np.uint16), o_scale), f"table {k}"
        assert np.array_equal(bias.cpu().view(torch.int16).numpy().view(np.uint16), o_bias), f"table {k}"


def test_batch_grouping(e4q, oracle_lib):
    """More tables of one dimension than fit one grouped launch (64; 150 make two full launches and a part), mixed
    with other dimensions, input types, an empty table and a table too odd to group."""
    from paper_1911_02079_amd import synth

    rng = np.random.default_rng(0)
    tables = []
    for k in range(150):
        tables.append(synth.gaussian_table(int(rng.integers(1, 3000)), 64, 0.1, seed=9000 + k, device="cuda"))
    for k in range(5):
        tables.append(synth.gaussian_table(int(rng.integers(5000, 30000)), 32, 0.1, seed=9100 + k, device="cuda",
                                           dtype=torch.float16))
    tables.append(torch.empty((0, 64), device="cuda"))
    tables.append(synth.gaussian_table(777, 100, 0.1, seed=9200, device="cuda"))
    tables.append(synth.gaussian_table(50, 128, 0.1, seed=9201, device="cuda"))
    # dimensions the grouped launches do not cover: one launch per table, in whatever layout the table takes
    for k, (rows, dim) in enumerate([(40_000, 200), (30_000, 199), (50_000, 384), (20_000, 300), (9_000, 768), (700, 3000)]):
        tables.append(synth.outlier_table(rows, dim, seed=9300 + k, device="cuda").to(torch.float16 if k % 2 else torch.float32))
    say(f"batch grouping: {len(tables)} tables")
    outs = e4q.quantize_rowwise_greedy_batch(tables, 200, 0.16)
    torch.cuda.synchronize()
    for k, (t, (codes, scale, bias)) in enumerate(zip(tables, outs)):
        if t.shape[0] == 0:
            continue
        o = oracle_lib.quantize_rowwise_greedy(t.cpu().numpy(), 200, 0.16)
        assert np.array_equal(codes.cpu().numpy(), o[0]), f"table {k}"
        assert np.array_equal(f16_bits(scale), o[1]) and np.array_equal(f16_bits(bias), o[2]), f"table {k}"


# --------------------------------------------------------------------------------------------
# Every kernel layout.  The library picks by (rows, dim, ratio) with a cost model: one row per lane for
# large tables of dimension up to 128 (a masked tail when the dimension is not a multiple of 8); otherwise
# L lanes per row with E elements per lane (E = 8 for few rows, 16 to 64 for mid-sized tables, up to 128
# above dimension 128), unmasked / masked per block of 8 / masked per element.
# --------------------------------------------------------------------------------------------
MANY = 64 * 512 + 17   # enough rows for the one-row-per-lane kernels (and a ragged tail)


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("dim", list(range(8, 129, 8)))
def test_row_per_lane_every_dimension(e4q, oracle_lib, dim, dtype):
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(MANY, dim, seed=1000 + dim, device="cuda").to(dtype)
    say(f"row-per-lane dim={dim} {dtype} rows={MANY}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 200, 0.16)
    torch.cuda.synchronize()
    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 200, 0.16)
    assert np.array_equal(codes.cpu().numpy(), o[0])
    assert np.array_equal(f16_bits(scale), o[1]) and np.array_equal(f16_bits(bias), o[2])


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("dim", [1, 2, 3, 5, 7, 8, 12, 16, 24, 33, 40, 63, 64, 100, 128, 130, 200, 256, 257, 504, 512,
                                 513, 1000, 1024, 2000, 2048, 3000])
def test_few_rows_every_layout(e4q, oracle_lib, dim, dtype):
    """Few rows: 8 elements per lane up to dim 512, then 16 / 32 / 64 per lane with 64 lanes per row."""
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(131, dim, seed=2000 + dim, device="cuda").to(dtype)
    compare_with_oracle(e4q, oracle_lib, t, 50, 0.3, f"few rows dim={dim}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("dim", [1, 2, 3, 4, 7, 9, 12, 15, 17, 20, 31, 33, 36, 50, 63, 65, 100, 121, 127, 129, 136, 192,
                                 200, 256, 300, 512, 1000, 1001, 1024, 2047, 2048, 2500])
def test_many_rows_long_chunks(e4q, oracle_lib, dim, dtype):
    """Many rows and a dimension that is not a multiple of 8 (below 128: one row per lane with a masked tail;
    above: 32 or 64 elements per lane) or above 128 (up to 128 elements per lane)."""
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    rows = MANY if dim <= 512 else 64 * 512 + 3
    t = synth.gaussian_table(rows, dim, 0.1, seed=3000 + dim, device="cuda").to(dtype)
    say(f"long chunks dim={dim} {dtype} rows={rows}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 20, 0.25)
    torch.cuda.synchronize()
    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 20, 0.25)
    bad = np.flatnonzero((codes.cpu().numpy() != o[0]).any(axis=1) | (f16_bits(scale) != o[1]) | (f16_bits(bias) != o[2]))
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"


@pytest.mark.parametrize("rows,dim,dtype", [(33_000, 32, torch.float32), (33_000, 64, torch.float32),
                                            (33_000, 128, torch.float32), (50_000, 64, torch.float16),
                                            (65_536, 128, torch.float32), (150_000, 32, torch.float16),
                                            (150_000, 64, torch.float32), (150_000, 128, torch.float32),
                                            (200_000, 128, torch.float16), (100_000, 96, torch.float32),
                                            (40_000, 100, torch.float32), (120_000, 50, torch.float16),
                                            (70_000, 127, torch.float32)])
def test_mid_sized_tables(e4q, oracle_lib, rows, dim, dtype):
    """Tables of one to six waves per SIMD, where the host spreads a row over 2 to 8 lanes (16 to 64
    elements per lane) instead of keeping it in one: every row against the oracle."""
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    t = synth.gaussian_table(rows, dim, 0.1, seed=5000 + rows % 977 + dim, device="cuda").to(dtype)
    say(f"mid-sized table rows={rows} dim={dim} {dtype}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 40, 0.2)
    torch.cuda.synchronize()
    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 40, 0.2)
    bad = np.flatnonzero((codes.cpu().numpy() != o[0]).any(axis=1) | (f16_bits(scale) != o[1]) | (f16_bits(bias) != o[2]))
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"


def test_largest_dimension(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.gaussian_table(9, 4096, 0.1, seed=7, device="cuda")
    compare_with_oracle(e4q, oracle_lib, t, 20, 0.25, "dim=4096 few rows")
    t = synth.gaussian_table(64 * 512 + 1, 4096, 0.1, seed=8, device="cuda")
    say("dim=4096 many rows")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 4, 0.5)
    torch.cuda.synchronize()
    from helpers import oracle_rows_in_parallel

    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 4, 0.5)
    assert np.array_equal(codes.cpu().numpy(), o[0]) and np.array_equal(f16_bits(scale), o[1])


@pytest.mark.parametrize("dim", [8, 24, 64, 100, 128, 256, 1000])
def test_ratio_zero_many_rows(e4q, oracle_lib, dim):
    """Plain min/max quantization (ratio 0) always takes the 8-elements-per-lane layout."""
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(50_001, dim, seed=4000 + dim, device="cuda")
    say(f"ratio=0 dim={dim}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 200, 0.0)
    torch.cuda.synchronize()
    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 200, 0.0)
    assert np.array_equal(codes.cpu().numpy(), o[0])
    assert np.array_equal(f16_bits(scale), o[1]) and np.array_equal(f16_bits(bias), o[2])


# --------------------------------------------------------------------------------------------
# Search settings: ASYM (r = 0), b = 100, "GREEDY (opt)" b = 1000, r = 0.5, tiny b
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n_bins,ratio", [(200, 0.0), (100, 0.16), (1000, 0.5), (1, 0.5), (2, 0.9), (37, 0.33)])
def test_search_settings(e4q, oracle_lib, n_bins, ratio):
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(1_031, 64, seed=77, device="cuda")
    compare_with_oracle(e4q, oracle_lib, t, n_bins, ratio, "settings")


def test_greedy_never_worse_than_minmax_on_the_gpu(e4q):
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(20_000, 64, seed=5, device="cuda")
    say("invariant: greedy <= asym")
    a = e4q.dequantize(*e4q.quantize_rowwise_greedy(t, 200, 0.0), 64)
    g = e4q.dequantize(*e4q.quantize_rowwise_greedy(t, 200, 0.16), 64)
    la = ((t.double() - a.double()) ** 2).sum(1)
    lg = ((t.double() - g.double()) ** 2).sum(1)
    assert bool((lg <= la * (1 + 1e-6)).all())
    assert float(lg.sum() / la.sum()) < 0.9  # clipping pays on outlier rows


# --------------------------------------------------------------------------------------------
# Edge cases
# --------------------------------------------------------------------------------------------
def test_empty_and_single_row(e4q, oracle_lib):
    say("empty table")
    t = torch.empty((0, 64), device="cuda")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t)
    assert codes.shape == (0, 32) and scale.shape == (0,)
    assert e4q.dequantize(codes, scale, bias, 64).shape == (0, 64)
    for dim in (64, 13):
        compare_with_oracle(e4q, oracle_lib, torch.randn(1, dim, device="cuda"), 200, 0.16, "one row")


def test_degenerate_rows(e4q, oracle_lib):
    t = torch.zeros((70, 16), device="cuda")
    t[1] = 0.375
    t[2] = -7.0
    t[3] = 1.0
    t[3, 4] = 1.0 + 2.0 ** -23          # range far below binary16 resolution: scale rounds to 0
    t[4, :8] = 1.0                       # two-valued row
    t[5] = torch.arange(16, device="cuda") * 0.25 - 2.0  # exact 16-point grid
    t[6] = 6.0e-8                        # binary16 subnormal bias
    t[7, 0] = 1.0e-7
    t[8:] = torch.randn(62, 16, device="cuda") * 1e-6    # tiny values: subnormal scale
    codes, scale, bias = compare_with_oracle(e4q, oracle_lib, t, 200, 0.16, "degenerate f32")
    assert int(codes[:4].sum()) == 0
    xh = e4q.dequantize(codes, scale, bias, 16)
    assert torch.equal(xh[5], t[5])      # Eq. 1 reproduces a row that lies on a 16-point grid
    compare_with_oracle(e4q, oracle_lib, t[:, :13].contiguous(), 200, 0.16, "degenerate generic")


def test_strided_and_unaligned_views(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    big = synth.gaussian_table(300, 100, 0.1, seed=3, device="cuda")
    say("row stride > dim (column slice of a wider table)")
    view = big[:, :64]                    # stride 100 elements: rows are 16-byte aligned only by luck
    assert view.stride(0) == 100
    codes, scale, bias = e4q.quantize_rowwise_greedy(view)
    torch.cuda.synchronize()
    o = oracle_lib.quantize_rowwise_greedy(np.ascontiguousarray(view.cpu().numpy()))
    assert np.array_equal(codes.cpu().numpy(), o[0])
    say("base pointer offset by one element (4-byte aligned only)")
    flat = synth.gaussian_table(1, 64 * 200 + 1, 0.1, seed=4, device="cuda").reshape(-1)
    off = flat[1:].reshape(200, 64)
    assert off.data_ptr() % 16 != 0
    codes, scale, bias = e4q.quantize_rowwise_greedy(off)
    torch.cuda.synchronize()
    o = oracle_lib.quantize_rowwise_greedy(np.ascontiguousarray(off.cpu().numpy()))
    assert np.array_equal(codes.cpu().numpy(), o[0])
    assert np.array_equal(scale.cpu().view(torch.int16).numpy().view(np.uint16), o[1])
    say("outputs at odd byte offsets")
    rows, dim = 200, 64
    cbuf = torch.zeros(rows * 32 + 1, dtype=torch.uint8, device="cuda")
    out = (cbuf[1:].reshape(rows, 32), torch.empty(rows, dtype=torch.float16, device="cuda"),
           torch.empty(rows, dtype=torch.float16, device="cuda"))
    e4q.quantize_rowwise_greedy(off, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out[0].cpu().numpy(), o[0])
    assert int(cbuf[0]) == 0
    say("dequantize from an unaligned code buffer")
    xh = e4q.dequantize(cbuf[1:].reshape(rows, 32), out[1], out[2], dim)
    torch.cuda.synchronize()
    assert np.array_equal(xh.cpu().numpy(), oracle_lib.dequantize(o[0], o[1], o[2], dim))


@pytest.mark.parametrize("nbits", [2, 4, 8])
@pytest.mark.parametrize("dim", [300, 320, 384, 768])
def test_lane_counts_that_are_not_powers_of_two_on_views_and_guarded_outputs(e4q, oracle_lib, dim, nbits):
    """Dimensions that take 3, 5 or 6 lanes per row (a wave then holds 21, 12 or 10 rows and its last lanes idle):
    column slices of wider tables with 16-byte aligned and unaligned rows, a row count that leaves the last workgroup
    partly empty, outputs at an odd byte offset between guard bytes."""
    from paper_1911_02079_amd import synth

    rows = 1003
    for extra in (4, 1):
        big = synth.outlier_table(rows, dim + extra, seed=6100 + dim + extra, device="cuda")
        view = big[:, :dim]
        nb = e4q.packed_bytes(dim, nbits)
        cbuf = torch.full((rows * nb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        sbuf = torch.full((rows + 16,), 1.5, dtype=torch.float16, device="cuda")
        bbuf = torch.full((rows + 16,), 1.5, dtype=torch.float16, device="cuda")
        out = (cbuf[31:31 + rows * nb].reshape(rows, nb), sbuf[8:8 + rows], bbuf[8:8 + rows])
        say(f"dim={dim} nbits={nbits} row stride {dim + extra}, guarded outputs")
        # what a large table of this dimension runs with; 1003 rows alone would be spread over 64 lanes each
        layout = {300: (64, 5), 320: (64, 5), 384: (128, 3), 768: (128, 6)}[dim]
        try:
            e4q.set_option("greedy_layout", e4q.greedy_layout_value(layout))
            e4q.quantize_rowwise_greedy(view, 50, 0.2, nbits=nbits, out=out)
            torch.cuda.synchronize()
        finally:
            e4q.set_option("greedy_layout", 0)
        assert e4q.get_option("greedy_layout_chosen") == e4q.greedy_layout_value(layout)
        o = oracle_lib.quantize_rowwise_greedy(np.ascontiguousarray(view.cpu().numpy()), 50, 0.2, nbits=nbits)
        assert np.array_equal(out[0].cpu().numpy(), o[0])
        assert np.array_equal(f16_bits(out[1]), o[1]) and np.array_equal(f16_bits(out[2]), o[2])
        assert bool((cbuf[:31] == 0xA5).all()) and bool((cbuf[31 + rows * nb:] == 0xA5).all())
        for guard in (sbuf, bbuf):
            assert bool((guard[:8] == 1.5).all()) and bool((guard[8 + rows:] == 1.5).all())


@pytest.mark.parametrize("nbits", [2, 4, 8])
@pytest.mark.parametrize("dim", [1, 3, 4, 5, 6, 7, 13, 50, 101, 127, 130])
def test_dequantize_odd_dimensions_aligned_and_not(e4q, oracle_lib, dim, nbits):
    """dim % 4 != 0: four flattened elements per thread into a 16-byte aligned output (groups straddle row
    boundaries, the last group is partial), one element per thread into an output that is not; and an odd
    dimension of the masked-tail quantizer written into a code buffer that is 4-byte aligned only."""
    from paper_1911_02079_amd import synth

    rows = 64 * 9 + 5
    t = synth.gaussian_table(rows, dim, 0.1, seed=7100 + dim, device="cuda")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 30, 0.2, nbits=nbits)
    torch.cuda.synchronize()
    o = oracle_lib.quantize_rowwise_greedy(t.cpu().numpy(), 30, 0.2, nbits=nbits)
    assert np.array_equal(codes.cpu().numpy(), o[0])
    want = oracle_lib.dequantize(o[0], o[1], o[2], dim, nbits=nbits)
    say(f"dequantize dim={dim} nbits={nbits}, aligned output")
    xh = e4q.dequantize(codes, scale, bias, dim, nbits=nbits)
    torch.cuda.synchronize()
    assert xh.data_ptr() % 16 == 0 and np.array_equal(xh.cpu().numpy(), want)
    say(f"dequantize dim={dim} nbits={nbits}, output offset by 4 bytes")
    buf = torch.full((rows * dim + 2,), -7.0, device="cuda")
    e4q.dequantize(codes, scale, bias, dim, nbits=nbits, out=buf[1:-1].reshape(rows, dim))
    torch.cuda.synchronize()
    assert np.array_equal(buf[1:-1].reshape(rows, dim).cpu().numpy(), want)
    assert float(buf[0]) == -7.0 and float(buf[-1]) == -7.0
    say(f"quantize dim={dim} nbits={nbits} into a code buffer offset by 4 bytes")
    nbytes = codes.shape[1]
    cbuf = torch.full((rows * nbytes + 8,), 0xAB, dtype=torch.uint8, device="cuda")
    out = (cbuf[4:-4].reshape(rows, nbytes), torch.empty_like(scale), torch.empty_like(bias))
    e4q.quantize_rowwise_greedy(t, 30, 0.2, nbits=nbits, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out[0].cpu().numpy(), o[0])
    assert bool((cbuf[:4] == 0xAB).all()) and bool((cbuf[-4:] == 0xAB).all())


@pytest.mark.parametrize("dim", [64, 100, 200])
def test_non_finite_rows_do_not_disturb_their_neighbours(e4q, oracle_lib, dim):
    """Rows with NaN, infinities or values whose squares overflow give unspecified outputs but no fault,
    and the rows next to them (same wave, same workgroup) still match the oracle bit for bit."""
    from paper_1911_02079_amd import synth

    rows = 64 * 600 + 9
    t = synth.gaussian_table(rows, dim, 0.1, seed=8800 + dim, device="cuda")
    bad = torch.arange(3, rows, 7, device="cuda")
    t[bad[0::4], 1] = float("nan")
    t[bad[1::4], 2] = float("inf")
    t[bad[2::4], 0] = float("-inf")
    t[bad[3::4], 5] = 3.0e30
    t[bad[3::4], 6] = -3.0e30
    say(f"non-finite rows dim={dim}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t)
    xh = e4q.dequantize(codes, scale, bias, dim)
    idx, cent = e4q.quantize_rowwise_kmeans16(t, 5)
    torch.cuda.synchronize()
    good = torch.ones(rows, dtype=torch.bool, device="cuda")
    good[bad] = False
    tg = t[good].contiguous()
    o = oracle_lib.quantize_rowwise_greedy(tg.cpu().numpy())
    assert np.array_equal(codes[good].cpu().numpy(), o[0])
    assert np.array_equal(f16_bits(scale[good]), o[1]) and np.array_equal(f16_bits(bias[good]), o[2])
    assert np.array_equal(xh[good].cpu().numpy(), oracle_lib.dequantize(o[0], o[1], o[2], dim))
    k = oracle_lib.quantize_rowwise_kmeans16(tg.cpu().numpy(), 5)
    assert np.array_equal(idx[good].cpu().numpy(), k[0]) and np.array_equal(f16_bits(cent[good]), k[1])


def random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        dim = int(rng.choice([rng.integers(1, 17), rng.integers(17, 129), rng.integers(129, 400), 8 * rng.integers(1, 17)]))
        rows = int(10 ** rng.uniform(2.0, 5.8))
        rows = min(rows, 12_000_000 // dim)
        out.append((rows, dim, bool(rng.integers(0, 2)), int(rng.choice([2, 4, 4, 4, 8])), int(rng.integers(3, 40)),
                    float(np.float32(rng.uniform(0.05, 0.6)))))
    return out


@pytest.mark.parametrize("rows,dim,half,nbits,n_bins,ratio", random_shapes(64, 20261127))
def test_random_shapes(e4q, oracle_lib, rows, dim, half, nbits, n_bins, ratio):
    """Seeded random (rows, dim, input type, code width, search setting): whatever layout the host picks for
    the shape, every row matches the oracle, and the de-quantizer matches on the emitted artefacts."""
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(rows, dim, seed=rows + dim, device="cuda")
    if half:
        t = t.half()
    say(f"random shape rows={rows} dim={dim} half={half} nbits={nbits} b={n_bins} r={ratio:.3f}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, n_bins, ratio, nbits=nbits)
    xh = e4q.dequantize(codes, scale, bias, dim, nbits=nbits)
    torch.cuda.synchronize()
    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), n_bins, ratio, nbits=nbits)
    bad = np.flatnonzero((codes.cpu().numpy() != o[0]).any(axis=1) | (f16_bits(scale) != o[1]) | (f16_bits(bias) != o[2]))
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"
    assert np.array_equal(xh.cpu().numpy(), oracle_lib.dequantize(o[0], o[1], o[2], dim, nbits=nbits))


@pytest.mark.parametrize("nbits", [2, 4, 8])
@pytest.mark.parametrize("dim,half", [(8, False), (24, False), (64, True), (100, False), (136, False), (320, False)])
def test_every_binade_of_scale(e4q, oracle_lib, dim, half, nbits):
    """Rows scaled by 2^-22 ... 2^13: the stored scale runs through the binary16 subnormals and every normal
    binade, so the per-range divisions (range / (2^n - 1) and 1 / scale, which the kernels take by a short
    sequence) are compared with the oracle's plain divisions across their whole working range."""
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    rows = 36 * 64 * 3 + 11
    t = synth.outlier_table(rows, dim, seed=4242 + dim + nbits, device="cuda")
    t = t / t.abs().amax(dim=1, keepdim=True)                                  # every row within [-1, 1]
    k = (torch.arange(rows, device="cuda") % 36 - 22).to(torch.float32)         # -22 ... 13
    t = t * torch.exp2(k)[:, None] * torch.linspace(1.0, 1.99, rows, device="cuda")[:, None]
    if half:
        t = t.half()
    say(f"every binade dim={dim} half={half} nbits={nbits}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 40, 0.3, nbits=nbits)
    torch.cuda.synchronize()
    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 40, 0.3, nbits=nbits)
    bad = np.flatnonzero((codes.cpu().numpy() != o[0]).any(axis=1) | (f16_bits(scale) != o[1]) | (f16_bits(bias) != o[2]))
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"
    assert len(np.unique(o[1] >> 10)) >= 20   # the stored scales do span the binary16 exponents, subnormals included


@pytest.mark.parametrize("dim", [8, 64, 100, 320])
def test_binary32_subnormal_rows(e4q, oracle_lib, dim):
    """Rows whose values are binary32 subnormals or just above them (2^-149 ... 2^-110): every stored scale
    rounds to zero in binary16, ranges and step sizes are subnormal, and the kernels must treat such numbers as
    the CPU does (no flush to zero), stored signs of zero included."""
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    rows = 64 * 9 + 3
    t = synth.gaussian_table(rows, dim, 1.0, seed=8800 + dim, device="cuda")
    k = (torch.arange(rows, device="cuda") % 40 - 149).to(torch.float32)          # -149 ... -110
    t = (t.double() * torch.exp2(k.double())[:, None]).float()                    # rounds into the subnormal grid
    assert bool((t.abs() < 1.2e-38).any()) and bool((t != 0).any())
    say(f"subnormal rows dim={dim}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 40, 0.3)
    xh = e4q.dequantize(codes, scale, bias, dim)
    torch.cuda.synchronize()
    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 40, 0.3)
    bad = np.flatnonzero((codes.cpu().numpy() != o[0]).any(axis=1) | (f16_bits(scale) != o[1]) | (f16_bits(bias) != o[2]))
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"
    assert np.array_equal(xh.cpu().numpy().view(np.uint32), oracle_lib.dequantize(o[0], o[1], o[2], dim).view(np.uint32))


@pytest.mark.parametrize("dim,half", [(8, False), (64, True), (100, False), (128, False), (200, False), (512, True)])
def test_rows_with_zeros_of_both_signs(e4q, oracle_lib, dim, half):
    """Sparse rows whose zeros carry either sign (what pruning or a binary16 conversion of tiny negative
    values leaves behind), rows of zeros only, rows whose maximum is zero: a zero bound is +0 on both
    sides, so the stored bias and scale bits agree whatever order the kernel compares the elements in."""
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    rows = 64 * 21 + 13
    g = torch.Generator(device="cuda").manual_seed(9100 + dim)
    t = synth.gaussian_table(rows, dim, 0.1, seed=9000 + dim, device="cuda")
    keep = torch.rand((rows, dim), device="cuda", generator=g) < 0.3
    negzero = torch.rand((rows, dim), device="cuda", generator=g) < 0.5
    t = torch.where(keep, t, torch.where(negzero, torch.full_like(t, -0.0), torch.zeros_like(t)))
    t[1::7] = t[1::7].abs()            # minimum zero
    t[2::7] = -t[2::7].abs()           # maximum zero
    t[3::7] = torch.where(negzero[3::7], torch.full_like(t[3::7], -0.0), torch.zeros_like(t[3::7]))  # zeros only
    t[4::49] = -0.0                    # nothing but -0
    if half:
        t = t.half()
    say(f"signed zeros dim={dim} half={half}")
    for ratio in (0.0, 0.25):
        codes, scale, bias = e4q.quantize_rowwise_greedy(t, 30, ratio)
        xh = e4q.dequantize(codes, scale, bias, dim)
        torch.cuda.synchronize()
        o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 30, ratio)
        bad = np.flatnonzero((codes.cpu().numpy() != o[0]).any(axis=1) | (f16_bits(scale) != o[1]) | (f16_bits(bias) != o[2]))
        assert bad.size == 0, f"ratio {ratio}: {bad.size} rows differ, first {bad[:5]}"
        want = oracle_lib.dequantize(o[0], o[1], o[2], dim)
        assert np.array_equal(xh.cpu().numpy().view(np.uint32), want.view(np.uint32))   # signs of zeros included


def test_outputs_do_not_overrun(e4q):
    """Guard bands around the outputs stay untouched (ragged row count, fast and fallback paths)."""
    from paper_1911_02079_amd import synth

    for dim, rows in ((64, 64 * 3 + 5), (13, 64 * 3 + 5), (64, 64 * 512 + 5), (200, 64 * 512 + 5), (13, 64 * 512 + 5),
                      (100, 64 * 512 + 1), (127, 64 * 600 + 63), (33, 150_001), (1001, 64 * 512 + 5)):
        t = synth.gaussian_table(rows, dim, 0.1, seed=9, device="cuda")
        nb = (dim + 1) // 2
        say(f"guard bands dim={dim} rows={rows}")
        cbuf = torch.full((rows * nb + 256,), 0xA5, dtype=torch.uint8, device="cuda")
        sbuf = torch.full((rows + 64,), -3.0, dtype=torch.float16, device="cuda")
        bbuf = torch.full((rows + 64,), -3.0, dtype=torch.float16, device="cuda")
        out = (cbuf[128:128 + rows * nb].reshape(rows, nb), sbuf[32:32 + rows], bbuf[32:32 + rows])
        e4q.quantize_rowwise_greedy(t, out=out)
        torch.cuda.synchronize()
        assert bool((cbuf[:128] == 0xA5).all()) and bool((cbuf[128 + rows * nb:] == 0xA5).all())
        for buf in (sbuf, bbuf):
            assert bool((buf[:32] == -3.0).all()) and bool((buf[32 + rows:] == -3.0).all())
        xbuf = torch.full((rows * dim + 64,), 7.0, device="cuda")
        e4q.dequantize(*out, dim, out=xbuf[32:32 + rows * dim].reshape(rows, dim))
        torch.cuda.synchronize()
        assert bool((xbuf[:32] == 7.0).all()) and bool((xbuf[32 + rows * dim:] == 7.0).all())


def test_runs_on_a_side_stream(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.gaussian_table(5_000, 32, 0.1, seed=12, device="cuda")
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    say("side stream")
    with torch.cuda.stream(s):
        codes, scale, bias = e4q.quantize_rowwise_greedy(t)
        xh = e4q.dequantize(codes, scale, bias, 32)
    s.synchronize()
    o = oracle_lib.quantize_rowwise_greedy(t.cpu().numpy())
    assert np.array_equal(codes.cpu().numpy(), o[0])
    assert np.array_equal(xh.cpu().numpy(), oracle_lib.dequantize(*o, 32))


def test_binding_reports_library_errors(e4q):
    t = torch.randn(4, 64, device="cuda")
    with pytest.raises(e4q.E4QError) as ei:
        e4q.quantize_rowwise_greedy(t, nbits=3)
    assert ei.value.code == -3
    with pytest.raises(e4q.E4QError):
        e4q.quantize_rowwise_greedy(t, ratio=1.5)


# --------------------------------------------------------------------------------------------
# Other bit widths (8 = the paper's ASYM-8BITS baseline, 2) through every kernel layout
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("nbits", [2, 8])
@pytest.mark.parametrize("rows,dim,dtype,ratio", [
    (MANY, 128, torch.float32, 0.16), (MANY, 64, torch.float16, 0.16), (MANY, 8, torch.float32, 0.16),
    (MANY, 24, torch.float32, 0.16),                                   # one row per lane
    (777, 64, torch.float32, 0.16), (777, 128, torch.float16, 0.16), (131, 24, torch.float32, 0.16),
    (131, 8, torch.float32, 0.16), (131, 13, torch.float32, 0.16), (131, 1, torch.float32, 0.16),
    (131, 5, torch.float16, 0.16), (131, 100, torch.float32, 0.16), (131, 1000, torch.float32, 0.16),
    (131, 2048, torch.float16, 0.16),                                  # few rows: 8..64 per lane
    (MANY, 100, torch.float32, 0.16), (MANY, 200, torch.float32, 0.16), (MANY, 256, torch.float16, 0.16),
    (MANY, 36, torch.float32, 0.16),                                   # many rows, long chunks, masked
    (MANY, 150, torch.float32, 0.16), (MANY, 199, torch.float16, 0.16), (MANY, 224, torch.float32, 0.16),  # one row per lane above 128
    (50_001, 128, torch.float32, 0.0), (50_001, 24, torch.float32, 0.0), (50_001, 100, torch.float32, 0.0),
])
def test_other_bit_widths(e4q, oracle_lib, nbits, rows, dim, dtype, ratio):
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(rows, dim, seed=7000 + dim + nbits, device="cuda").to(dtype)
    say(f"nbits={nbits} rows={rows} dim={dim} {dtype} ratio={ratio}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t, 20, ratio if ratio == 0 else 0.25, nbits=nbits)
    xh = e4q.dequantize(codes, scale, bias, dim, nbits=nbits)
    torch.cuda.synchronize()
    o = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), 20, ratio if ratio == 0 else 0.25, nbits=nbits)
    assert codes.shape[1] == e4q.packed_bytes(dim, nbits)
    bad = np.flatnonzero((codes.cpu().numpy() != o[0]).any(axis=1) | (f16_bits(scale) != o[1]) | (f16_bits(bias) != o[2]))
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"
    sample = slice(0, min(rows, 3000))
    assert np.array_equal(xh[sample].cpu().numpy(), oracle_lib.dequantize(o[0][sample], o[1][sample], o[2][sample], dim, nbits))


def test_other_bit_widths_batch_and_guard_bands(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    tables = [synth.gaussian_table(20_000 + 13 * k, 64, 0.1, seed=7100 + k, device="cuda") for k in range(3)]
    for nbits in (2, 8):
        say(f"batch nbits={nbits}")
        outs = e4q.quantize_rowwise_greedy_batch(tables, 20, 0.25, nbits=nbits)
        torch.cuda.synchronize()
        for t, (codes, scale, bias) in zip(tables, outs):
            o = oracle_lib.quantize_rowwise_greedy(t.cpu().numpy(), 20, 0.25, nbits=nbits)
            assert np.array_equal(codes.cpu().numpy(), o[0]) and np.array_equal(f16_bits(scale), o[1])
        for dim, rows in ((64, 64 * 512 + 5), (13, 197), (200, 64 * 512 + 5), (199, 64 * 512 + 5)):
            t = synth.gaussian_table(rows, dim, 0.1, seed=9, device="cuda")
            nb = e4q.packed_bytes(dim, nbits)
            cbuf = torch.full((rows * nb + 256,), 0xA5, dtype=torch.uint8, device="cuda")
            out = (cbuf[128:128 + rows * nb].reshape(rows, nb), torch.empty(rows, dtype=torch.float16, device="cuda"),
                   torch.empty(rows, dtype=torch.float16, device="cuda"))
            e4q.quantize_rowwise_greedy(t, 20, 0.25, nbits=nbits, out=out)
            torch.cuda.synchronize()
            assert bool((cbuf[:128] == 0xA5).all()) and bool((cbuf[128 + rows * nb:] == 0xA5).all())
            o = oracle_lib.quantize_rowwise_greedy(t.cpu().numpy(), 20, 0.25, nbits=nbits)
            assert np.array_equal(out[0].cpu().numpy(), o[0])
