"""Tables with more than 2^32 groups or elements: the 64-bit index paths of the de-quantizers and of the search.

The paper's own tables (50 M rows of 128 values, Section 5) have 6.4e9 elements.  The codes here are
random bytes (any byte string is a valid packed row) and the outputs are compared with the oracle on
the first rows, the last rows, the rows on either side of the 2^32 boundary and a strided sample;
the first mismatch ends the test."""
import sys

import numpy as np
import pytest
import torch

from helpers import f16_bits

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def e4q():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1911_02079_amd as pkg

    pkg.binding.load_library()
    return pkg


def random_bytes(shape, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    n = int(np.prod(shape))
    assert n % 8 == 0
    words = torch.randint(-2 ** 62, 2 ** 62, (n // 8,), dtype=torch.int64, device="cuda", generator=g)
    return words.view(torch.uint8).reshape(shape)


def sample_rows(rows, per_row, boundary_item):
    """Rows to compare: both ends, around the row that holds item number `boundary_item`, a stride."""
    b = boundary_item // per_row
    picks = list(range(0, 40)) + list(range(rows - 40, rows)) + list(range(max(b - 20, 0), min(b + 21, rows)))
    picks += list(range(0, rows, max(rows // 997, 1)))
    return np.unique(np.array(picks, dtype=np.int64))


def small_params(rows, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    scale = (torch.rand(rows, device="cuda", generator=g) * 0.01 + 0.001).half()
    bias = (torch.rand(rows, device="cuda", generator=g) - 0.5).half()
    return scale, bias


@pytest.mark.parametrize("dim,rows,nbits,what", [
    (4096, 4_194_353, 2, "dequantize_w4_kernel<2, wide>: 4.29e9 groups of four"),
    (4095, 1_048_850, 2, "dequantize_flat4_kernel<wide>: 4.29e9 elements, rows of 4095"),
])
def test_dequantize_beyond_2_pow_32(e4q, oracle_lib, dim, rows, nbits, what):
    per = 8 // nbits
    nbytes = (dim + per - 1) // per
    items = rows * (dim // 4) if dim % 4 == 0 else rows * dim
    assert items > 2 ** 32
    say(f"{what}: {rows} x {dim}, codes {rows * nbytes / 2**30:.1f} GiB, output {rows * dim * 4 / 2**30:.1f} GiB")
    pad = (-rows * nbytes) % 8
    codes = random_bytes((rows * nbytes + pad,), 1)[: rows * nbytes].reshape(rows, nbytes)
    scale, bias = small_params(rows, 2)
    out = e4q.dequantize(codes, scale, bias, dim, nbits=nbits)
    torch.cuda.synchronize()
    picks = sample_rows(rows, dim // 4 if dim % 4 == 0 else dim, 2 ** 32)
    sel = torch.from_numpy(picks).cuda()
    want = oracle_lib.dequantize(codes[sel].cpu().numpy(), f16_bits(scale[sel]), f16_bits(bias[sel]), dim, nbits=nbits)
    got = out[sel].cpu().numpy()
    bad = np.flatnonzero((got.view(np.uint32) != want.view(np.uint32)).any(axis=1))
    assert bad.size == 0, f"rows {picks[bad[:5]]} differ"
    del out, codes
    torch.cuda.empty_cache()


def test_codebook_dequantize_beyond_2_pow_32(e4q, oracle_lib):
    dim, rows = 4095, 1_048_850
    nbytes = (dim + 1) // 2
    say(f"dequantize_codebook_flat4_kernel<wide>: {rows} x {dim}, output {rows * dim * 4 / 2**30:.1f} GiB")
    pad = (-rows * nbytes) % 8
    idx = random_bytes((rows * nbytes + pad,), 3)[: rows * nbytes].reshape(rows, nbytes)
    if dim % 2:
        idx[:, -1] &= 0x0F  # the unused nibble of the last byte is 0 in a valid row
    g = torch.Generator(device="cuda").manual_seed(4)
    book = (torch.rand((rows, 16), device="cuda", generator=g) - 0.5).half()
    out = e4q.dequantize_codebook(idx, book, dim)
    torch.cuda.synchronize()
    picks = sample_rows(rows, dim, 2 ** 32)
    sel = torch.from_numpy(picks).cuda()
    want = oracle_lib.dequantize_codebook(idx[sel].cpu().numpy(), f16_bits(book[sel]), dim)
    got = out[sel].cpu().numpy()
    bad = np.flatnonzero((got.view(np.uint32) != want.view(np.uint32)).any(axis=1))
    assert bad.size == 0, f"rows {picks[bad[:5]]} differ"
    del out, idx
    torch.cuda.empty_cache()


def test_greedy_on_a_table_of_the_papers_size(e4q, oracle_lib):
    """50 M rows x 128 binary32 (the largest tables of Section 5; 6.4e9 elements, 25.6 GB): Algorithm 1 at its
    defaults over the whole table in one call, then compared with the oracle on both ends, on the rows on either side
    of element number 2^32, and on a strided sample; de-quantized rows of the same sample as well."""
    from helpers import oracle_rows_in_parallel
    from paper_1911_02079_amd import synth

    rows, dim = 50_000_000, 128
    say(f"paper-size table: drawing {rows} x {dim} binary32 ({rows * dim * 4 / 1e9:.1f} GB)")
    table = synth.laplace_offset_table(rows, dim, seed=5050, device="cuda")
    out = e4q.alloc_outputs(rows, dim, table.device)
    say("paper-size table: GPU quantize")
    e4q.quantize_rowwise_greedy(table, 200, 0.16, out=out)
    torch.cuda.synchronize()
    assert e4q.get_option("greedy_layout_chosen") == 1  # one row per lane
    picks = np.unique(np.concatenate([sample_rows(rows, dim, 1 << 32), np.arange(0, rows, 499)]))
    sel = torch.from_numpy(picks).cuda()
    say(f"paper-size table: oracle on {picks.size} sampled rows")
    o_codes, o_scale, o_bias = oracle_rows_in_parallel(oracle_lib, table[sel].cpu().numpy(), 200, 0.16)
    bad = np.flatnonzero((out[0][sel].cpu().numpy() != o_codes).any(axis=1) | (f16_bits(out[1][sel]) != o_scale) |
                         (f16_bits(out[2][sel]) != o_bias))
    assert bad.size == 0, f"rows {picks[bad[:5]]} differ"
    del table
    torch.cuda.empty_cache()
    say("paper-size table: de-quantize and compare the same rows")
    xh = e4q.dequantize(*out, dim)
    torch.cuda.synchronize()
    want = oracle_lib.dequantize(o_codes, o_scale, o_bias, dim)
    assert np.array_equal(xh[sel].cpu().numpy().view(np.uint32), want.view(np.uint32))
    del xh, out
    torch.cuda.empty_cache()


def test_greedy_launch_folded_into_two_grid_dimensions(e4q, oracle_lib):
    """More workgroups than one grid dimension is given (2^21): plain min/max quantization of a
    binary16 table of 8.4 M rows x 512, which runs with 64 lanes per row, four rows per workgroup."""
    from paper_1911_02079_amd import synth

    rows, dim = (1 << 23) + 1_003, 512
    say(f"folded grid: {rows} x {dim} binary16, ratio 0 ({rows * dim * 2 / 2**30:.1f} GiB)")
    table = synth.gaussian_table(rows, dim, 0.1, seed=7000, device="cuda", dtype=torch.float16)
    codes, scale, bias = e4q.quantize_rowwise_greedy(table, 200, 0.0)
    torch.cuda.synchronize()
    assert e4q.get_option("greedy_layout_chosen") == (8 << 8) | 64
    picks = sample_rows(rows, 1, 4 * (1 << 21))  # the row where the grid's second row of workgroups starts
    sel = torch.from_numpy(picks).cuda()
    want = oracle_lib.quantize_rowwise_greedy(table[sel].cpu().numpy(), 200, 0.0)
    assert np.array_equal(codes[sel].cpu().numpy(), want[0])
    assert np.array_equal(f16_bits(scale[sel]), want[1]) and np.array_equal(f16_bits(bias[sel]), want[2])
    del table, codes
    torch.cuda.empty_cache()


def test_lookup_launch_folded_into_two_grid_dimensions(e4q, oracle_lib):
    """2.2 M bags of dimension 4096 are 5.6e8 threads, more than 2^21 workgroups: almost all bags
    are empty (zeros), the few that are not sit at both ends and around the fold."""
    from paper_1911_02079_amd import synth

    dim, rows, n_bags = 4096, 64, 2_200_000
    say(f"folded lookup grid: {n_bags} bags x {dim} ({n_bags * dim * 4 / 2**30:.1f} GiB of output)")
    table = synth.gaussian_table(rows, dim, 0.1, seed=77, device="cuda")
    codes, scale, bias = e4q.quantize_rowwise_greedy(table, 50, 0.2)
    fold = (1 << 21) * 256 // (dim // 16)   # first bag of the grid's second row (16 elements per thread)
    busy = np.unique(np.array([0, 1, 5, fold - 2, fold - 1, fold, fold + 1, fold + 77, n_bags - 2, n_bags - 1]))
    rng = np.random.default_rng(5)
    lengths = np.zeros(n_bags, dtype=np.int64)
    lengths[busy] = rng.integers(1, 9, busy.size)
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    indices = rng.integers(0, rows, int(offsets[-1])).astype(np.int64)
    fused = e4q.fuse_rows(codes, scale, bias, dim)
    out = e4q.sparse_lengths_sum_fused(fused, dim, torch.from_numpy(indices).cuda(), torch.from_numpy(offsets).cuda())
    torch.cuda.synchronize()
    s_off = np.concatenate([[0], np.cumsum(lengths[busy])]).astype(np.int64)
    want = oracle_lib.sparse_lengths_sum(codes.cpu().numpy(), f16_bits(scale), f16_bits(bias), dim, indices, s_off)
    assert np.array_equal(out[torch.from_numpy(busy).cuda()].cpu().numpy().view(np.uint32), want.view(np.uint32))
    idle = np.setdiff1d(sample_rows(n_bags, 1, fold), busy)
    assert bool((out[torch.from_numpy(idle).cuda()] == 0).all())
    assert int((out != 0).any(dim=1).sum()) == busy.size  # every other bag is all zeros
    del out
    torch.cuda.empty_cache()
