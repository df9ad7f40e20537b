"""Every thread layout of the greedy search, forced through the "greedy_layout" diagnostic option,
gives the oracle's result bit for bit: one row per lane, and L lanes per row with E contiguous
elements each, for every (E, L) the library compiles that can hold the row.  Without the option the
library picks one of them by its cost model, so most are otherwise reached only at particular
table sizes."""
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


def layouts_for(dim):
    """One row per lane where it exists, then every compiled (E, L) with the smallest power of two L that
    holds the row, plus one with twice that many lanes (lanes beyond the row hold no element); and the lane
    counts that are not powers of two: the smallest that holds the row, one more, and 3 where 2 would do; and the
    layouts with two groups of lanes per row, (E, L, True), for E = 8 and 16."""
    out = ["rpl"] if dim <= 224 else []
    for e in (8, 16, 32, 64, 128):
        l = 1
        while e * l < dim:
            l *= 2
        lmax = 32 if e == 128 else 64
        if l <= lmax:
            out.append((e, l))
            if 2 * l <= lmax and e in (8, 32):
                out.append((e, 2 * l))
        if e <= 16 and l <= 32:  # two groups of l lanes per row, one per candidate range of a trip
            out.append((e, l, True))
            if 2 * l <= 32 and e == 8:
                out.append((e, 2 * l, True))
        need = -(-dim // e)
        for lanes in sorted({need, need + 1, 3, 63}):
            if need <= lanes <= 64 and lanes & (lanes - 1) and (lanes <= need + 1 or e == 8):
                out.append((e, lanes))
    return out


@pytest.mark.parametrize("half", [False, True], ids=["f32", "f16"])
@pytest.mark.parametrize("dim", [1, 7, 8, 13, 16, 32, 64, 100, 128, 136, 150, 192, 199, 200, 223, 224, 250, 300, 320, 384, 768, 999, 1000, 1999, 3000])
def test_every_forced_layout_matches_the_oracle(e4q, oracle_lib, dim, half):
    from paper_1911_02079_amd import synth

    rows = 1_301
    table = synth.outlier_table(rows, dim, seed=500 + dim, device="cuda")
    if half:
        table = table.half()
    want = oracle_lib.quantize_rowwise_greedy(np.ascontiguousarray(table.cpu().numpy()), 200, 0.16)
    try:
        for layout in layouts_for(dim):
            say(f"forced layout {layout}: {rows} x {dim} {'f16' if half else 'f32'}")
            e4q.set_option("greedy_layout", e4q.greedy_layout_value(layout))
            codes, scale, bias = e4q.quantize_rowwise_greedy(table, 200, 0.16)
            torch.cuda.synchronize()
            assert np.array_equal(codes.cpu().numpy(), want[0]), f"codes differ with layout {layout}"
            assert np.array_equal(f16_bits(scale), want[1]) and np.array_equal(f16_bits(bias), want[2]), layout
    finally:
        e4q.set_option("greedy_layout", 0)


def test_forced_layout_applies_to_batches_and_plain_min_max(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    tables = [synth.gaussian_table(700 + 13 * k, 64, 0.1, seed=800 + k, device="cuda") for k in range(4)]
    try:
        for layout in ["rpl", (16, 4), (64, 1), (16, 5), (8, 11), (8, 8, True), (16, 4, True)]:
            for n_bins, ratio in [(100, 0.16), (200, 0.0)]:
                say(f"batch of 4 tables with forced layout {layout}, b={n_bins} r={ratio}")
                e4q.set_option("greedy_layout", e4q.greedy_layout_value(layout))
                outs = e4q.quantize_rowwise_greedy_batch(tables, n_bins, ratio)
                torch.cuda.synchronize()
                for t, (codes, scale, bias) in zip(tables, outs):
                    want = oracle_lib.quantize_rowwise_greedy(t.cpu().numpy(), n_bins, ratio)
                    assert np.array_equal(codes.cpu().numpy(), want[0])
                    assert np.array_equal(f16_bits(scale), want[1]) and np.array_equal(f16_bits(bias), want[2])
    finally:
        e4q.set_option("greedy_layout", 0)


def test_a_layout_too_small_for_the_row_is_refused(e4q):
    table = torch.zeros((10, 256), device="cuda")
    try:
        e4q.set_option("greedy_layout", e4q.greedy_layout_value((8, 4)))
        with pytest.raises(e4q.E4QError) as err:
            e4q.quantize_rowwise_greedy(table, 200, 0.16)
        assert err.value.code == -8
    finally:
        e4q.set_option("greedy_layout", 0)


@pytest.mark.parametrize("waves", [1, 4])
def test_forced_workgroup_sizes_match_the_oracle(e4q, oracle_lib, waves):
    """The kernels that give a row a lane of its own run in one-wave or four-wave workgroups, normally chosen from the
    row count; both sizes, forced through the "workgroup_waves" option, on row counts around whole workgroups: the
    greedy search (single table, dimension with and without a masked tail, and a grouped batch) and 16-means."""
    from helpers import oracle_kmeans_in_parallel
    from paper_1911_02079_amd import synth

    try:
        e4q.set_option("workgroup_waves", waves)
        e4q.set_option("greedy_layout", 1)
        for rows, dim in [(1, 64), (63, 64), (64, 32), (65, 128), (255, 64), (256, 64), (257, 200), (1000, 100), (4099, 64)]:
            say(f"{waves} wave(s) per workgroup: greedy {rows} x {dim}")
            table = synth.outlier_table(rows, dim, seed=600 + rows + dim, device="cuda")
            codes, scale, bias = e4q.quantize_rowwise_greedy(table, 100, 0.16)
            torch.cuda.synchronize()
            want = oracle_lib.quantize_rowwise_greedy(table.cpu().numpy(), 100, 0.16)
            assert np.array_equal(codes.cpu().numpy(), want[0]) and np.array_equal(f16_bits(scale), want[1]) and \
                np.array_equal(f16_bits(bias), want[2]), (rows, dim)
        e4q.set_option("greedy_layout", 0)
        tables = [synth.gaussian_table(r, 64, 0.1, seed=650 + r, device="cuda") for r in (1, 64, 65, 255, 256, 257, 700, 3000)]
        say(f"{waves} wave(s) per workgroup: batch of {len(tables)} tables")
        outs = e4q.quantize_rowwise_greedy_batch(tables, 100, 0.16)
        torch.cuda.synchronize()
        for t, (codes, scale, bias) in zip(tables, outs):
            want = oracle_lib.quantize_rowwise_greedy(t.cpu().numpy(), 100, 0.16)
            assert np.array_equal(codes.cpu().numpy(), want[0]) and np.array_equal(f16_bits(scale), want[1]) and \
                np.array_equal(f16_bits(bias), want[2]), tuple(t.shape)
        for rows, dim in [(1, 64), (64, 64), (65, 40), (255, 64), (257, 100), (1500, 64)]:
            say(f"{waves} wave(s) per workgroup: 16-means {rows} x {dim}")
            table = synth.mixture_table(rows, dim, seed=700 + rows, device="cuda")
            idx, cen = e4q.quantize_rowwise_kmeans16(table, 5)
            torch.cuda.synchronize()
            w_idx, w_cen = oracle_kmeans_in_parallel(oracle_lib, table.cpu().numpy(), 5)
            assert np.array_equal(idx.cpu().numpy(), w_idx) and np.array_equal(f16_bits(cen), w_cen), (rows, dim)
    finally:
        e4q.set_option("workgroup_waves", 0)
        e4q.set_option("greedy_layout", 0)
