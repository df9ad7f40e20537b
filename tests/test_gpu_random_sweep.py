"""Randomized parity sweep: seeded cases whose shapes, row strides, buffer alignments, code widths, search settings,
forced thread layouts and value distributions are drawn at random (valid inputs only); every output is compared with the
CPU oracle bit for bit and the memory around the quantizer's outputs is checked for stray writes.  The parametrized tests
elsewhere cover the cases that were thought of; this covers combinations that were not.  (The same generator, run for
minutes on other seeds, compared more than 80 000 cases without a difference.)"""
import sys

import numpy as np
import pytest
import torch

from helpers import f16_bits, oracle_kmeans_in_parallel, oracle_rows_in_parallel

pytestmark = pytest.mark.gpu

GUARD = 64  # elements kept around every output buffer, which must come back untouched


def say(*a):
    print("[gpu-case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def e4q():
    assert torch.cuda.is_available()
    import paper_1911_02079_amd as pkg

    pkg.binding.load_library()
    return pkg


class Draw:
    """Random sources of one test: NumPy for shapes and settings, a device generator for the values."""

    def __init__(self, seed):
        self.rng = np.random.default_rng(seed)
        self.g = torch.Generator(device="cuda").manual_seed(seed)

    def dim(self):
        u = self.rng.random()
        if u < 0.55:
            return int(self.rng.integers(1, 261))
        if u < 0.85:
            return int(self.rng.integers(261, 1101))
        return int(self.rng.integers(1101, 4097))

    def table(self, rows, dim, half):
        """rows x dim view with a random row stride and a random element offset into its buffer (so the base is
        not always 16-byte aligned), filled from one of seven value families."""
        rng, g = self.rng, self.g
        kind = int(rng.integers(0, 7))
        stride = dim + int(rng.choice([0, 0, 0, 1, 3, 8, 13]))
        off = int(rng.choice([0, 0, 0, 1, 2, 4, 5]))
        buf = torch.empty(off + rows * stride + 8, device="cuda", dtype=torch.float32)
        buf.normal_(generator=g)
        t = torch.as_strided(buf, (rows, dim), (stride, 1), off)
        if kind == 0:    # Gaussian
            t.mul_(0.1)
        elif kind == 1:  # heavy tails around a per-row offset
            t.copy_(torch.sign(t) * t.abs().pow(2) * 0.05 + torch.rand((rows, 1), device="cuda", generator=g) - 0.5)
        elif kind == 2:  # a handful of distinct values: many exact ties
            t.copy_(torch.round(t * 2) / 4)
        elif kind == 3:  # tiny magnitudes (binary16 subnormal scales)
            t.mul_(1e-6)
        elif kind == 4:  # large magnitudes
            t.mul_(300.0)
        elif kind == 5:  # 2 % outliers
            m = torch.rand((rows, dim), device="cuda", generator=g) < 0.02
            t.copy_(torch.where(m, t * 30, t * 0.05))
        else:            # constant rows, rows of zeros of either and of both signs
            t.mul_(0.1)
            if rows > 3:
                t[0] = 0.25
                t[1] = 0.0
                t[2] = -0.0
            if dim > 2 and rows > 4:
                t[3, : dim // 2] = 0.0
                t[3, dim // 2:] = -0.0
        if half:
            hb = torch.empty(off + rows * stride + 8, device="cuda", dtype=torch.float16)
            th = torch.as_strided(hb, (rows, dim), (stride, 1), off)
            th.copy_(t)
            return th, f"kind={kind} stride={stride} off={off}"
        return t, f"kind={kind} stride={stride} off={off}"


def guarded(shape, dtype, fill, off_elems):
    n = int(np.prod(shape))
    buf = torch.full((GUARD + off_elems + n + GUARD,), fill, dtype=dtype, device="cuda")
    return buf, buf[GUARD + off_elems: GUARD + off_elems + n].view(shape), (GUARD + off_elems, n)


def untouched(buf, span, fill):
    start, n = span
    return bool((buf[:start] == fill).all()) and bool((buf[start + n:] == fill).all())


def layouts_for(dim):
    """Values of the `greedy_layout` option that can hold a row of `dim` elements: automatic (three times as likely),
    one row per lane, for every E the fewest lanes, one lane more, and the next power of two, and for E = 8 and 16 the
    layout with two groups of lanes per row."""
    out = [0, 0, 0]
    if dim <= 224:
        out.append(1)
    for e in (8, 16, 32, 64, 128):
        lmin = (dim + e - 1) // e
        if lmin > 64:
            continue
        p2 = 1
        while p2 < lmin:
            p2 *= 2
        for lanes in {lmin, p2, min(64, lmin + 1)}:
            if lanes > 64 or ((lanes & (lanes - 1)) == 0 and e == 128 and lanes > 32):
                continue
            out.append((e << 8) | lanes)
        if e <= 16 and p2 <= 32:
            out.append((1 << 16) | (e << 8) | p2)  # two groups of p2 lanes, one per candidate range of a trip
    return out


def test_greedy_and_dequantize_random_cases(e4q, oracle_lib):
    d = Draw(20191105)
    rng = d.rng
    for k in range(240):
        dim, half = d.dim(), bool(rng.integers(0, 2))
        nbits = int(rng.choice([4, 4, 4, 2, 8]))
        n_bins = int(rng.choice([1, 2, 5, 37, 100, 200, 256]))
        ratio = float(rng.choice([0.0, 0.05, 0.16, 0.16, 0.5, 0.9]))
        n_iter = oracle_lib.n_iter(n_bins, ratio)
        rows = int(min(rng.integers(1, 4000), max(1, 40_000_000 // (dim * (1 + 2 * n_iter)))))
        layout = int(rng.choice(layouts_for(dim)))
        table, how = d.table(rows, dim, half)
        nb = oracle_lib.packed_bytes(dim, nbits)
        cbuf, codes, cspan = guarded((rows, nb), torch.uint8, 0xA5, int(rng.choice([0, 0, 1, 3, 4, 16])))
        sbuf, scale, sspan = guarded((rows,), torch.float16, 7.0, int(rng.integers(0, 2)))
        bbuf, bias, bspan = guarded((rows,), torch.float16, 7.0, int(rng.integers(0, 2)))
        say(f"random greedy {k}: {rows} x {dim} {'binary16' if half else 'binary32'} nbits={nbits} b={n_bins} r={ratio} "
            f"layout={e4q.greedy_layout_name(layout)} {how} codes at +{cspan[0] - GUARD}")
        e4q.set_option("greedy_layout", layout)
        try:
            e4q.quantize_rowwise_greedy(table, n_bins, ratio, nbits=nbits, out=(codes, scale, bias))
        finally:
            e4q.set_option("greedy_layout", 0)
        torch.cuda.synchronize()
        want = oracle_rows_in_parallel(oracle_lib, table.cpu().numpy(), n_bins, ratio, nbits=nbits)
        bad = np.flatnonzero((codes.cpu().numpy() != want[0]).any(axis=1) | (f16_bits(scale) != want[1]) |
                             (f16_bits(bias) != want[2]))
        assert bad.size == 0, f"case {k}: rows {bad[:8]} differ"
        assert untouched(cbuf, cspan, 0xA5) and untouched(sbuf, sspan, 7.0) and untouched(bbuf, bspan, 7.0), f"case {k}: stray write"
        xh = e4q.dequantize(codes, scale, bias, dim, nbits=nbits)
        assert np.array_equal(xh.cpu().numpy().view(np.uint32),
                              oracle_lib.dequantize(want[0], want[1], want[2], dim, nbits=nbits).view(np.uint32)), f"case {k}"


def test_kmeans16_random_cases(e4q, oracle_lib):
    d = Draw(20191106)
    rng = d.rng
    for k in range(80):
        dim, half = int(rng.integers(1, 301)), bool(rng.integers(0, 2))
        iters = int(rng.choice([0, 1, 3, 20]))
        rows = int(min(rng.integers(1, 3000), max(1, 3_000_000 // (dim * (1 + iters)))))
        table, how = d.table(rows, dim, half)
        say(f"random 16-means {k}: {rows} x {dim} {'binary16' if half else 'binary32'} rounds={iters} {how}")
        idx, cen = e4q.quantize_rowwise_kmeans16(table, iters)
        torch.cuda.synchronize()
        w_idx, w_cen = oracle_kmeans_in_parallel(oracle_lib, table.cpu().numpy(), iters)
        assert np.array_equal(idx.cpu().numpy(), w_idx) and np.array_equal(f16_bits(cen), w_cen), f"case {k}"
        xh = e4q.dequantize_codebook(idx, cen, dim)
        assert np.array_equal(xh.cpu().numpy().view(np.uint32),
                              oracle_lib.dequantize_codebook(w_idx, w_cen, dim).view(np.uint32)), f"case {k}"


def test_lookup_random_cases(e4q, oracle_lib):
    d = Draw(20191107)
    rng = d.rng
    for k in range(80):
        dim = int(rng.choice([int(rng.integers(1, 530)), int(rng.choice([8, 16, 32, 64, 128, 256, 512]))]))
        rows, n_bags = int(rng.integers(1, 5000)), int(rng.integers(1, 1500))
        max_len = int(rng.choice([1, 3, 4, 5, 8, 40, 200]))
        idx_dtype = [torch.int32, torch.int64][int(rng.integers(0, 2))]
        table, how = d.table(rows, dim, False)
        lengths = rng.integers(0, max_len + 1, n_bags)
        offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
        indices = rng.integers(0, rows, int(offsets[-1])).astype(np.int64)
        if indices.size and rng.random() < 0.5:  # some indices outside the table, on either side
            where = rng.integers(0, indices.size, max(1, indices.size // 20))
            indices[where[::2]] = rows + rng.integers(0, 3, where[::2].size)
            indices[where[1::2]] = -1 - rng.integers(0, 3, where[1::2].size)
        pitch = e4q.fused_row_bytes(dim) + int(rng.choice([0, 0, 2, 4, 6, 12, 60]))
        say(f"random lookup {k}: {rows} x {dim}, {n_bags} bags of up to {max_len}, {idx_dtype}, record pitch {pitch}, {how}")
        codes, scale, bias = e4q.quantize_rowwise_greedy(table, 20, 0.2)
        di, do = torch.from_numpy(indices).to("cuda", idx_dtype), torch.from_numpy(offsets).cuda()
        got = e4q.sparse_lengths_sum(codes, scale, bias, dim, di, do)
        torch.cuda.synchronize()
        want = oracle_lib.sparse_lengths_sum(codes.cpu().numpy(), f16_bits(scale), f16_bits(bias), dim, indices, offsets)
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), f"case {k}: three arrays"
        fused = e4q.fuse_rows(codes, scale, bias, dim, pitch)
        got = e4q.sparse_lengths_sum_fused(fused, dim, di, do)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), f"case {k}: fused records"


def test_batch_random_cases(e4q, oracle_lib):
    """Batches of 1 - 90 tables of up to three dimensions (some with a grouped launch, some without), rows from 0 to
    3 000 around the workgroup sizes, now and then one large table, mixed input types."""
    d = Draw(20191108)
    rng = d.rng
    for k in range(30):
        n = int(rng.integers(1, 90))
        dims = [int(x) for x in rng.choice([8, 16, 32, 64, 100, 128, 136, 40, 256], size=int(rng.integers(1, 4)), replace=False)]
        n_bins, ratio = int(rng.choice([5, 37, 100, 200])), float(rng.choice([0.0, 0.16, 0.5]))
        nbits = int(rng.choice([4, 4, 2, 8]))
        big = int(rng.integers(0, n)) if rng.random() < 0.3 else -1
        tables = []
        for t in range(n):
            dim = int(rng.choice(dims))
            rows = int(rng.choice([0, 1, 5, 63, 64, 65, 255, 256, 257, 1000, 3000])) if t != big else int(rng.integers(100_000, 700_000))
            half = bool(rng.integers(0, 2)) if rng.random() < 0.3 else False
            if rows == 0:
                tables.append(torch.empty((0, dim), device="cuda", dtype=torch.float16 if half else torch.float32))
            else:
                tables.append(d.table(rows, dim, half)[0])
        say(f"random batch {k}: {n} tables, dims {dims}, nbits={nbits} b={n_bins} r={ratio}, rows {[t.shape[0] for t in tables][:10]} ...")
        outs = e4q.quantize_rowwise_greedy_batch(tables, n_bins, ratio, nbits=nbits)
        torch.cuda.synchronize()
        for i, (t, o) in enumerate(zip(tables, outs)):
            if t.shape[0] == 0:
                continue
            if t.shape[0] > 20_000:  # the large table: both ends and a random sample of rows
                pick = np.unique(np.concatenate([np.arange(300), np.arange(t.shape[0] - 300, t.shape[0]),
                                                 rng.integers(0, t.shape[0], 3000)]))
                sel = torch.from_numpy(pick).cuda()
                t, o = t[sel], tuple(x[sel] for x in o)
            want = oracle_rows_in_parallel(oracle_lib, t.cpu().numpy(), n_bins, ratio, nbits=nbits)
            assert np.array_equal(o[0].cpu().numpy(), want[0]), f"case {k} table {i}"
            assert np.array_equal(f16_bits(o[1]), want[1]) and np.array_equal(f16_bits(o[2]), want[2]), f"case {k} table {i}"
