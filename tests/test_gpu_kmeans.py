"""GPU parity of the codebook (row-wise 16-means) entry points against the CPU oracle.

Indices and codebook bit patterns are compared for exact equality on every row: both sides take
the nearest-centre decisions in binary32 and accumulate each cluster's binary64 sum in element
order, so any difference is a bug.
"""
import sys

import numpy as np
import pytest
import torch

from helpers import f16_bits, oracle_kmeans_in_parallel

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def e4q():
    assert torch.cuda.is_available()
    import paper_1911_02079_amd as pkg

    pkg.binding.load_library()
    return pkg


def compare(e4q, oracle, table, iters, label):
    say(f"{label}: shape={tuple(table.shape)} dtype={table.dtype} lloyd_iters={iters}")
    idx, cent = e4q.quantize_rowwise_kmeans16(table, iters)
    torch.cuda.synchronize()
    o_idx, o_cent = oracle_kmeans_in_parallel(oracle, table.cpu().numpy(), iters)
    g_cent = f16_bits(cent)
    bad = np.flatnonzero((idx.cpu().numpy() != o_idx).any(axis=1) | (g_cent != o_cent).any(axis=1))
    assert bad.size == 0, f"{label}: {bad.size} rows differ, first {bad[:5]}"
    dim = table.shape[1]
    xh = e4q.dequantize_codebook(idx, cent, dim)
    torch.cuda.synchronize()
    assert np.array_equal(xh.cpu().numpy(), oracle.dequantize_codebook(o_idx, o_cent, dim)), f"{label}: dequantize"
    return idx, cent


def test_config5_mixture_rows(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.mixture_table(20_011, 64, device="cuda")
    idx, cent = compare(e4q, oracle_lib, t, 20, "config5-reduced")
    xh = e4q.dequantize_codebook(idx, cent, 64)
    g = e4q.dequantize(*e4q.quantize_rowwise_greedy(t), 64)
    # the codebook beats uniform greedy quantization on mixture rows (Table 2: KMEANS < GREEDY)
    assert float(((t - xh) ** 2).sum()) < float(((t - g) ** 2).sum())


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("dim", list(range(24, 129, 8)))
def test_register_resident_dimensions(e4q, oracle_lib, dim, dtype):
    from paper_1911_02079_amd import synth

    t = synth.mixture_table(64 * 9 + 5, dim, seed=500 + dim, device="cuda").to(dtype)
    compare(e4q, oracle_lib, t, 20, f"rpl dim={dim}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("dim", [1, 2, 5, 8, 15, 16, 17, 18, 33, 63, 100, 127, 130, 200, 1000])
def test_other_dimensions(e4q, oracle_lib, dim, dtype):
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(64 * 3 + 7, dim, seed=600 + dim, device="cuda").to(dtype)
    compare(e4q, oracle_lib, t, 6, f"any dim={dim}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("dim", [17, 19, 23, 25, 39, 50, 57, 71, 100, 121, 127])
def test_masked_tail_dimensions(e4q, oracle_lib, dim, dtype):
    """16 < dim < 128, not a multiple of 8: the register-resident kernel of the next multiple of 8 with a
    masked tail, several waves and a ragged last one; rows of (dim + 1) / 2 bytes, dense."""
    from paper_1911_02079_amd import synth

    t = synth.mixture_table(64 * 40 + 13, dim, seed=800 + dim, device="cuda").to(dtype)
    compare(e4q, oracle_lib, t, 9, f"masked tail dim={dim}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("dim", [129, 136, 192, 200, 256, 333, 1000, 4096])
def test_dimensions_above_128(e4q, oracle_lib, dim, dtype):
    """Rows that do not fit the register file are walked 64 elements at a time (whole and partial chunks,
    word and byte stores), several waves and a ragged last one."""
    from paper_1911_02079_amd import synth

    rows = 64 * 5 + 3 if dim <= 1000 else 67
    t = synth.mixture_table(rows, dim, seed=900 + dim, device="cuda").to(dtype)
    compare(e4q, oracle_lib, t, 7, f"chunked dim={dim}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("dim", [8, 16, 24, 64, 100, 200])
def test_signed_zeros_and_tiny_rows(e4q, oracle_lib, dim, dtype):
    """Sparse rows whose zeros carry either sign, rows of zeros only, and rows of binary32 subnormals or (for
    binary16 tables) binary16 subnormals: centres, stored codebook bits (signs of zero included) and indices."""
    from paper_1911_02079_amd import synth

    rows = 64 * 7 + 5
    g = torch.Generator(device="cuda").manual_seed(9300 + dim)
    t = synth.gaussian_table(rows, dim, 0.1, seed=9200 + dim, device="cuda")
    keep = torch.rand((rows, dim), device="cuda", generator=g) < 0.3
    negzero = torch.rand((rows, dim), device="cuda", generator=g) < 0.5
    t = torch.where(keep, t, torch.where(negzero, torch.full_like(t, -0.0), torch.zeros_like(t)))
    t[1::7] = t[1::7].abs()
    t[2::7] = -t[2::7].abs()
    t[3::7] = torch.where(negzero[3::7], torch.full_like(t[3::7], -0.0), torch.zeros_like(t[3::7]))
    tiny = 2.0 ** -20 if dtype == torch.float16 else 2.0 ** -140
    t[5::7] = (t[5::7].double() * tiny).float()
    compare(e4q, oracle_lib, t.to(dtype), 6, "signed zeros and tiny rows")


def test_outputs_do_not_overrun(e4q):
    """Guard bands around indices and codebooks stay untouched (masked-tail rows staged through LDS, chunked
    rows, plain rows; ragged row counts)."""
    from paper_1911_02079_amd import synth

    for dim, rows in ((64, 64 * 7 + 5), (50, 64 * 7 + 1), (101, 64 * 9 + 63), (23, 64 * 5 + 31), (200, 64 * 3 + 2),
                      (130, 64 * 3 + 2), (13, 77)):
        t = synth.mixture_table(rows, dim, seed=31 + dim, device="cuda")
        nb = (dim + 1) // 2
        say(f"guard bands dim={dim} rows={rows}")
        ibuf = torch.full((rows * nb + 256,), 0xA5, dtype=torch.uint8, device="cuda")
        cbuf = torch.full((rows * 16 + 128,), -3.0, dtype=torch.float16, device="cuda")
        out = (ibuf[128:128 + rows * nb].reshape(rows, nb), cbuf[64:64 + rows * 16].reshape(rows, 16))
        e4q.quantize_rowwise_kmeans16(t, 4, out=out)
        torch.cuda.synchronize()
        assert bool((ibuf[:128] == 0xA5).all()) and bool((ibuf[128 + rows * nb:] == 0xA5).all())
        assert bool((cbuf[:64] == -3.0).all()) and bool((cbuf[64 + rows * 16:] == -3.0).all())
        xbuf = torch.full((rows * dim + 64,), 7.0, device="cuda")
        e4q.dequantize_codebook(*out, dim, out=xbuf[32:32 + rows * dim].reshape(rows, dim))
        torch.cuda.synchronize()
        assert bool((xbuf[:32] == 7.0).all()) and bool((xbuf[32 + rows * dim:] == 7.0).all())


def random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        dim = int(rng.choice([rng.integers(1, 17), rng.integers(17, 129), rng.integers(129, 400), 8 * rng.integers(3, 17)]))
        rows = min(int(10 ** rng.uniform(2.0, 4.8)), 3_000_000 // dim)
        out.append((rows, dim, bool(rng.integers(0, 2)), int(rng.integers(0, 13))))
    return out


@pytest.mark.parametrize("rows,dim,half,iters", random_shapes(40, 19110207))
def test_random_shapes(e4q, oracle_lib, rows, dim, half, iters):
    """Seeded random (rows, dim, input type, rounds): whichever kernel the shape selects matches the oracle."""
    from paper_1911_02079_amd import synth

    t = synth.mixture_table(rows, dim, seed=7 * rows + dim, device="cuda")
    compare(e4q, oracle_lib, t.half() if half else t, iters, f"random shape rows={rows} dim={dim}")


@pytest.mark.parametrize("iters", [0, 1, 2, 7, 40])
def test_round_counts(e4q, oracle_lib, iters):
    from paper_1911_02079_amd import synth

    t = synth.gaussian_table(1_003, 64, 0.1, seed=70, device="cuda")
    compare(e4q, oracle_lib, t, iters, "rounds")


def test_edge_cases(e4q, oracle_lib):
    say("empty table")
    t = torch.empty((0, 64), device="cuda")
    idx, cent = e4q.quantize_rowwise_kmeans16(t)
    assert idx.shape == (0, 32) and cent.shape == (0, 16)
    assert e4q.dequantize_codebook(idx, cent, 64).shape == (0, 64)
    t = torch.zeros((70, 32), device="cuda")
    t[1] = 0.375
    t[2, :16] = 1.0
    t[3] = torch.arange(32, device="cuda").float() % 16 * 0.25 - 2.0   # populated 16-point grid
    t[4:] = torch.randn(66, 32, device="cuda") * 1e-6
    idx, cent = compare(e4q, oracle_lib, t, 20, "degenerate rows")
    assert torch.equal(e4q.dequantize_codebook(idx, cent, 32)[3], t[3])
    compare(e4q, oracle_lib, torch.randn(1, 64, device="cuda"), 20, "one row")
    say("strided rows and unaligned outputs")
    big = torch.randn(300, 100, device="cuda")
    view = big[:, 3:67]
    rows = 300
    ibuf = torch.zeros(rows * 32 + 1, dtype=torch.uint8, device="cuda")
    cbuf = torch.zeros(rows * 16 + 1, dtype=torch.float16, device="cuda")
    out = (ibuf[1:].reshape(rows, 32), cbuf[1:].reshape(rows, 16))
    e4q.quantize_rowwise_kmeans16(view, 20, out=out)
    torch.cuda.synchronize()
    o_idx, o_cent = oracle_lib.quantize_rowwise_kmeans16(np.ascontiguousarray(view.cpu().numpy()), 20)
    assert np.array_equal(out[0].cpu().numpy(), o_idx) and np.array_equal(f16_bits(out[1]), o_cent)
    assert int(ibuf[0]) == 0 and float(cbuf[0]) == 0.0
    xh = e4q.dequantize_codebook(out[0], out[1], 64)
    torch.cuda.synchronize()
    assert np.array_equal(xh.cpu().numpy(), oracle_lib.dequantize_codebook(o_idx, o_cent, 64))
    with pytest.raises(e4q.E4QError):
        e4q.quantize_rowwise_kmeans16(big, -1)


def clumped_rows(rows, dim, seed):
    """Rows made of a few tight clumps (widths of 0..8 units in the last place) at positions spread
    over seven decades, some clumps nearly on top of each other: centres that coincide, stay empty,
    or differ by one unit in the last place, which is where the order of the centres is at stake."""
    rng = np.random.default_rng(seed)
    out = np.empty((rows, dim), np.float32)
    for r in range(rows):
        k = int(rng.integers(2, 7))
        pos = (10.0 ** rng.uniform(-3, 4, size=k)) * rng.choice([-1.0, 1.0], size=k)
        if rng.random() < 0.5:
            pos[1] = np.float32(pos[0]) * (1.0 + rng.uniform(0, 4e-7))
        width = rng.choice([0, 1, 2, 8], size=k)
        which = rng.integers(0, k, size=dim)
        vals = pos[which].astype(np.float32)
        steps = rng.integers(0, 1 + width[which])
        for _ in range(8):
            m = steps > 0
            vals[m] = np.nextafter(vals[m], np.float32(np.inf))
            steps = steps - 1
        out[r] = vals
    return out


@pytest.mark.parametrize("dim", [24, 50, 64, 101, 128, 200])
def test_clumped_rows_and_forced_scan(e4q, oracle_lib, dim):
    """The bisection over ordered centres and the 16-centre scan give the oracle's result on rows with
    coinciding and nearly coinciding centres; the scan is forced through the diagnostic switch."""
    t = torch.from_numpy(clumped_rows(4_099, dim, 900 + dim)).cuda()
    idx, cent = compare(e4q, oracle_lib, t, 6, "clumped rows, bisection")
    from paper_1911_02079_amd import synth

    e4q.set_option("kmeans_force_scan", 1)
    try:
        idx2, cent2 = compare(e4q, oracle_lib, t, 6, "clumped rows, forced scan")
        assert torch.equal(idx, idx2) and torch.equal(cent.view(torch.int16), cent2.view(torch.int16))
        g = synth.mixture_table(5_003, dim, device="cuda")
        compare(e4q, oracle_lib, g, 20, "mixture rows, forced scan")
    finally:
        e4q.set_option("kmeans_force_scan", 0)


def test_full_config5_mixture_2M_x_64(e4q, oracle_lib):
    """Every row of the benchmark configuration, in the launch configuration bench.py times."""
    from paper_1911_02079_amd import synth

    t = synth.mixture_table(2_000_000, 64, device="cuda")
    idx, cent = compare(e4q, oracle_lib, t, 20, "config5")
    say("config5: indices are the first nearest entry of the stored codebook, on all rows")
    book = cent.float()
    for r0 in range(0, 2_000_000, 1 << 18):
        sl = slice(r0, min(2_000_000, r0 + (1 << 18)))
        q = torch.stack([idx[sl] & 0xF, idx[sl] >> 4], dim=2).reshape(-1, 64).long()
        d = (t[sl][:, :, None] - book[sl][:, None, :]).abs()
        assert torch.equal(d.argmin(dim=2), q) or bool((d.gather(2, q[:, :, None])[:, :, 0] == d.min(dim=2).values).all())
