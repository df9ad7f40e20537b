"""GPU parity of e4q_sparse_lengths_sum against the CPU oracle: binary32 outputs compared bit for
bit (both sides add the de-quantized rows of a bag left to right in binary32)."""
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
    assert torch.cuda.is_available()
    import paper_1911_02079_amd as pkg

    pkg.binding.load_library()
    return pkg


def make_bags(rows, n_bags, max_len, seed, bad=0):
    rng = np.random.default_rng(seed)
    lengths = rng.integers(0, max_len + 1, n_bags)
    lengths[rng.integers(0, n_bags, max(1, n_bags // 8))] = 0
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    indices = rng.integers(0, rows, int(offsets[-1])).astype(np.int64)
    if bad and indices.size:
        where = rng.integers(0, indices.size, bad)
        indices[where[::2]] = rows + rng.integers(0, 3, where[::2].size)
        indices[where[1::2]] = -1 - rng.integers(0, 3, where[1::2].size)
    return indices, offsets


def check(e4q, oracle, table, indices, offsets, idx_dtype, label):
    dim = table.shape[1]
    say(f"{label}: table {tuple(table.shape)}, {offsets.size - 1} bags, {indices.size} indices, {idx_dtype}")
    codes, scale, bias = e4q.quantize_rowwise_greedy(table, 50, 0.2)
    got = e4q.sparse_lengths_sum(codes, scale, bias, dim, torch.from_numpy(indices).to("cuda", idx_dtype),
                                 torch.from_numpy(offsets).cuda())
    torch.cuda.synchronize()
    want = oracle.sparse_lengths_sum(codes.cpu().numpy(), f16_bits(scale), f16_bits(bias), dim, indices, offsets)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), label
    # the same lookup over fused records: smallest record, and a padded pitch
    for pitch in (e4q.fused_row_bytes(dim), e4q.fused_row_bytes(dim) + 6, 2 * ((dim + 1) // 2 + 5)):
        fused = e4q.fuse_rows(codes, scale, bias, dim, pitch)
        got = e4q.sparse_lengths_sum_fused(fused, dim, torch.from_numpy(indices).to("cuda", idx_dtype),
                                           torch.from_numpy(offsets).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(fused.cpu().numpy(), oracle.fuse_rows(codes.cpu().numpy(), f16_bits(scale), f16_bits(bias),
                                                                    dim, pitch)), f"{label} fuse pitch={pitch}"
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), f"{label} fused pitch={pitch}"


@pytest.mark.parametrize("idx_dtype", [torch.int64, torch.int32])
@pytest.mark.parametrize("dim", [8, 24, 64, 128, 256, 13, 100, 1, 7, 50, 127, 130])
def test_random_bags(e4q, oracle_lib, dim, idx_dtype):
    from paper_1911_02079_amd import synth

    t = synth.outlier_table(3_000, dim, seed=dim, device="cuda")
    indices, offsets = make_bags(3_000, 777, 40, seed=dim, bad=40)
    check(e4q, oracle_lib, t, indices, offsets, idx_dtype, f"dim={dim}")


def test_long_and_short_bags(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.gaussian_table(5_000, 64, 0.1, seed=1, device="cuda")
    lengths = np.array([0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 1000, 0, 4097, 1], dtype=np.int64)
    offsets = np.concatenate([[0], np.cumsum(lengths)])
    indices = np.random.default_rng(2).integers(0, 5_000, int(offsets[-1]))
    check(e4q, oracle_lib, t, indices.astype(np.int64), offsets.astype(np.int64), torch.int64, "lengths 0..4097")


def test_single_index_bags_equal_dequantize(e4q):
    from paper_1911_02079_amd import synth

    t = synth.gaussian_table(2_000, 128, 0.1, seed=3, device="cuda")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t)
    perm = torch.randperm(2_000, device="cuda")
    say("single-index bags")
    got = e4q.sparse_lengths_sum(codes, scale, bias, 128, perm, torch.arange(2_001, device="cuda"))
    assert torch.equal(got, e4q.dequantize(codes, scale, bias, 128)[perm])


def test_empty_and_malformed_inputs(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    t = synth.gaussian_table(100, 64, 0.1, seed=4, device="cuda")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t)
    say("no bags / no indices")
    z = torch.zeros(1, dtype=torch.int64, device="cuda")
    assert e4q.sparse_lengths_sum(codes, scale, bias, 64, torch.zeros(0, dtype=torch.int64, device="cuda"), z).shape == (0, 64)
    out = e4q.sparse_lengths_sum(codes, scale, bias, 64, torch.zeros(0, dtype=torch.int64, device="cuda"),
                                 torch.zeros(6, dtype=torch.int64, device="cuda"))
    assert out.shape == (5, 64) and bool((out == 0).all())
    say("offsets outside [0, n_indices] are clamped")
    indices = np.arange(10, dtype=np.int64)
    offsets = np.array([-5, 3, 2, 8, 50], dtype=np.int64)       # bag 1 is reversed (-> empty), bag 3 runs past the end
    clamped = np.array([[0, 3], [3, 3], [2, 8], [8, 10]], dtype=np.int64)
    got = e4q.sparse_lengths_sum(codes, scale, bias, 64, torch.from_numpy(indices).cuda(), torch.from_numpy(offsets).cuda())
    torch.cuda.synchronize()
    for b, (lo, hi) in enumerate(clamped):
        want = oracle_lib.sparse_lengths_sum(codes.cpu().numpy(), f16_bits(scale), f16_bits(bias), 64, indices[lo:hi],
                                             np.array([0, hi - lo], dtype=np.int64))
        assert np.array_equal(got[b].cpu().numpy(), want[0])
    with pytest.raises(e4q.E4QError):
        e4q.sparse_lengths_sum(codes, scale, bias, 64, torch.from_numpy(indices).cuda(), torch.from_numpy(offsets).cuda(), nbits=8)


def test_full_size_lookup_sampled_bags(e4q, oracle_lib):
    """The benchmark's lookup workload (10 M x 128 table, 2^20 bags, 1..64 indices per bag): every
    64th bag is recomputed by the oracle."""
    from paper_1911_02079_amd import synth

    rows, dim, n_bags = 10_000_000, 128, 1 << 20
    t = synth.laplace_offset_table(rows, dim, device="cuda")
    codes, scale, bias = e4q.quantize_rowwise_greedy(t)
    del t
    indices, offsets = synth.lookup_bags(rows, n_bags, device="cuda")
    say(f"full size: {n_bags} bags, {indices.numel()} indices")
    out = e4q.sparse_lengths_sum(codes, scale, bias, dim, indices, offsets)
    torch.cuda.synchronize()
    off = offsets.cpu().numpy()
    sample = np.arange(0, n_bags, 64)
    idx_host = indices.cpu().numpy()
    used = np.unique(np.concatenate([idx_host[off[b]:off[b + 1]] for b in sample]))
    remap = {int(r): k for k, r in enumerate(used)}
    sub = torch.from_numpy(used).cuda()
    s_codes, s_scale, s_bias = codes[sub].cpu().numpy(), f16_bits(scale[sub]), f16_bits(bias[sub])
    s_idx = np.concatenate([[remap[int(r)] for r in idx_host[off[b]:off[b + 1]]] for b in sample]).astype(np.int64)
    s_off = np.concatenate([[0], np.cumsum([off[b + 1] - off[b] for b in sample])]).astype(np.int64)
    want = oracle_lib.sparse_lengths_sum(s_codes, s_scale, s_bias, dim, s_idx, s_off)
    assert np.array_equal(out[torch.from_numpy(sample).cuda()].cpu().numpy(), want)
    say("full size: fused records, pitch 68 and 128, equal the three-array lookup on every bag")
    for pitch in (68, 128):
        fused = e4q.fuse_rows(codes, scale, bias, dim, pitch)
        assert torch.equal(e4q.sparse_lengths_sum_fused(fused, dim, indices, offsets), out)
        del fused


@pytest.mark.parametrize("dim", [128, 64, 8, 13])
def test_empty_table_with_non_empty_bags_gives_zeros(e4q, dim):
    """rows == 0: every index is outside the table, so every bag sums to +0 and nothing is read
    from the (absent) table -- for the three arrays and for fused records, whose pointer is NULL."""
    say(f"empty table, dim={dim}: 9 bags over 40 indices")
    codes = torch.empty((0, (dim + 1) // 2), dtype=torch.uint8, device="cuda")
    scale = torch.empty((0,), dtype=torch.float16, device="cuda")
    bias = torch.empty((0,), dtype=torch.float16, device="cuda")
    indices = torch.arange(-3, 37, dtype=torch.int64, device="cuda")
    offsets = torch.tensor([0, 0, 1, 5, 9, 17, 17, 30, 39, 40], dtype=torch.int64, device="cuda")
    for idx in (indices, indices.to(torch.int32)):
        out = torch.full((9, dim), float("nan"), device="cuda")
        e4q.sparse_lengths_sum(codes, scale, bias, dim, idx, offsets, out=out)
        torch.cuda.synchronize()
        assert bool((out == 0).all())
        pitch = e4q.fused_row_bytes(dim)
        fused = torch.empty((0, pitch), dtype=torch.uint8, device="cuda")
        out = torch.full((9, dim), float("nan"), device="cuda")
        e4q.sparse_lengths_sum_fused(fused, dim, idx, offsets, out=out)
        torch.cuda.synchronize()
        assert bool((out == 0).all())


def test_non_temporal_gathers_give_the_same_sums(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    for dim in (128, 72):
        t = synth.outlier_table(4_000, dim, seed=60 + dim, device="cuda")
        codes, scale, bias = e4q.quantize_rowwise_greedy(t, 50, 0.2)
        indices, offsets = make_bags(4_000, 500, 50, seed=61, bad=30)
        want = oracle_lib.sparse_lengths_sum(codes.cpu().numpy(), f16_bits(scale), f16_bits(bias), dim, indices, offsets)
        fused = e4q.fuse_rows(codes, scale, bias, dim)
        say(f"non-temporal gathers, dim={dim}")
        try:
            e4q.set_option("sls_nontemporal", 1)
            got = e4q.sparse_lengths_sum_fused(fused, dim, torch.from_numpy(indices).cuda(), torch.from_numpy(offsets).cuda())
            torch.cuda.synchronize()
        finally:
            e4q.set_option("sls_nontemporal", 0)
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))
