"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
memset), so its calls can run on concurrent streams and can be captured into a HIP graph."""
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


def test_two_streams_at_once(e4q, oracle_lib):
    from paper_1911_02079_amd import synth

    a = synth.gaussian_table(200_000, 64, 0.1, seed=1, device="cuda")
    b = synth.mixture_table(100_000, 64, seed=2, device="cuda")
    out_a = e4q.alloc_outputs(200_000, 64, "cuda")
    out_b = (torch.empty((100_000, 32), dtype=torch.uint8, device="cuda"),
             torch.empty((100_000, 16), dtype=torch.float16, device="cuda"))
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    say("greedy on one stream, 16-means on another")
    for _ in range(3):
        e4q.quantize_rowwise_greedy(a, 200, 0.16, out=out_a, stream=s1)
        e4q.quantize_rowwise_kmeans16(b, 20, out=out_b, stream=s2)
    s1.synchronize()
    s2.synchronize()
    rows = np.arange(0, 200_000, 97)
    o = oracle_lib.quantize_rowwise_greedy(a[torch.from_numpy(rows).cuda()].cpu().numpy(), 200, 0.16)
    assert np.array_equal(out_a[0].cpu().numpy()[rows], o[0]) and np.array_equal(f16_bits(out_a[1])[rows], o[1])
    rows = np.arange(0, 100_000, 53)
    o = oracle_lib.quantize_rowwise_kmeans16(b[torch.from_numpy(rows).cuda()].cpu().numpy(), 20)
    assert np.array_equal(out_b[0].cpu().numpy()[rows], o[0]) and np.array_equal(f16_bits(out_b[1])[rows], o[1])


@pytest.mark.parametrize("rows,dim", [(70_003, 64), (40_001, 100)])
def test_capture_into_a_graph_and_replay(e4q, oracle_lib, rows, dim):
    """dim 64: the plain kernels; dim 100: the masked-tail kernels that stage rows through LDS."""
    from paper_1911_02079_amd import synth

    table = synth.outlier_table(rows, dim, seed=10, device="cuda")
    out = e4q.alloc_outputs(rows, dim, "cuda")
    xh = torch.empty((rows, dim), device="cuda")
    indices, offsets = synth.lookup_bags(rows, 5_000, 1, 20, device="cuda")
    pooled = torch.empty((5_000, dim), device="cuda")
    kidx = torch.empty((rows, (dim + 1) // 2), dtype=torch.uint8, device="cuda")
    kcb = torch.empty((rows, 16), dtype=torch.float16, device="cuda")
    kxh = torch.empty((rows, dim), device="cuda")

    def path():
        e4q.quantize_rowwise_greedy(table, 200, 0.16, out=out)
        e4q.dequantize(*out, dim, out=xh)
        e4q.sparse_lengths_sum(*out, dim, indices, offsets, out=pooled)
        e4q.quantize_rowwise_kmeans16(table, 5, out=(kidx, kcb))
        e4q.dequantize_codebook(kidx, kcb, dim, out=kxh)

    path()  # eager reference
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    say("capture quantize + dequantize + lookup")
    with torch.cuda.graph(graph, stream=side):
        path()
    torch.cuda.synchronize()
    for k in range(3):
        new = synth.outlier_table(rows, dim, seed=20 + k, device="cuda")
        table.copy_(new)
        path()
        torch.cuda.synchronize()
        eager = (out[0].clone(), out[1].clone(), out[2].clone(), xh.clone(), pooled.clone(), kidx.clone(), kcb.clone(),
                 kxh.clone())
        for t in (*out, xh, pooled, kidx, kcb, kxh):
            t.zero_()
        torch.cuda.synchronize()
        say(f"replay {k}")
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((*out, xh, pooled, kidx, kcb, kxh), eager):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), f"replay {k}"
    o = oracle_lib.quantize_rowwise_greedy(table[:2000].cpu().numpy(), 200, 0.16)
    assert np.array_equal(out[0][:2000].cpu().numpy(), o[0])


def test_capture_a_batch_into_a_graph_and_replay(e4q, oracle_lib):
    """The batch entry point under capture: 70 tables of dimension 64 go out as grouped launches whose table list is a
    kernel argument of several kilobytes (it is copied at capture time: the replays must not depend on the descriptors
    the call was given), three of dimension 100 as launches of their own."""
    from paper_1911_02079_amd import synth

    rng = np.random.default_rng(3)
    tables = [synth.gaussian_table(int(rng.integers(1, 900)), 64, 0.1, seed=40 + k, device="cuda") for k in range(70)]
    tables += [synth.gaussian_table(300 + k, 100, 0.1, seed=140 + k, device="cuda") for k in range(3)]
    outs = [e4q.alloc_outputs(t.shape[0], t.shape[1], "cuda") for t in tables]

    def path():
        e4q.quantize_rowwise_greedy_batch(tables, 50, 0.16, out=outs)

    path()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    say("capture a batch of 73 tables")
    with torch.cuda.graph(graph, stream=side):
        path()
    torch.cuda.synchronize()
    for k in range(3):
        for j, t in enumerate(tables):
            t.copy_(synth.gaussian_table(t.shape[0], t.shape[1], 0.1, seed=1000 * (k + 1) + j, device="cuda"))
        path()
        torch.cuda.synchronize()
        eager = [tuple(x.clone() for x in o) for o in outs]
        for o in outs:
            for x in o:
                x.zero_()
        torch.cuda.synchronize()
        say(f"replay {k}")
        graph.replay()
        torch.cuda.synchronize()
        for j, (o, want) in enumerate(zip(outs, eager)):
            for got, w in zip(o, want):
                assert torch.equal(got.view(torch.uint8), w.view(torch.uint8)), f"replay {k}, table {j}"
    for j in (0, 33, 69, 72):
        o = oracle_lib.quantize_rowwise_greedy(tables[j].cpu().numpy(), 50, 0.16)
        assert np.array_equal(outs[j][0].cpu().numpy(), o[0]) and np.array_equal(f16_bits(outs[j][1]), o[1])
