"""The C-ABI library loads without a GPU and exports every symbol that include/e4q.h declares;
host-only entry points and argument validation behave as documented (no kernel is launched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "e4q.h")


@pytest.fixture(scope="module")
def lib():
    from paper_1911_02079_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        from paper_1911_02079_amd import build

        build.build_library()
    return binding.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(e4q_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ["e4q_quantize_rowwise_greedy", "e4q_dequantize", "e4q_quantize_rowwise_greedy_batch",
                 "e4q_greedy_iterations", "e4q_strerror", "e4q_last_hip_error", "e4q_version",
                 "e4q_quantize_rowwise_kmeans16", "e4q_dequantize_codebook", "e4q_sparse_lengths_sum", "e4q_fuse_rows",
                 "e4q_sparse_lengths_sum_fused", "e4q_fused_row_bytes", "e4q_set_option", "e4q_get_option",
                 "e4q_greedy_layout_cost"]:
        assert must in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in e4q.h but not exported by libe4q.so"


def test_version_and_strerror(lib):
    assert lib.e4q_version() >= 100
    for code in range(0, -9, -1):
        assert lib.e4q_strerror(code)
    assert b"unknown" in lib.e4q_strerror(-99)
    assert lib.e4q_last_hip_error() == b""


def test_greedy_iterations_host_helper(lib):
    assert lib.e4q_greedy_iterations(200, 0.16) == 32
    assert lib.e4q_greedy_iterations(100, 0.16) == 16
    assert lib.e4q_greedy_iterations(1000, 0.5) == 500
    assert lib.e4q_greedy_iterations(20, 0.4) == 8
    assert lib.e4q_greedy_iterations(200, 0.0) == 0
    assert lib.e4q_greedy_iterations(3, 0.999) == 2
    assert lib.e4q_greedy_iterations(0, 0.1) == -4
    assert lib.e4q_greedy_iterations(10, 1.0) == -4
    assert lib.e4q_greedy_iterations(10, float("nan")) == -4


def test_greedy_iterations_agrees_with_the_oracles_own_formula(lib, oracle_lib):
    for b in [1, 2, 7, 20, 100, 200, 1000, 4096]:
        for r in [0.0, 0.01, 0.16, 0.25, 0.4, 0.5, 0.75, 0.99]:
            assert lib.e4q_greedy_iterations(b, r) == oracle_lib.n_iter(b, r)


def test_validation_rejects_bad_arguments_before_any_launch(lib):
    """All of these return before touching the device, so they are safe without a GPU.
    Pointers are fake non-NULL values that are never dereferenced on a validation error."""
    p = ctypes.c_void_p(0x1000)
    q = lib.e4q_quantize_rowwise_greedy
    ok_args = dict(table=p, dtype=0, rows=10, dim=64, stride=64, nbits=4, n_bins=200, ratio=0.16,
                   codes=p, scale=p, bias=p)

    def call(**kw):
        a = dict(ok_args, **kw)
        return q(a["table"], a["dtype"], a["rows"], a["dim"], a["stride"], a["nbits"], a["n_bins"], a["ratio"],
                 a["codes"], a["scale"], a["bias"], None)

    assert call(nbits=3) == -3
    assert call(nbits=16) == -3
    assert call(n_bins=0) == -4
    assert call(ratio=1.0) == -4
    assert call(ratio=-0.1) == -4
    assert call(dtype=2) == -5
    assert call(rows=-1) == -2
    assert call(rows=2 ** 31 + 1) == -2
    assert call(dim=0) == -2
    assert call(dim=4097) == -2
    assert call(stride=63) == -2
    assert call(table=None) == -1
    assert call(codes=None) == -1
    assert call(scale=None) == -1
    assert call(bias=None) == -1
    assert call(table=ctypes.c_void_p(0x1002)) == -7
    assert call(rows=0, table=None, codes=None, scale=None, bias=None) == 0  # empty table: no-op

    dq = lib.e4q_dequantize
    assert dq(p, p, p, 10, 64, 5, p, None) == -3
    assert dq(p, p, p, -1, 64, 4, p, None) == -2
    assert dq(p, p, p, 10, 0, 4, p, None) == -2
    assert dq(None, p, p, 10, 64, 4, p, None) == -1
    assert dq(p, p, p, 10, 64, 4, None, None) == -1
    assert dq(None, None, None, 0, 64, 4, None, None) == 0

    km = lib.e4q_quantize_rowwise_kmeans16
    assert km(p, 0, 10, 64, 64, -1, p, p, None) == -4
    assert km(p, 3, 10, 64, 64, 20, p, p, None) == -5
    assert km(p, 0, 10, 0, 64, 20, p, p, None) == -2
    assert km(p, 0, 10, 64, 32, 20, p, p, None) == -2
    assert km(None, 0, 10, 64, 64, 20, p, p, None) == -1
    assert km(p, 0, 10, 64, 64, 20, p, None, None) == -1
    assert km(None, 0, 0, 64, 64, 20, None, None, None) == 0
    dc = lib.e4q_dequantize_codebook
    assert dc(p, p, -1, 64, p, None) == -2
    assert dc(p, None, 10, 64, p, None) == -1
    assert dc(None, None, 0, 64, None, None) == 0

    sls = lib.e4q_sparse_lengths_sum
    p8 = ctypes.c_void_p(0x1000)
    assert sls(p, p, p, 10, 64, 8, p8, 8, 5, p8, 2, p, None) == -3
    assert sls(p, p, p, 10, 64, 4, p8, 2, 5, p8, 2, p, None) == -5
    assert sls(p, p, p, 10, 0, 4, p8, 8, 5, p8, 2, p, None) == -2
    assert sls(p, p, p, 10, 64, 4, p8, 8, -1, p8, 2, p, None) == -2
    assert sls(p, p, p, 10, 64, 4, None, 8, 5, p8, 2, p, None) == -1
    assert sls(p, p, p, 10, 64, 4, p8, 8, 5, None, 2, p, None) == -1
    assert sls(p, p, p, 10, 64, 4, p8, 8, 5, ctypes.c_void_p(0x1004), 2, p, None) == -7
    assert sls(None, None, None, 0, 64, 4, None, 8, 0, None, 0, None, None) == 0

    lib.e4q_fused_row_bytes.restype = ctypes.c_int64
    assert lib.e4q_fused_row_bytes(128) == 68 and lib.e4q_fused_row_bytes(64) == 36 and lib.e4q_fused_row_bytes(8) == 8
    assert lib.e4q_fused_row_bytes(5) == 8 and lib.e4q_fused_row_bytes(6) == 8 and lib.e4q_fused_row_bytes(0) == -2
    fr = lib.e4q_fuse_rows
    assert fr(p, p, p, 10, 128, 4, 66, p, None) == -2      # smaller than the record
    assert fr(p, p, p, 10, 128, 4, 69, p, None) == -2      # odd
    assert fr(p, p, p, 10, 128, 8, 68, p, None) == -3
    assert fr(p, p, p, 10, 128, 4, 68, None, None) == -1
    assert fr(None, None, None, 0, 128, 4, 68, None, None) == 0
    sf = lib.e4q_sparse_lengths_sum_fused
    assert sf(p, 10, 128, 4, 66, p8, 8, 5, p8, 2, p, None) == -2
    assert sf(p, 10, 128, 4, 68, p8, 3, 5, p8, 2, p, None) == -5
    assert sf(None, 10, 128, 4, 68, p8, 8, 5, p8, 2, p, None) == -1
    assert sf(None, 0, 128, 4, 68, None, 8, 0, None, 0, None, None) == 0

    from paper_1911_02079_amd.binding import TableDesc

    descs = (TableDesc * 2)()
    for d in descs:
        d.table, d.dtype, d.dim, d.rows, d.row_stride = 0x1000, 1, 32, 5, 32
        d.codes, d.scale_f16, d.bias_f16 = 0x1000, 0x1000, 0x1000
    descs[1].dim = 0
    assert lib.e4q_quantize_rowwise_greedy_batch(descs, 2, 4, 100, 0.16, None) == -2
    assert lib.e4q_quantize_rowwise_greedy_batch(descs, 0, 4, 100, 0.16, None) == 0
    assert lib.e4q_quantize_rowwise_greedy_batch(None, 2, 4, 100, 0.16, None) == -1
    assert lib.e4q_quantize_rowwise_greedy_batch(descs, 2, 3, 100, 0.16, None) == -3


def test_diagnostic_options(lib):
    """Options are validated on the host; a forced layout that cannot hold a row is refused before
    anything is launched (so this is safe without a GPU)."""
    lib.e4q_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int64]
    lib.e4q_get_option.argtypes = [ctypes.c_char_p]
    lib.e4q_get_option.restype = ctypes.c_int64
    for name in (b"greedy_layout", b"kmeans_force_scan", b"sls_nontemporal", b"workgroup_waves"):
        assert lib.e4q_get_option(name) == 0
    assert lib.e4q_set_option(b"no_such_option", 1) == -8
    assert lib.e4q_get_option(b"no_such_option") == -8
    assert lib.e4q_set_option(None, 1) == -8
    assert lib.e4q_set_option(b"kmeans_force_scan", 2) == -8
    assert lib.e4q_set_option(b"sls_nontemporal", -1) == -8
    for bad in (2, 3, 8, -1):
        assert lib.e4q_set_option(b"workgroup_waves", bad) == -8
    for good in (1, 4, 0):
        assert lib.e4q_set_option(b"workgroup_waves", good) == 0 and lib.e4q_get_option(b"workgroup_waves") == good
    twin = 1 << 16  # two groups of L lanes per row: E in {8, 16}, L a power of two up to 32
    for bad in [(8 << 8) | 65, (8 << 8) | 128, (12 << 8) | 4, (128 << 8) | 64, (8 << 8), 2, -1,
                twin | (32 << 8) | 2, twin | (8 << 8) | 64, twin | (8 << 8) | 3, twin, twin | 1, (2 << 16) | (8 << 8) | 4]:
        assert lib.e4q_set_option(b"greedy_layout", bad) == -8
        assert lib.e4q_get_option(b"greedy_layout") == 0
    p = ctypes.c_void_p(0x1000)
    q = lib.e4q_quantize_rowwise_greedy
    try:
        assert lib.e4q_set_option(b"greedy_layout", (8 << 8) | 4) == 0      # holds 32 elements per row
        assert lib.e4q_get_option(b"greedy_layout") == (8 << 8) | 4
        assert q(p, 0, 10, 64, 64, 4, 200, 0.16, p, p, p, None) == -8
        assert q(p, 0, 10, 64, 64, 3, 200, 0.16, p, p, p, None) == -3       # ordinary validation comes first
        assert lib.e4q_set_option(b"greedy_layout", twin | (8 << 8) | 4) == 0
        assert lib.e4q_get_option(b"greedy_layout") == twin | (8 << 8) | 4
        assert q(p, 0, 10, 64, 64, 4, 200, 0.16, p, p, p, None) == -8       # two groups of 4 lanes x 8 hold 32, not 64
        assert lib.e4q_set_option(b"greedy_layout", 1) == 0                  # one row per lane: dim <= 224
        assert q(p, 0, 10, 256, 256, 4, 200, 0.16, p, p, p, None) == -8
        from paper_1911_02079_amd.binding import TableDesc

        descs = (TableDesc * 2)()
        for d, dim in zip(descs, (64, 256)):
            d.table, d.dtype, d.dim, d.rows, d.row_stride = 0x1000, 0, dim, 5, dim
            d.codes, d.scale_f16, d.bias_f16 = 0x1000, 0x1000, 0x1000
        assert lib.e4q_quantize_rowwise_greedy_batch(descs, 2, 4, 100, 0.16, None) == -8
    finally:
        assert lib.e4q_set_option(b"greedy_layout", 0) == 0
    lib.e4q_greedy_layout_cost.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64]
    lib.e4q_greedy_layout_cost.restype = ctypes.c_double
    cost = lib.e4q_greedy_layout_cost
    assert cost(10_000_000, 128, 32, 1) > 0 and cost(10_000_000, 128, 32, (8 << 8) | 16) > cost(10_000_000, 128, 32, 1)
    assert cost(20_000, 128, 32, (16 << 8) | 8) < cost(20_000, 128, 32, 1)       # few rows: spread them over lanes
    assert cost(1000, 256, 32, 1) < 0 and cost(1000, 256, 32, (8 << 8) | 4) < 0 and cost(1000, 64, 32, 0) < 0
    # a lane count that is not a power of two: 384 elements on 3 lanes beat 4 lanes of which one idles
    assert 0 < cost(10_000_000, 384, 32, (128 << 8) | 3) < cost(10_000_000, 384, 32, (128 << 8) | 4)
    assert cost(1000, 384, 32, (64 << 8) | 5) < 0
    # few rows: a second group of lanes per row halves the chain of dependent trips; many rows: it only adds a range
    assert 0 < cost(1000, 64, 32, twin | (8 << 8) | 8) < cost(1000, 64, 32, (8 << 8) | 8)
    assert cost(1_000_000, 64, 32, twin | (8 << 8) | 8) > cost(1_000_000, 64, 32, (8 << 8) | 8)
    assert cost(1000, 64, 32, twin | (8 << 8) | 4) < 0
    assert lib.e4q_set_option(b"kmeans_force_scan", 1) == 0 and lib.e4q_get_option(b"kmeans_force_scan") == 1
    assert lib.e4q_set_option(b"kmeans_force_scan", 0) == 0


def test_binding_checks_caller_supplied_outputs():
    """The checks run before the library is called; CPU tensors are refused first, so the shape and
    type checks are exercised on the private helper."""
    import torch

    from paper_1911_02079_amd import binding

    dev = torch.device("cpu")
    good = torch.empty((4, 32), dtype=torch.uint8)
    with pytest.raises(ValueError):
        binding._check_out(good, torch.uint8, (4, 32), torch.device("cpu"), "codes")  # not a GPU tensor
    assert binding.greedy_layout_value(None) == 0 and binding.greedy_layout_value("rpl") == 1
    assert binding.greedy_layout_value("64,2") == (64 << 8) | 2 and binding.greedy_layout_value((8, 16)) == (8 << 8) | 16
    assert binding.greedy_layout_value("8,4,twin") == (1 << 16) | (8 << 8) | 4 == binding.greedy_layout_value((8, 4, True))
    assert "2 groups" in binding.greedy_layout_name((1 << 16) | (8 << 8) | 4) and binding.greedy_layout_name(1) == "one row per lane"
    with pytest.raises(ValueError):
        binding.greedy_layout_value("8,4,5")
    del dev


def test_binding_refuses_cpu_tensors():
    import torch

    import paper_1911_02079_amd as e4q

    with pytest.raises(ValueError):
        e4q.quantize_rowwise_greedy(torch.zeros(4, 8))
