"""CPU oracle for row-wise greedy 4-bit quantization (arXiv 1911.02079).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
CPU-baseline leg are the only callers.  The HIP library never imports this
package and this package never imports the HIP binding.

`oracle.build()` compiles `e4q_oracle.c`, `e4q_oracle_kmeans.c` and `e4q_oracle_sls.c` with gcc into `libe4q_oracle.so`
next to it; the functions below are thin ctypes wrappers taking and returning
NumPy arrays.  See the header of `e4q_oracle.c` for what is computed and which
passages of the paper each step follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("e4q_oracle.c", "e4q_oracle_kmeans.c", "e4q_oracle_sls.c")]
_LIB_PATH = os.path.join(_HERE, "libe4q_oracle.so")
_lib = None

# No -march=native: the library is built in one container and run in another.
_CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-mfma", "-msse4.1", "-std=c11",
           "-Wall", "-Wextra", "-shared", "-fPIC"]


def build(force: bool = True) -> str:
    """Compile the C oracle.  Returns the path of the shared library."""
    if (force or not os.path.exists(_LIB_PATH)
            or os.path.getmtime(_LIB_PATH) < max(os.path.getmtime(p) for p in _SRCS)):
        tmp = _LIB_PATH + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *_CFLAGS, "-o", tmp, *_SRCS, "-lm"], check=True)
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    lib.e4q_oracle_f32_to_f16.argtypes = [c.c_float]
    lib.e4q_oracle_f32_to_f16.restype = c.c_uint16
    lib.e4q_oracle_f16_to_f32.argtypes = [c.c_uint16]
    lib.e4q_oracle_f16_to_f32.restype = c.c_float
    lib.e4q_oracle_n_iter.argtypes = [c.c_int32, c.c_float]
    lib.e4q_oracle_n_iter.restype = c.c_int32
    lib.e4q_oracle_quantize_rowwise_greedy.argtypes = [
        c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_int64, c.c_int32, c.c_float, c.c_int,
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32]
    lib.e4q_oracle_quantize_rowwise_greedy.restype = c.c_int
    lib.e4q_oracle_range_loss.argtypes = [c.c_void_p, c.c_int32, c.c_float, c.c_float, c.c_int32]
    lib.e4q_oracle_range_loss.restype = c.c_float
    lib.e4q_oracle_brute_force_row.argtypes = [
        c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32]
    lib.e4q_oracle_brute_force_row.restype = c.c_int
    lib.e4q_oracle_dequantize.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int32,
                                          c.c_void_p, c.c_int32]
    lib.e4q_oracle_dequantize.restype = c.c_int
    lib.e4q_oracle_quantize_rowwise_kmeans16.argtypes = [
        c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.e4q_oracle_quantize_rowwise_kmeans16.restype = c.c_int
    lib.e4q_oracle_dequantize_codebook.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int32,
                                                   c.c_void_p]
    lib.e4q_oracle_dequantize_codebook.restype = c.c_int
    lib.e4q_oracle_sparse_lengths_sum.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int32,
                                                  c.c_void_p, c.c_void_p, c.c_int64, c.c_void_p]
    lib.e4q_oracle_sparse_lengths_sum.restype = c.c_int
    lib.e4q_oracle_fuse_rows.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int32, c.c_int64,
                                         c.c_void_p]
    lib.e4q_oracle_fuse_rows.restype = c.c_int
    _lib = lib
    return lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _as_table(table: np.ndarray):
    """Return (contiguous 2-D array, dtype code)."""
    if table.ndim != 2:
        raise ValueError("table must be 2-D")
    if table.dtype == np.float32:
        return np.ascontiguousarray(table), 0
    if table.dtype == np.float16:
        return np.ascontiguousarray(table), 1
    raise TypeError("table must be float32 or float16")


def f32_to_f16_bits(x) -> np.ndarray:
    """Oracle's own binary32 -> binary16 (RNE) conversion, elementwise; returns uint16 bit patterns."""
    lib = _load()
    x = np.asarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    flat_in, flat_out = x.reshape(-1), out.reshape(-1)
    for k in range(flat_in.size):
        flat_out[k] = lib.e4q_oracle_f32_to_f16(float(flat_in[k]))
    return out


def f16_bits_to_f32(h) -> np.ndarray:
    lib = _load()
    h = np.asarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    flat_in, flat_out = h.reshape(-1), out.reshape(-1)
    for k in range(flat_in.size):
        flat_out[k] = lib.e4q_oracle_f16_to_f32(int(flat_in[k]))
    return out


def n_iter(n_bins: int, ratio: float) -> int:
    return int(_load().e4q_oracle_n_iter(int(n_bins), float(ratio)))


def packed_bytes(dim: int, nbits: int = 4) -> int:
    """Bytes of one row of codes: 8/nbits codes per byte."""
    per = 8 // nbits
    return (dim + per - 1) // per


def quantize_rowwise_greedy(table: np.ndarray, n_bins: int = 200, ratio: float = 0.16,
                            literal_alg1: bool = False, return_search: bool = False, nbits: int = 4):
    """Algorithm 1 per row, then Eq. 1.  Returns (codes uint8 [rows, ceil(dim*nbits/8)],
    scale_f16 uint16 [rows], bias_f16 uint16 [rows]) and, if `return_search`, also
    (loss float32 [rows], ij int32 [rows, 2])."""
    lib = _load()
    t, dtype = _as_table(table)
    rows, dim = t.shape
    codes = np.zeros((rows, packed_bytes(dim, nbits)), dtype=np.uint8)
    scale = np.zeros(rows, dtype=np.uint16)
    bias = np.zeros(rows, dtype=np.uint16)
    loss = np.zeros(rows, dtype=np.float32)
    ij = np.zeros((rows, 2), dtype=np.int32)
    rc = lib.e4q_oracle_quantize_rowwise_greedy(_ptr(t), dtype, rows, dim, dim, int(n_bins),
                                                float(ratio), int(bool(literal_alg1)), _ptr(codes),
                                                _ptr(scale), _ptr(bias), _ptr(loss), _ptr(ij), int(nbits))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    if return_search:
        return codes, scale, bias, loss, ij
    return codes, scale, bias


def range_loss(x: np.ndarray, lo: float, hi: float, nbits: int = 4) -> float:
    """Eq. 2 for one row and an explicit range, in the oracle's binary32 arithmetic."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return float(_load().e4q_oracle_range_loss(_ptr(x), x.size, float(np.float32(lo)),
                                               float(np.float32(hi)), int(nbits)))


def brute_force_row(x: np.ndarray, n_bins: int, n_iter_: int, nbits: int = 4):
    """Minimum of Eq. 2 over every (i, j), i + j <= n_iter, of Algorithm 1's grid."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    loss = ctypes.c_float()
    bi, bj = ctypes.c_int32(), ctypes.c_int32()
    rc = _load().e4q_oracle_brute_force_row(_ptr(x), x.size, int(n_bins), int(n_iter_),
                                            ctypes.byref(loss), ctypes.byref(bi), ctypes.byref(bj), int(nbits))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return float(loss.value), int(bi.value), int(bj.value)


def dequantize(codes: np.ndarray, scale_f16: np.ndarray, bias_f16: np.ndarray, dim: int, nbits: int = 4) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scale_f16 = np.ascontiguousarray(scale_f16, dtype=np.uint16)
    bias_f16 = np.ascontiguousarray(bias_f16, dtype=np.uint16)
    rows = codes.shape[0]
    assert codes.shape[1] == packed_bytes(dim, nbits)
    out = np.empty((rows, dim), dtype=np.float32)
    rc = _load().e4q_oracle_dequantize(_ptr(codes), _ptr(scale_f16), _ptr(bias_f16), rows, dim, _ptr(out), int(nbits))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out


def quantize_rowwise_kmeans16(table: np.ndarray, lloyd_iters: int = 20, return_centres: bool = False):
    """Row-wise 16-entry codebook (Section 3, "Codebook-based Quantization").  Returns
    (idx uint8 [rows, ceil(dim/2)], centroids_f16 uint16 [rows, 16]) and, if `return_centres`,
    also the float32 centres before binary16 rounding."""
    t, dtype = _as_table(table)
    rows, dim = t.shape
    idx = np.zeros((rows, (dim + 1) // 2), dtype=np.uint8)
    cent = np.zeros((rows, 16), dtype=np.uint16)
    c32 = np.zeros((rows, 16), dtype=np.float32)
    rc = _load().e4q_oracle_quantize_rowwise_kmeans16(_ptr(t), dtype, rows, dim, dim, int(lloyd_iters),
                                                      _ptr(idx), _ptr(cent), _ptr(c32))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return (idx, cent, c32) if return_centres else (idx, cent)


def dequantize_codebook(idx: np.ndarray, centroids_f16: np.ndarray, dim: int) -> np.ndarray:
    """out[r][k] = codebook[r][index[r][k]] widened to float32."""
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    centroids_f16 = np.ascontiguousarray(centroids_f16, dtype=np.uint16)
    rows = idx.shape[0]
    assert idx.shape[1] == (dim + 1) // 2 and centroids_f16.shape == (rows, 16)
    out = np.empty((rows, dim), dtype=np.float32)
    rc = _load().e4q_oracle_dequantize_codebook(_ptr(idx), _ptr(centroids_f16), rows, dim, _ptr(out))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out


def sparse_lengths_sum(codes: np.ndarray, scale_f16: np.ndarray, bias_f16: np.ndarray, dim: int,
                       indices: np.ndarray, offsets: np.ndarray) -> np.ndarray:
    """4-bit SparseLengthsSum (Section 4): out[b] = sum of the de-quantized rows indices[offsets[b]:offsets[b+1]],
    accumulated left to right in binary32.  Returns float32 [n_bags, dim]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scale_f16 = np.ascontiguousarray(scale_f16, dtype=np.uint16)
    bias_f16 = np.ascontiguousarray(bias_f16, dtype=np.uint16)
    indices = np.ascontiguousarray(indices, dtype=np.int64)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    n_bags = offsets.size - 1
    assert n_bags >= 0 and (n_bags == 0 or (offsets[0] >= 0 and offsets[-1] <= indices.size))
    assert np.all(np.diff(offsets) >= 0)
    out = np.empty((n_bags, dim), dtype=np.float32)
    rc = _load().e4q_oracle_sparse_lengths_sum(_ptr(codes), _ptr(scale_f16), _ptr(bias_f16), codes.shape[0], dim,
                                               _ptr(indices), _ptr(offsets), n_bags, _ptr(out))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out


def fuse_rows(codes: np.ndarray, scale_f16: np.ndarray, bias_f16: np.ndarray, dim: int, row_pitch: int) -> np.ndarray:
    """Records of `row_pitch` bytes: codes, then (at the next even offset) binary16 scale and bias."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scale_f16 = np.ascontiguousarray(scale_f16, dtype=np.uint16)
    bias_f16 = np.ascontiguousarray(bias_f16, dtype=np.uint16)
    rows = codes.shape[0]
    out = np.full((rows, row_pitch), 0xEE, dtype=np.uint8)
    rc = _load().e4q_oracle_fuse_rows(_ptr(codes), _ptr(scale_f16), _ptr(bias_f16), rows, dim, row_pitch, _ptr(out))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out


def unpack_codes(codes: np.ndarray, dim: int, nbits: int = 4) -> np.ndarray:
    """Codes of a packed array: 8/nbits per byte, the first element in the lowest bits."""
    codes = np.asarray(codes, dtype=np.uint8)
    per = 8 // nbits
    out = np.empty((codes.shape[0], codes.shape[1] * per), dtype=np.uint8)
    for s_ in range(per):
        out[:, s_::per] = (codes >> (s_ * nbits)) & ((1 << nbits) - 1)
    return out[:, :dim]
