"""ctypes binding of libe4q.so -- argument marshalling only.

Every function here has the name of the C entry point it calls (minus the `e4q_` prefix) and
does nothing but check tensor types, allocate outputs with torch and pass device pointers, sizes
and the current HIP stream across the C ABI declared in `include/e4q.h`.  All arithmetic runs in
the HIP kernels.  There is no CPU fallback: without the built library, or with tensors that are
not on a GPU, these functions raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libe4q.so")

E4Q_F32, E4Q_F16 = 0, 1
_lib = None


class E4QError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libe4q error {code}: {text}")
        self.code = code


class TableDesc(ctypes.Structure):
    """Mirror of `e4q_table_desc`."""
    _fields_ = [("table", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("dim", ctypes.c_int32),
                ("rows", ctypes.c_int64), ("row_stride", ctypes.c_int64), ("codes", ctypes.c_void_p),
                ("scale_f16", ctypes.c_void_p), ("bias_f16", ctypes.c_void_p)]


def load_library() -> ctypes.CDLL:
    """Load libe4q.so; raises if it has not been built (python -m paper_1911_02079_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1911_02079_amd.build` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    lib.e4q_quantize_rowwise_greedy.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_int64,
                                                c.c_int32, c.c_int32, c.c_float, c.c_void_p, c.c_void_p,
                                                c.c_void_p, c.c_void_p]
    lib.e4q_quantize_rowwise_greedy.restype = c.c_int
    lib.e4q_quantize_rowwise_greedy_batch.argtypes = [c.POINTER(TableDesc), c.c_int32, c.c_int32, c.c_int32,
                                                      c.c_float, c.c_void_p]
    lib.e4q_quantize_rowwise_greedy_batch.restype = c.c_int
    lib.e4q_dequantize.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int32, c.c_int32,
                                   c.c_void_p, c.c_void_p]
    lib.e4q_dequantize.restype = c.c_int
    lib.e4q_quantize_rowwise_kmeans16.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_int64, c.c_int32,
                                                  c.c_void_p, c.c_void_p, c.c_void_p]
    lib.e4q_quantize_rowwise_kmeans16.restype = c.c_int
    lib.e4q_dequantize_codebook.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p]
    lib.e4q_dequantize_codebook.restype = c.c_int
    lib.e4q_sparse_lengths_sum.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int32, c.c_int32,
                                           c.c_void_p, c.c_int32, c.c_int64, c.c_void_p, c.c_int64, c.c_void_p,
                                           c.c_void_p]
    lib.e4q_sparse_lengths_sum.restype = c.c_int
    lib.e4q_fused_row_bytes.argtypes = [c.c_int32]
    lib.e4q_fused_row_bytes.restype = c.c_int64
    lib.e4q_fuse_rows.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_int64,
                                  c.c_void_p, c.c_void_p]
    lib.e4q_fuse_rows.restype = c.c_int
    lib.e4q_sparse_lengths_sum_fused.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_int64, c.c_void_p,
                                                 c.c_int32, c.c_int64, c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p]
    lib.e4q_sparse_lengths_sum_fused.restype = c.c_int
    lib.e4q_greedy_iterations.argtypes = [c.c_int32, c.c_float]
    lib.e4q_greedy_iterations.restype = c.c_int32
    lib.e4q_set_option.argtypes = [c.c_char_p, c.c_int64]
    lib.e4q_set_option.restype = c.c_int
    lib.e4q_get_option.argtypes = [c.c_char_p]
    lib.e4q_get_option.restype = c.c_int64
    lib.e4q_greedy_layout_cost.argtypes = [c.c_int64, c.c_int32, c.c_int32, c.c_int64]
    lib.e4q_greedy_layout_cost.restype = c.c_double
    lib.e4q_strerror.argtypes = [c.c_int]
    lib.e4q_strerror.restype = c.c_char_p
    lib.e4q_last_hip_error.argtypes = []
    lib.e4q_last_hip_error.restype = c.c_char_p
    lib.e4q_version.argtypes = []
    lib.e4q_version.restype = c.c_int
    _lib = lib
    return lib


def _check(code: int) -> None:
    if code != 0:
        lib = load_library()
        text = lib.e4q_strerror(code).decode()
        hip = lib.e4q_last_hip_error().decode()
        raise E4QError(code, text + (f" [{hip}]" if hip and code == -6 else ""))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return E4Q_F32
    if t.dtype == torch.float16:
        return E4Q_F16
    raise TypeError(f"table must be float32 or float16, got {t.dtype}")


def _check_table(t: torch.Tensor) -> None:
    if not t.is_cuda:
        raise ValueError("libe4q works on device memory only: the table must be a GPU tensor")
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("table must be 2-D with contiguous rows")


def _stream_ptr(stream: Optional[torch.cuda.Stream], device) -> int:
    s = stream if stream is not None else torch.cuda.current_stream(device)
    return int(s.cuda_stream)


def version() -> int:
    return int(load_library().e4q_version())


def strerror(code: int) -> str:
    return load_library().e4q_strerror(int(code)).decode()


def greedy_iterations(n_bins: int, ratio: float) -> int:
    n = int(load_library().e4q_greedy_iterations(int(n_bins), float(ratio)))
    if n < 0:
        _check(n)
    return n


def set_option(name: str, value: int) -> None:
    """e4q_set_option: a process-wide diagnostic switch ("greedy_layout", "workgroup_waves", "kmeans_force_scan",
    "sls_nontemporal"); see include/e4q.h."""
    _check(int(load_library().e4q_set_option(name.encode(), int(value))))


def get_option(name: str) -> int:
    v = int(load_library().e4q_get_option(name.encode()))
    if v < 0:
        _check(v)
    return v


def greedy_layout_cost(rows: int, dim: int, n_iter: int, layout) -> float:
    """e4q_greedy_layout_cost: the library's estimate (SIMD cycles) for one layout; negative if it does not fit."""
    value = layout if isinstance(layout, int) else greedy_layout_value(layout)
    return float(load_library().e4q_greedy_layout_cost(int(rows), int(dim), int(n_iter), value))


GREEDY_LAYOUT_TWIN = 1 << 16  # flag of a layout value: two groups of L lanes per row, one per candidate range of a trip


def greedy_layout_value(layout) -> int:
    """Value of the "greedy_layout" option: None or "auto" -> 0, "rpl" -> 1 (one row per lane),
    (E, L) or "E,L" -> (E << 8) | L, (E, L, True) or "E,L,twin" -> the same with the twin flag."""
    if layout is None or layout == "auto":
        return 0
    if layout == "rpl":
        return 1
    parts = layout.split(",") if isinstance(layout, str) else list(layout)
    twin = len(parts) == 3 and parts[2] in (True, 1, "twin", "1")
    if len(parts) not in (2, 3) or (len(parts) == 3 and not twin):
        raise ValueError('layout must be "auto", "rpl", "E,L" or "E,L,twin"')
    return (GREEDY_LAYOUT_TWIN if twin else 0) | (int(parts[0]) << 8) | int(parts[1])


def greedy_layout_name(value: int) -> str:
    """Readable form of a "greedy_layout" / "greedy_layout_chosen" value."""
    if value == 0:
        return "automatic"
    if value == 1:
        return "one row per lane"
    e, lanes = (value & ~GREEDY_LAYOUT_TWIN) >> 8, value & 0xFF
    if value & GREEDY_LAYOUT_TWIN:
        return f"E={e} elements x 2 groups of L={lanes} lanes per row (one group per candidate range)"
    return f"E={e} elements x L={lanes} lanes per row"


def packed_bytes(dim: int, nbits: int = 4) -> int:
    """Bytes of one row of codes: 8/nbits codes per byte."""
    per = 8 // nbits
    return (dim + per - 1) // per


def alloc_outputs(rows: int, dim: int, device, nbits: int = 4) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Output buffers of the layout the library writes: codes uint8 [rows, ceil(dim*nbits/8)],
    scale and bias float16 [rows]."""
    codes = torch.empty((rows, packed_bytes(dim, nbits)), dtype=torch.uint8, device=device)
    scale = torch.empty((rows,), dtype=torch.float16, device=device)
    bias = torch.empty((rows,), dtype=torch.float16, device=device)
    return codes, scale, bias


def _check_out(t: torch.Tensor, dtype: torch.dtype, shape: Tuple[int, ...], device, what: str) -> None:
    """A caller-supplied output buffer must be exactly what the kernels write: dense, of the right
    type and shape, on the table's device (a wrong one would be an out-of-bounds device write)."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.device != device:
        raise ValueError(f"{what} must be a GPU tensor on the input's device ({device})")
    if t.dtype != dtype:
        raise TypeError(f"{what} must be {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape) or not t.is_contiguous():
        raise ValueError(f"{what} must be a dense tensor of shape {tuple(shape)}, got {tuple(t.shape)} "
                         f"with strides {tuple(t.stride())}")


def _check_greedy_out(out, rows: int, dim: int, nbits: int, device) -> None:
    if nbits not in (2, 4, 8):
        raise E4QError(-3, strerror(-3))
    if len(out) != 3:
        raise ValueError("out must be (codes, scale_f16, bias_f16)")
    _check_out(out[0], torch.uint8, (rows, packed_bytes(dim, nbits)), device, "out codes")
    _check_out(out[1], torch.float16, (rows,), device, "out scale")
    _check_out(out[2], torch.float16, (rows,), device, "out bias")


def quantize_rowwise_greedy(table: torch.Tensor, n_bins: int = 200, ratio: float = 0.16, nbits: int = 4,
                            out: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None,
                            stream: Optional[torch.cuda.Stream] = None):
    """e4q_quantize_rowwise_greedy on a GPU tensor.  Returns (codes, scale_f16, bias_f16);
    asynchronous on the given (default: current) stream."""
    lib = load_library()
    _check_table(table)
    rows, dim = table.shape
    if out is not None:
        _check_greedy_out(out, rows, dim, nbits, table.device)
    codes, scale, bias = out if out is not None else alloc_outputs(rows, dim, table.device, nbits)
    with torch.cuda.device(table.device):
        rc = lib.e4q_quantize_rowwise_greedy(table.data_ptr(), _dtype_code(table), rows, dim,
                                             table.stride(0) if rows > 1 else max(dim, table.stride(0)),
                                             int(nbits), int(n_bins), float(ratio), codes.data_ptr(),
                                             scale.data_ptr(), bias.data_ptr(), _stream_ptr(stream, table.device))
    _check(rc)
    return codes, scale, bias


def quantize_rowwise_greedy_batch(tables: Sequence[torch.Tensor], n_bins: int = 200, ratio: float = 0.16,
                                  nbits: int = 4, out: Optional[List[Tuple[torch.Tensor, ...]]] = None,
                                  stream: Optional[torch.cuda.Stream] = None):
    """e4q_quantize_rowwise_greedy_batch: all tables in one launch sequence on one stream."""
    lib = load_library()
    if len(tables) == 0:
        return []
    for t in tables:
        _check_table(t)
    device = tables[0].device
    for t in tables:
        if t.device != device:
            raise ValueError("all tables of a batch must be on one device")
    if out is not None:
        if len(out) != len(tables):
            raise ValueError("out must hold one (codes, scale_f16, bias_f16) per table")
        for t, o in zip(tables, out):
            _check_greedy_out(o, t.shape[0], t.shape[1], nbits, device)
    outs = out if out is not None else [alloc_outputs(t.shape[0], t.shape[1], device, nbits) for t in tables]
    descs = (TableDesc * len(tables))()
    for d, t, (codes, scale, bias) in zip(descs, tables, outs):
        d.table, d.dtype, d.dim, d.rows = t.data_ptr(), _dtype_code(t), t.shape[1], t.shape[0]
        d.row_stride = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))
        d.codes, d.scale_f16, d.bias_f16 = codes.data_ptr(), scale.data_ptr(), bias.data_ptr()
    with torch.cuda.device(device):
        rc = lib.e4q_quantize_rowwise_greedy_batch(descs, len(tables), int(nbits), int(n_bins), float(ratio),
                                                   _stream_ptr(stream, device))
    _check(rc)
    return outs


def dequantize(codes: torch.Tensor, scale_f16: torch.Tensor, bias_f16: torch.Tensor, dim: int, nbits: int = 4,
               out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """e4q_dequantize: float32 [rows, dim] from packed codes and float16 scale/bias."""
    lib = load_library()
    if not (codes.is_cuda and scale_f16.is_cuda and bias_f16.is_cuda):
        raise ValueError("libe4q works on device memory only")
    if codes.dtype != torch.uint8 or scale_f16.dtype != torch.float16 or bias_f16.dtype != torch.float16:
        raise TypeError("codes must be uint8, scale and bias float16")
    if not (codes.is_contiguous() and scale_f16.is_contiguous() and bias_f16.is_contiguous()):
        raise ValueError("codes, scale and bias must be dense")
    rows = codes.shape[0]
    if nbits not in (2, 4, 8):
        raise E4QError(-3, load_library().e4q_strerror(-3).decode())
    if codes.shape[1] != packed_bytes(dim, nbits) or scale_f16.numel() != rows or bias_f16.numel() != rows:
        raise ValueError("shapes of codes / scale / bias do not match dim and nbits")
    if out is None:
        out = torch.empty((rows, dim), dtype=torch.float32, device=codes.device)
    elif out.dtype != torch.float32 or not out.is_contiguous() or tuple(out.shape) != (rows, dim):
        raise ValueError("out must be a dense float32 [rows, dim] tensor")
    with torch.cuda.device(codes.device):
        rc = lib.e4q_dequantize(codes.data_ptr(), scale_f16.data_ptr(), bias_f16.data_ptr(), rows, int(dim),
                                int(nbits), out.data_ptr(), _stream_ptr(stream, codes.device))
    _check(rc)
    return out


def quantize_rowwise_kmeans16(table: torch.Tensor, lloyd_iters: int = 20,
                              out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
                              stream: Optional[torch.cuda.Stream] = None):
    """e4q_quantize_rowwise_kmeans16.  Returns (idx uint8 [rows, ceil(dim/2)], centroids float16 [rows, 16])."""
    lib = load_library()
    _check_table(table)
    rows, dim = table.shape
    if out is None:
        out = (torch.empty((rows, (dim + 1) // 2), dtype=torch.uint8, device=table.device),
               torch.empty((rows, 16), dtype=torch.float16, device=table.device))
    else:
        if len(out) != 2:
            raise ValueError("out must be (idx, centroids_f16)")
        _check_out(out[0], torch.uint8, (rows, (dim + 1) // 2), table.device, "out idx")
        _check_out(out[1], torch.float16, (rows, 16), table.device, "out centroids")
    idx, cent = out
    with torch.cuda.device(table.device):
        rc = lib.e4q_quantize_rowwise_kmeans16(table.data_ptr(), _dtype_code(table), rows, dim,
                                               table.stride(0) if rows > 1 else max(dim, table.stride(0)),
                                               int(lloyd_iters), idx.data_ptr(), cent.data_ptr(),
                                               _stream_ptr(stream, table.device))
    _check(rc)
    return idx, cent


def dequantize_codebook(idx: torch.Tensor, centroids_f16: torch.Tensor, dim: int,
                        out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """e4q_dequantize_codebook: float32 [rows, dim] from packed indices and the float16 codebooks."""
    lib = load_library()
    if not (idx.is_cuda and centroids_f16.is_cuda):
        raise ValueError("libe4q works on device memory only")
    if idx.dtype != torch.uint8 or centroids_f16.dtype != torch.float16:
        raise TypeError("idx must be uint8 and centroids float16")
    rows = idx.shape[0]
    if not (idx.is_contiguous() and centroids_f16.is_contiguous()) or idx.shape[1] != (dim + 1) // 2 \
            or tuple(centroids_f16.shape) != (rows, 16):
        raise ValueError("idx must be dense [rows, ceil(dim/2)] and centroids dense [rows, 16]")
    if out is None:
        out = torch.empty((rows, dim), dtype=torch.float32, device=idx.device)
    elif out.dtype != torch.float32 or not out.is_contiguous() or tuple(out.shape) != (rows, dim):
        raise ValueError("out must be a dense float32 [rows, dim] tensor")
    with torch.cuda.device(idx.device):
        rc = lib.e4q_dequantize_codebook(idx.data_ptr(), centroids_f16.data_ptr(), rows, int(dim), out.data_ptr(),
                                         _stream_ptr(stream, idx.device))
    _check(rc)
    return out


def sparse_lengths_sum(codes: torch.Tensor, scale_f16: torch.Tensor, bias_f16: torch.Tensor, dim: int,
                       indices: torch.Tensor, offsets: torch.Tensor, nbits: int = 4,
                       out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """e4q_sparse_lengths_sum: float32 [n_bags, dim]; `indices` int32 or int64, `offsets` int64 [n_bags + 1]."""
    lib = load_library()
    for t in (codes, scale_f16, bias_f16, indices, offsets):
        if not t.is_cuda:
            raise ValueError("libe4q works on device memory only")
        if not t.is_contiguous():
            raise ValueError("all inputs must be dense")
    if codes.dtype != torch.uint8 or scale_f16.dtype != torch.float16 or bias_f16.dtype != torch.float16:
        raise TypeError("codes must be uint8, scale and bias float16")
    if indices.dtype not in (torch.int32, torch.int64) or offsets.dtype != torch.int64:
        raise TypeError("indices must be int32 or int64 and offsets int64")
    rows = codes.shape[0]
    if codes.shape[1] != (dim + 1) // 2 or scale_f16.numel() != rows or bias_f16.numel() != rows:
        raise ValueError("shapes of codes / scale / bias do not match dim")
    n_bags = offsets.numel() - 1
    if n_bags < 0:
        raise ValueError("offsets needs n_bags + 1 entries")
    if out is None:
        out = torch.empty((n_bags, dim), dtype=torch.float32, device=codes.device)
    elif out.dtype != torch.float32 or not out.is_contiguous() or tuple(out.shape) != (n_bags, dim):
        raise ValueError("out must be a dense float32 [n_bags, dim] tensor")
    with torch.cuda.device(codes.device):
        rc = lib.e4q_sparse_lengths_sum(codes.data_ptr(), scale_f16.data_ptr(), bias_f16.data_ptr(), rows, int(dim),
                                        int(nbits), indices.data_ptr(), indices.element_size(), indices.numel(),
                                        offsets.data_ptr(), n_bags, out.data_ptr(), _stream_ptr(stream, codes.device))
    _check(rc)
    return out


def fused_row_bytes(dim: int) -> int:
    n = int(load_library().e4q_fused_row_bytes(int(dim)))
    if n < 0:
        _check(n)
    return n


def fuse_rows(codes: torch.Tensor, scale_f16: torch.Tensor, bias_f16: torch.Tensor, dim: int,
              row_pitch: Optional[int] = None, nbits: int = 4, out: Optional[torch.Tensor] = None,
              stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """e4q_fuse_rows: uint8 [rows, row_pitch] records (codes, then scale and bias)."""
    lib = load_library()
    if not (codes.is_cuda and scale_f16.is_cuda and bias_f16.is_cuda):
        raise ValueError("libe4q works on device memory only")
    if codes.dtype != torch.uint8 or scale_f16.dtype != torch.float16 or bias_f16.dtype != torch.float16:
        raise TypeError("codes must be uint8, scale and bias float16")
    if not (codes.is_contiguous() and scale_f16.is_contiguous() and bias_f16.is_contiguous()):
        raise ValueError("codes, scale and bias must be dense")
    rows = codes.shape[0]
    if codes.shape[1] != (dim + 1) // 2 or scale_f16.numel() != rows or bias_f16.numel() != rows:
        raise ValueError("shapes of codes / scale / bias do not match dim")
    pitch = int(row_pitch) if row_pitch is not None else fused_row_bytes(dim)
    if out is None:
        out = torch.empty((rows, pitch), dtype=torch.uint8, device=codes.device)
    elif out.dtype != torch.uint8 or not out.is_contiguous() or tuple(out.shape) != (rows, pitch):
        raise ValueError("out must be a dense uint8 [rows, row_pitch] tensor")
    with torch.cuda.device(codes.device):
        rc = lib.e4q_fuse_rows(codes.data_ptr(), scale_f16.data_ptr(), bias_f16.data_ptr(), rows, int(dim), int(nbits),
                               pitch, out.data_ptr(), _stream_ptr(stream, codes.device))
    _check(rc)
    return out


def sparse_lengths_sum_fused(fused: torch.Tensor, dim: int, indices: torch.Tensor, offsets: torch.Tensor,
                             nbits: int = 4, out: Optional[torch.Tensor] = None,
                             stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """e4q_sparse_lengths_sum_fused on records written by fuse_rows (row pitch = fused.shape[1])."""
    lib = load_library()
    for t in (fused, indices, offsets):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("libe4q works on dense device memory only")
    if fused.dtype != torch.uint8 or fused.dim() != 2:
        raise TypeError("fused must be a uint8 [rows, row_pitch] tensor")
    if indices.dtype not in (torch.int32, torch.int64) or offsets.dtype != torch.int64:
        raise TypeError("indices must be int32 or int64 and offsets int64")
    rows, pitch = fused.shape
    n_bags = offsets.numel() - 1
    if n_bags < 0:
        raise ValueError("offsets needs n_bags + 1 entries")
    if out is None:
        out = torch.empty((n_bags, dim), dtype=torch.float32, device=fused.device)
    elif out.dtype != torch.float32 or not out.is_contiguous() or tuple(out.shape) != (n_bags, dim):
        raise ValueError("out must be a dense float32 [n_bags, dim] tensor")
    with torch.cuda.device(fused.device):
        rc = lib.e4q_sparse_lengths_sum_fused(fused.data_ptr(), rows, int(dim), int(nbits), pitch, indices.data_ptr(),
                                              indices.element_size(), indices.numel(), offsets.data_ptr(), n_bags,
                                              out.data_ptr(), _stream_ptr(stream, fused.device))
    _check(rc)
    return out
