"""Row-wise greedy 4-bit quantization of embedding tables on MI355X (arXiv 1911.02079).

The product is `libe4q.so` (hand-written HIP kernels behind the C ABI of `include/e4q.h`);
this package holds its sources (`csrc/`), the build step (`build.py`), a ctypes binding with the
same entry-point names (`binding.py`, imported lazily so that the package itself imports without
the built library) and seeded synthetic-table generators (`synth.py`).
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding", "quantize_rowwise_greedy", "quantize_rowwise_greedy_batch", "dequantize",
           "greedy_iterations", "quantize_rowwise_kmeans16", "dequantize_codebook", "sparse_lengths_sum",
           "fuse_rows", "sparse_lengths_sum_fused", "fused_row_bytes", "set_option", "get_option"]


def __getattr__(name):
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    if name in ("quantize_rowwise_greedy", "quantize_rowwise_greedy_batch", "dequantize", "greedy_iterations",
                "alloc_outputs", "packed_bytes", "load_library", "E4QError", "quantize_rowwise_kmeans16", "dequantize_codebook",
                "sparse_lengths_sum", "fuse_rows", "sparse_lengths_sum_fused", "fused_row_bytes", "set_option", "get_option",
                "greedy_layout_value", "greedy_layout_cost", "greedy_layout_name", "GREEDY_LAYOUT_TWIN"):
        import importlib

        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError(name)
