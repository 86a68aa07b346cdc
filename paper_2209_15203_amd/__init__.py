"""MI355X-native bidirectional Top_K SGD step (Algorithm 2 of arxiv 2209.15203).

The product is ``libbts.so`` (hand-written HIP for gfx950, C ABI in ``include/bts.h``).
This package is a thin ctypes binding with the same entry points; it only marshals
arguments (tensor pointers, the current HIP stream) and raises on error codes.  There is
no CPU fallback: importing :mod:`paper_2209_15203_amd.binding` without the built library
fails loudly.
"""
from .binding import (BtsContext, BtsError, bidir_step, bidir_step_diag, downlink_topk, lib_path, load_library,
                      sparse_aggregate, sparse_sgd_update, topk_compress, topk_compress_noalloc,
                      unidir_step)

__all__ = ["BtsContext", "BtsError", "bidir_step", "bidir_step_diag", "downlink_topk", "lib_path", "load_library",
           "sparse_aggregate", "sparse_sgd_update", "topk_compress", "topk_compress_noalloc", "unidir_step"]
