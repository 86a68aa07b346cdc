"""ctypes binding of libbts.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbts.so")

EXPORTS = ["bts_create", "bts_destroy", "bts_last_hip_error", "topk_compress",
           "topk_compress_noalloc",
           "sparse_aggregate", "downlink_topk", "sparse_sgd_update", "bidir_step",
           "unidir_step", "bts_enable_diagnostics", "bidir_step_diag"]
# testing and measurement aids of the same library (include/bts_testing.h)
TESTING_EXPORTS = ["bts_profile_enable", "bts_profile_read", "bts_last_path", "bts_set_path",
                   "bts_testing_mark_dirty", "bts_testing_plan"]
# the measurement instrument, a library of its own (include/bts_probe.h)
PROBE_EXPORTS = ["bts_hbm_probe"]
_PROBE_PATH = os.path.join(_HERE, "libbts_probe.so")

_lib = None
_probe = None


class BtsError(RuntimeError):
    pass


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built HIP library.  It is never built here: run ``__graft_entry__.build()``
    (or ``python -m paper_2209_15203_amd.build``) first."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise BtsError(f"{_LIB_PATH} is missing: build the HIP library first "
                       f"(python -m paper_2209_15203_amd.build); there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, u32, u64, i32, f32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int32, C.c_float
    lib.bts_create.argtypes = [C.POINTER(vp), i32, u64, u32, u32, vp]
    lib.bts_destroy.argtypes = [vp]
    lib.bts_destroy.restype = None
    lib.bts_last_hip_error.argtypes = [vp]
    lib.topk_compress.argtypes = [vp, vp, vp, f32, vp, vp]
    lib.topk_compress_noalloc.argtypes = [vp, vp, i32, u64, u32, f32, vp, vp, vp]
    lib.sparse_aggregate.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.downlink_topk.argtypes = [vp, vp, vp, vp]
    lib.sparse_sgd_update.argtypes = [vp, vp, vp, u32, f32, vp]
    lib.bidir_step.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, vp, vp, vp, vp, vp]
    lib.unidir_step.argtypes = [vp, vp, vp, vp, vp, f32, f32, vp, vp, vp, vp, vp]
    lib.bts_enable_diagnostics.argtypes = [vp]
    lib.bidir_step_diag.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, vp, vp, vp, vp, vp]
    lib.bts_profile_enable.argtypes = [vp, C.c_int]
    lib.bts_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(u64)]
    lib.bts_last_path.argtypes = [vp, C.c_int, C.POINTER(u32), C.POINTER(u32)]
    lib.bts_set_path.argtypes = [vp, C.c_int]
    lib.bts_testing_mark_dirty.argtypes = [vp]
    lib.bts_testing_plan.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.POINTER(C.c_uint32)]
    for name in EXPORTS + TESTING_EXPORTS:
        if name != "bts_destroy":
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


PLAN_FIELDS = ("path", "single_pass_possible", "list_cap", "sample_stride", "sample_target",
               "rank_next", "tiles", "dir_entries", "waves_per_simd", "three_launch_possible",
               "three_launch_cap", "three_launch_tiles", "three_launch_dir_entries",
               "three_launch_blocks", "three_launch_hist_blocks", "lists")


def testing_plan(rows: int, d: int, K: int) -> dict:
    """How the library plans a select of this shape (host logic only: needs no GPU)."""
    out = (C.c_uint32 * 16)()
    rc = load_library().bts_testing_plan(rows, d, K, out)
    if rc != 0:
        raise BtsError(f"bts_testing_plan failed: {rc}")
    return dict(zip(PLAN_FIELDS, list(out)))


def load_probe_library():
    """Load libbts_probe.so (plain HBM streams; a measurement instrument, not the product)."""
    global _probe
    if _probe is None:
        if not os.path.exists(_PROBE_PATH):
            raise BtsError(f"{_PROBE_PATH} is missing: python -m paper_2209_15203_amd.build")
        lib = C.CDLL(_PROBE_PATH)
        lib.bts_hbm_probe.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_uint64,
                                      C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double)]
        lib.bts_hbm_probe.restype = C.c_int
        _probe = lib
    return _probe


def hbm_probe(kind: int, src: torch.Tensor, dst: torch.Tensor, waves_per_cu: int = 0,
              by_registers: bool = False, repeats: int = 5) -> float:
    """Mean milliseconds of one plain stream over src/dst (0 read, 1 copy, 2 fma-stream) on
    the current torch stream."""
    ms = C.c_double(0.0)
    n = min(src.numel(), dst.numel())
    rc = load_probe_library().bts_hbm_probe(
        C.c_void_p(torch.cuda.current_stream().cuda_stream), int(kind),
        _ptr(src, torch.float32, "src"), _ptr(dst, torch.float32, "dst"), C.c_uint64(n),
        int(waves_per_cu), int(by_registers), int(repeats), C.byref(ms))
    if rc != 0:
        raise BtsError(f"bts_hbm_probe failed: {rc}")
    return ms.value


_CODES = {-1: "BTS_EINVAL", -2: "BTS_ENOMEM", -3: "BTS_EHIP", -4: "BTS_ELIMIT"}


def _ptr(t: Optional[torch.Tensor], dtype, name: str, numel: Optional[int] = None):
    """Device pointer of a tensor argument.  numel: the elements the library will read or
    write there; a smaller tensor is refused here, on the host, because the kernels would
    run past its end."""
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous {dtype} tensor on the GPU")
    if numel is not None and t.numel() < numel:
        raise TypeError(f"{name} has {t.numel()} elements, the call needs {numel}")
    return C.c_void_p(t.data_ptr())


class BtsContext:
    """Owns a ``bts_ctx`` bound to the current torch HIP stream."""

    def __init__(self, N: int, d: int, K_up: int, K_dn: int,
                 stream: Optional[torch.cuda.Stream] = None):
        self._lib = load_library()
        self.N, self.d, self.K_up, self.K_dn = N, d, K_up, K_dn
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        rc = self._lib.bts_create(C.byref(h), N, d, K_up, K_dn, C.c_void_p(self.stream.cuda_stream))
        if rc != 0:
            raise BtsError(f"bts_create failed: {_CODES.get(rc, rc)}")
        self._h = h

    def check(self, rc: int, what: str) -> None:
        if rc != 0:
            hip = self._lib.bts_last_hip_error(self._h) if rc == -3 else 0
            raise BtsError(f"{what} failed: {_CODES.get(rc, rc)} (hip error {hip})")

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.bts_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # profiling of the dominant kernel
    def profile_enable(self, on: bool) -> None:
        self.check(self._lib.bts_profile_enable(self._h, int(on)), "bts_profile_enable")

    def profile_read(self) -> Tuple[float, int]:
        ms, n = C.c_double(0.0), C.c_uint64(0)
        self.check(self._lib.bts_profile_read(self._h, C.byref(ms), C.byref(n)), "bts_profile_read")
        return ms.value, n.value

    def enable_diagnostics(self) -> None:
        self.check(self._lib.bts_enable_diagnostics(self._h), "bts_enable_diagnostics")

    def set_path(self, mode: int) -> None:
        """0 = by shape, 1 = dense path only, 2 = single-pass path wherever possible,
        3 = three-launch path wherever possible."""
        self.check(self._lib.bts_set_path(self._h, int(mode)), "bts_set_path")

    def testing_mark_dirty(self) -> None:
        """Testing aid: the next calls behave as after a call that failed half way."""
        self.check(self._lib.bts_testing_mark_dirty(self._h), "bts_testing_mark_dirty")

    def last_path(self, which: int) -> Tuple[int, int]:
        a, b = C.c_uint32(0), C.c_uint32(0)
        self.check(self._lib.bts_last_path(self._h, which, C.byref(a), C.byref(b)), "bts_last_path")
        return a.value, b.value


F32, U32 = torch.float32, torch.int32   # uint32 words travel in int32 tensors


def topk_compress(ctx: BtsContext, g, eps, alpha_in: float, up_idx, up_val) -> None:
    nd, nk = ctx.N * ctx.d, ctx.N * ctx.K_up
    ctx.check(ctx._lib.topk_compress(ctx._h, _ptr(g, F32, "g", nd), _ptr(eps, F32, "eps", nd),
                                     alpha_in, _ptr(up_idx, U32, "up_idx", nk),
                                     _ptr(up_val, F32, "up_val", nk)), "topk_compress")


def topk_compress_noalloc(g, eps, alpha_in: float, up_idx, up_val,
                          stream: Optional[torch.cuda.Stream] = None) -> None:
    """topk_compress without a context and without any allocation (fixed scratch, bounded
    shapes); the shape is taken from g (N x d) and up_idx (N x K_up)."""
    N, d = g.shape
    K_up = 0 if up_idx is None else up_idx.shape[1]
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = load_library().topk_compress_noalloc(
        _ptr(g, F32, "g", N * d), _ptr(eps, F32, "eps", N * d), N, d, K_up, alpha_in,
        _ptr(up_idx, U32, "up_idx", N * K_up), _ptr(up_val, F32, "up_val", N * K_up),
        C.c_void_p(st.cuda_stream))
    if rc != 0:
        what = _CODES.get(rc, f"hip error {-1000 - rc}" if rc <= -1000 else rc)
        raise BtsError(f"topk_compress_noalloc failed: {what}")


def sparse_aggregate(ctx: BtsContext, up_idx, up_val, p, delta, union_nnz=None) -> None:
    nk = ctx.N * ctx.K_up
    ctx.check(ctx._lib.sparse_aggregate(ctx._h, _ptr(up_idx, U32, "up_idx", nk),
                                        _ptr(up_val, F32, "up_val", nk),
                                        _ptr(p, F32, "p", ctx.N), _ptr(delta, F32, "delta", ctx.d),
                                        _ptr(union_nnz, U32, "union_nnz", 1)), "sparse_aggregate")


def downlink_topk(ctx: BtsContext, delta, dn_idx, dn_val) -> None:
    ctx.check(ctx._lib.downlink_topk(ctx._h, _ptr(delta, F32, "delta", ctx.d),
                                     _ptr(dn_idx, U32, "dn_idx", ctx.K_dn),
                                     _ptr(dn_val, F32, "dn_val", ctx.K_dn)), "downlink_topk")


def sparse_sgd_update(ctx: BtsContext, idx, val, K: int, alpha_out: float, w) -> None:
    ctx.check(ctx._lib.sparse_sgd_update(ctx._h, _ptr(idx, U32, "idx", K), _ptr(val, F32, "val", K),
                                         K, alpha_out, _ptr(w, F32, "w", ctx.d)),
              "sparse_sgd_update")


def _step_ptrs(ctx: BtsContext, g, eps, w, p, up_idx, up_val):
    nd, nk = ctx.N * ctx.d, ctx.N * ctx.K_up
    return (_ptr(g, F32, "g", nd), _ptr(eps, F32, "eps", nd), _ptr(w, F32, "w", ctx.d),
            _ptr(p, F32, "p", ctx.N), _ptr(up_idx, U32, "up_idx", nk),
            _ptr(up_val, F32, "up_val", nk))


def bidir_step(ctx: BtsContext, g, eps, delta, w, p, alpha_in: float, alpha_out: float,
               up_idx, up_val, dn_idx, dn_val, union_nnz=None) -> None:
    pg, pe, pw, pp, pui, puv = _step_ptrs(ctx, g, eps, w, p, up_idx, up_val)
    ctx.check(ctx._lib.bidir_step(ctx._h, pg, pe, _ptr(delta, F32, "delta", ctx.d), pw, pp,
                                  alpha_in, alpha_out, pui, puv,
                                  _ptr(dn_idx, U32, "dn_idx", ctx.K_dn),
                                  _ptr(dn_val, F32, "dn_val", ctx.K_dn),
                                  _ptr(union_nnz, U32, "union_nnz", 1)), "bidir_step")


def unidir_step(ctx: BtsContext, g, eps, w, p, alpha_in: float, alpha_out: float, up_idx, up_val,
                dn_idx=None, dn_val=None, dn_count=None) -> None:
    pg, pe, pw, pp, pui, puv = _step_ptrs(ctx, g, eps, w, p, up_idx, up_val)
    nk = ctx.N * ctx.K_up
    ctx.check(ctx._lib.unidir_step(ctx._h, pg, pe, pw, pp, alpha_in, alpha_out, pui, puv,
                                   _ptr(dn_idx, U32, "dn_idx", nk), _ptr(dn_val, F32, "dn_val", nk),
                                   _ptr(dn_count, U32, "dn_count", 1)), "unidir_step")


def bidir_step_diag(ctx: BtsContext, g, eps, delta, w, p, alpha_in: float, alpha_out: float,
                    up_idx, up_val, dn_idx, dn_val, diag) -> None:
    """diag: float64 tensor of 8 + N elements on the GPU."""
    pg, pe, pw, pp, pui, puv = _step_ptrs(ctx, g, eps, w, p, up_idx, up_val)
    ctx.check(ctx._lib.bidir_step_diag(ctx._h, pg, pe, _ptr(delta, F32, "delta", ctx.d), pw, pp,
                                       alpha_in, alpha_out, pui, puv,
                                       _ptr(dn_idx, U32, "dn_idx", ctx.K_dn),
                                       _ptr(dn_val, F32, "dn_val", ctx.K_dn),
                                       _ptr(diag, torch.float64, "diag", 8 + ctx.N)),
              "bidir_step_diag")
