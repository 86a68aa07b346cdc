"""CPU oracle for bidirectional Top_K SGD (Algorithm 2 of the paper).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product (the HIP library and
its Python binding) never does, and this package never imports the product.

The arithmetic lives in ``bts_oracle.cpp`` (plain C++: full stable sort for
Top_K, fixed worker order and one fused multiply-add per term for the
aggregation).  This file only compiles it with g++ and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bts_oracle.cpp")
_LIB = os.path.join(_HERE, "libbts_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared",
               "-fPIC", "-pthread", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized() -> str:
    """Compile the oracle together with sanitize_driver.cpp into one executable under
    AddressSanitizer and UndefinedBehaviorSanitizer (host code only) and return its path.
    The runtimes are linked statically so that a preloaded library cannot come before them."""
    exe = os.path.join(_HERE, "oracle_sanitized")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-static-libasan", "-static-libubsan", "-pthread", "-o", exe, _SRC,
           os.path.join(_HERE, "sanitize_driver.cpp")]
    subprocess.run(cmd, check=True)
    return exe


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    c = ctypes
    fp, up, u64p = c.c_void_p, c.c_void_p, c.c_void_p
    lib.oracle_topk.argtypes = [fp, c.c_uint64, c.c_uint64, up, fp, fp]
    lib.oracle_worker_stage.argtypes = [fp, fp, c.c_int32, c.c_uint64, c.c_float, c.c_uint64,
                                        up, fp, c.c_int32]
    lib.oracle_aggregate.argtypes = [up, fp, fp, c.c_int32, c.c_uint64, fp, c.c_uint64, u64p]
    lib.oracle_downlink.argtypes = [fp, c.c_uint64, c.c_uint64, up, fp]
    lib.oracle_update.argtypes = [up, fp, c.c_uint64, c.c_float, fp, c.c_uint64]
    lib.oracle_bidir_step.argtypes = [fp, fp, fp, fp, fp, c.c_int32, c.c_uint64, c.c_uint64,
                                      c.c_uint64, c.c_float, c.c_float, up, fp, up, fp, u64p,
                                      c.c_int32]
    lib.oracle_unidir_step.argtypes = [fp, fp, fp, fp, c.c_int32, c.c_uint64, c.c_uint64,
                                       c.c_float, c.c_float, up, fp, up, fp, u64p, c.c_int32]
    lib.oracle_unidir_step.restype = c.c_int
    lib.oracle_bidir_step_diag.argtypes = [fp, fp, fp, fp, fp, c.c_int32, c.c_uint64, c.c_uint64,
                                           c.c_uint64, c.c_float, c.c_float, up, fp, up, fp,
                                           c.c_void_p, c.c_int32]
    lib.oracle_bidir_step_diag.restype = c.c_int
    for f in (lib.oracle_topk, lib.oracle_worker_stage, lib.oracle_aggregate,
              lib.oracle_downlink, lib.oracle_update, lib.oracle_bidir_step):
        f.restype = c.c_int
    _lib = lib
    return lib


def _f32(a: np.ndarray, name: str) -> np.ndarray:
    if a.dtype != np.float32 or not a.flags.c_contiguous:
        raise TypeError(f"{name} must be a C-contiguous float32 array")
    return a


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def default_threads(N: int) -> int:
    return max(1, min(N, len(os.sched_getaffinity(0))))


def topk(x: np.ndarray, K: int, want_residual: bool = True
         ) -> Tuple[np.ndarray, np.ndarray, Optional[np.ndarray]]:
    """Top_K(x) as (indices ascending, values, residual x - Top_K(x))."""
    x = _f32(x, "x")
    d = x.shape[0]
    idx = np.empty(K, dtype=np.uint32)
    val = np.empty(K, dtype=np.float32)
    res = np.empty(d, dtype=np.float32) if want_residual else None
    rc = _load().oracle_topk(_ptr(x), d, K, _ptr(idx), _ptr(val), _ptr(res))
    if rc:
        raise ValueError(f"oracle_topk failed rc={rc}")
    return idx, val, res


def worker_stage(g: np.ndarray, eps: np.ndarray, alpha_in: float, K_up: int,
                 nthreads: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Worker lines of Algorithm 2; eps (N x d) is updated in place."""
    g, eps = _f32(g, "g"), _f32(eps, "eps")
    N, d = g.shape
    assert eps.shape == (N, d)
    up_idx = np.empty((N, K_up), dtype=np.uint32)
    up_val = np.empty((N, K_up), dtype=np.float32)
    nt = default_threads(N) if nthreads is None else nthreads
    rc = _load().oracle_worker_stage(_ptr(g), _ptr(eps), N, d, alpha_in, K_up, _ptr(up_idx),
                                     _ptr(up_val), nt)
    if rc:
        raise ValueError(f"oracle_worker_stage failed rc={rc}")
    return up_idx, up_val


def aggregate(up_idx: np.ndarray, up_val: np.ndarray, p: np.ndarray, delta: np.ndarray,
              want_union: bool = True) -> Optional[int]:
    """Server aggregation line of Algorithm 2; delta becomes g_t in place."""
    N, K_up = up_idx.shape
    assert up_idx.dtype == np.uint32 and up_idx.flags.c_contiguous
    up_val, p, delta = _f32(up_val, "up_val"), _f32(p, "p"), _f32(delta, "delta")
    nnz = ctypes.c_uint64(0)
    rc = _load().oracle_aggregate(_ptr(up_idx), _ptr(up_val), _ptr(p), N, K_up, _ptr(delta),
                                  delta.shape[0],
                                  ctypes.cast(ctypes.byref(nnz), ctypes.c_void_p)
                                  if want_union else None)
    if rc:
        raise ValueError(f"oracle_aggregate failed rc={rc}")
    return int(nnz.value) if want_union else None


def downlink(delta: np.ndarray, K_dn: int) -> Tuple[np.ndarray, np.ndarray]:
    """Server compression lines of Algorithm 2; delta (holding g_t) becomes the residual."""
    delta = _f32(delta, "delta")
    idx = np.empty(K_dn, dtype=np.uint32)
    val = np.empty(K_dn, dtype=np.float32)
    rc = _load().oracle_downlink(_ptr(delta), delta.shape[0], K_dn, _ptr(idx), _ptr(val))
    if rc:
        raise ValueError(f"oracle_downlink failed rc={rc}")
    return idx, val


def update(idx: np.ndarray, val: np.ndarray, alpha_out: float, w: np.ndarray) -> None:
    """Model update line of Algorithm 2 on the received pairs, in place."""
    assert idx.dtype == np.uint32 and idx.flags.c_contiguous
    val, w = _f32(val, "val"), _f32(w, "w")
    rc = _load().oracle_update(_ptr(idx), _ptr(val), idx.shape[0], alpha_out, _ptr(w),
                               w.shape[0])
    if rc:
        raise ValueError(f"oracle_update failed rc={rc}")


def bidir_step(g: np.ndarray, eps: np.ndarray, delta: np.ndarray, w: np.ndarray, p: np.ndarray,
               K_up: int, K_dn: int, alpha_in: float, alpha_out: float,
               nthreads: Optional[int] = None) -> dict:
    """One iteration of Algorithm 2; eps, delta, w are updated in place."""
    g, eps, delta, w, p = (_f32(g, "g"), _f32(eps, "eps"), _f32(delta, "delta"), _f32(w, "w"),
                           _f32(p, "p"))
    N, d = g.shape
    assert eps.shape == (N, d) and delta.shape == (d,) and w.shape == (d,) and p.shape == (N,)
    up_idx = np.empty((N, K_up), dtype=np.uint32)
    up_val = np.empty((N, K_up), dtype=np.float32)
    dn_idx = np.empty(K_dn, dtype=np.uint32)
    dn_val = np.empty(K_dn, dtype=np.float32)
    nnz = ctypes.c_uint64(0)
    nt = default_threads(N) if nthreads is None else nthreads
    rc = _load().oracle_bidir_step(_ptr(g), _ptr(eps), _ptr(delta), _ptr(w), _ptr(p), N, d,
                                   K_up, K_dn, alpha_in, alpha_out, _ptr(up_idx), _ptr(up_val),
                                   _ptr(dn_idx), _ptr(dn_val),
                                   ctypes.cast(ctypes.byref(nnz), ctypes.c_void_p), nt)
    if rc:
        raise ValueError(f"oracle_bidir_step failed rc={rc}")
    return {"up_idx": up_idx, "up_val": up_val, "dn_idx": dn_idx, "dn_val": dn_val,
            "union_nnz": int(nnz.value)}


def unidir_step(g: np.ndarray, eps: np.ndarray, w: np.ndarray, p: np.ndarray, K_up: int,
                alpha_in: float, alpha_out: float, nthreads: Optional[int] = None) -> dict:
    """One iteration of Algorithm 1 (unidirectional Top_K SGD); eps and w updated in place.
    The server's message g_t is returned sparse (named coordinates, ascending)."""
    g, eps, w, p = _f32(g, "g"), _f32(eps, "eps"), _f32(w, "w"), _f32(p, "p")
    N, d = g.shape
    assert eps.shape == (N, d) and w.shape == (d,) and p.shape == (N,)
    up_idx = np.empty((N, K_up), dtype=np.uint32)
    up_val = np.empty((N, K_up), dtype=np.float32)
    dn_idx = np.empty(N * K_up, dtype=np.uint32)
    dn_val = np.empty(N * K_up, dtype=np.float32)
    cnt = ctypes.c_uint64(0)
    nt = default_threads(N) if nthreads is None else nthreads
    rc = _load().oracle_unidir_step(_ptr(g), _ptr(eps), _ptr(w), _ptr(p), N, d, K_up, alpha_in,
                                    alpha_out, _ptr(up_idx), _ptr(up_val), _ptr(dn_idx),
                                    _ptr(dn_val),
                                    ctypes.cast(ctypes.byref(cnt), ctypes.c_void_p), nt)
    if rc:
        raise ValueError(f"oracle_unidir_step failed rc={rc}")
    n = int(cnt.value)
    return {"up_idx": up_idx, "up_val": up_val, "dn_idx": dn_idx[:n].copy(),
            "dn_val": dn_val[:n].copy(), "dn_count": n}


DIAG_FIELDS = ("rho", "rho_hat", "one_minus_gamma_max", "denominator", "rho_numerator",
               "rho_hat_numerator", "nnz_fraction", "one_minus_gamma_server")


def bidir_step_diag(g: np.ndarray, eps: np.ndarray, delta: np.ndarray, w: np.ndarray,
                    p: np.ndarray, K_up: int, K_dn: int, alpha_in: float, alpha_out: float,
                    nthreads: Optional[int] = None) -> dict:
    """One iteration of Algorithm 2 plus the per-step estimates of rho, rho_hat and 1-gamma
    (the constants of Assumptions 2, 5 and 6 the paper measures)."""
    g, eps, delta, w, p = (_f32(g, "g"), _f32(eps, "eps"), _f32(delta, "delta"), _f32(w, "w"),
                           _f32(p, "p"))
    N, d = g.shape
    up_idx = np.empty((N, K_up), dtype=np.uint32)
    up_val = np.empty((N, K_up), dtype=np.float32)
    dn_idx = np.empty(K_dn, dtype=np.uint32)
    dn_val = np.empty(K_dn, dtype=np.float32)
    diag = np.zeros(8 + N, dtype=np.float64)
    nt = default_threads(N) if nthreads is None else nthreads
    rc = _load().oracle_bidir_step_diag(_ptr(g), _ptr(eps), _ptr(delta), _ptr(w), _ptr(p), N, d,
                                        K_up, K_dn, alpha_in, alpha_out, _ptr(up_idx),
                                        _ptr(up_val), _ptr(dn_idx), _ptr(dn_val), _ptr(diag), nt)
    if rc:
        raise ValueError(f"oracle_bidir_step_diag failed rc={rc}")
    out = {"up_idx": up_idx, "up_val": up_val, "dn_idx": dn_idx, "dn_val": dn_val, "diag": diag}
    out.update({k: float(diag[i]) for i, k in enumerate(DIAG_FIELDS)})
    out["one_minus_gamma_workers"] = diag[8:].copy()
    return out
