"""ctypes loader for the CPU float64 oracle (``topk_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
``cpu_baseline`` leg.  The product package never imports this module, and this module never imports
the product package.  Every function here only marshals numpy arrays into the C entry points; all
arithmetic of the method is in ``topk_oracle.cpp``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "topk_oracle.cpp")
_LIB = os.path.join(_HERE, "libtopk_oracle.so")

P_CODES = {"2": 0, "4/3": 1}


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (-O2, OpenMP over rows).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             _SRC, "-o", _LIB])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i64 = ctypes.c_int64
        L.oracle_argsort_desc.argtypes = [f32p, i64, i64, i32p]
        L.oracle_argsort_desc.restype = ctypes.c_int
        for fn in (L.oracle_topk_mask, L.oracle_topkmag, L.oracle_topk_signed_mask,
                   L.oracle_topk_masked_value):
            fn.argtypes = [f32p, f32p, i64, i64, i64, ctypes.c_int, ctypes.c_double, f64p, f64p,
                           i32p, i64p]
            fn.restype = ctypes.c_int
        for fn in (L.oracle_topk_mask_f64, L.oracle_topkmag_f64, L.oracle_topk_signed_mask_f64,
                   L.oracle_topk_masked_value_f64):
            fn.argtypes = [f64p, f64p, i64, i64, i64, ctypes.c_int, ctypes.c_double, f64p, f64p,
                           i32p, i64p]
            fn.restype = ctypes.c_int
        L.oracle_topk_mask_dykstra.argtypes = [f32p, i64, i64, i64, ctypes.c_double, i64, f64p]
        L.oracle_topk_mask_dykstra.restype = ctypes.c_int
        L.oracle_topk_general.argtypes = [ctypes.c_int, f32p, f32p, i64, f32p, i64, i64, ctypes.c_int,
                                          ctypes.c_double, f64p, f64p]
        L.oracle_topk_general.restype = ctypes.c_int
        L.oracle_topk_general_f64.argtypes = [ctypes.c_int, f64p, f32p, i64, f64p, i64, i64,
                                              ctypes.c_int, ctypes.c_double, f64p, f64p]
        L.oracle_topk_general_f64.restype = ctypes.c_int
        L.oracle_pav.argtypes = [f64p, f64p, i64, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                 f64p, i64p]
        L.oracle_pav.restype = ctypes.c_int
        L.oracle_topk_value.argtypes = [ctypes.c_int, f64p, i64, i64, i64, ctypes.c_int,
                                        ctypes.c_double, f64p]
        L.oracle_topk_value.restype = ctypes.c_int
        L.oracle_max_threads.restype = ctypes.c_int
        L.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def p_code(p) -> int:
    """Map the regulariser exponent to the oracle's code (only p = 2 and p = 4/3 exist)."""
    p = float(p)
    if abs(p - 2.0) < 1e-9:
        return 0
    if abs(p - 4.0 / 3.0) < 1e-6:
        return 1
    raise ValueError(f"unsupported p = {p}")


def _ptr(a, ty):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ty))


def _as_rows(x, dtype=np.float32):
    x = np.ascontiguousarray(x, dtype=dtype)
    if x.ndim == 1:
        x = x[None, :]
    assert x.ndim == 2
    return x


def argsort_desc(z) -> np.ndarray:
    z2 = _as_rows(z)
    perm = np.empty(z2.shape, dtype=np.int32)
    rc = lib().oracle_argsort_desc(_ptr(z2, ctypes.c_float), z2.shape[0], z2.shape[1],
                                   _ptr(perm, ctypes.c_int32))
    if rc != 0:
        raise RuntimeError(f"oracle_argsort_desc failed: {rc}")
    return perm.reshape(np.shape(z))


def _run(fn, x, k, p, lam, tangent, want_perm, want_block, f64=False):
    dt, cty = (np.float64, ctypes.c_double) if f64 else (np.float32, ctypes.c_float)
    x2 = _as_rows(x, dt)
    rows, n = x2.shape
    t2 = None
    if tangent is not None:
        t2 = _as_rows(tangent, dt)
        assert t2.shape == x2.shape
    out = np.empty((rows, n), dtype=np.float64)
    jvp = np.empty((rows, n), dtype=np.float64) if t2 is not None else None
    perm = np.empty((rows, n), dtype=np.int32) if want_perm else None
    ab = np.empty((rows, 2), dtype=np.int64) if want_block else None
    rc = fn(_ptr(x2, cty), _ptr(t2, cty), rows, n, int(k), p_code(p),
            float(lam), _ptr(out, ctypes.c_double), _ptr(jvp, ctypes.c_double),
            _ptr(perm, ctypes.c_int32), _ptr(ab, ctypes.c_int64))
    if rc != 0:
        raise RuntimeError(f"oracle call failed: {rc}")
    shp = np.shape(x)
    res = {"out": out.reshape(shp)}
    if jvp is not None:
        res["jvp"] = jvp.reshape(shp)
    if perm is not None:
        res["perm"] = perm.reshape(shp)
    if ab is not None:
        res["block"] = ab if len(shp) == 2 else ab[0]
    return res


def topk_mask(theta, k, p, lam, tangent=None, want_perm=False, want_block=False, f64=False):
    """Relaxed top-k mask (phi = identity) of each row; float64 results in a dict.

    Inputs are taken as float32 (the library's input type) unless ``f64`` is set."""
    fn = lib().oracle_topk_mask_f64 if f64 else lib().oracle_topk_mask
    return _run(fn, theta, k, p, lam, tangent, want_perm, want_block, f64)


def topkmag(x, k, p, lam, tangent=None, want_perm=False, want_block=False, f64=False):
    """Relaxed top-k in magnitude (phi = x^2/2) of each row; float64 results in a dict."""
    fn = lib().oracle_topkmag_f64 if f64 else lib().oracle_topkmag
    return _run(fn, x, k, p, lam, tangent, want_perm, want_block, f64)


def topk_signed_mask(x, k, p, lam, tangent=None, want_perm=False, want_block=False, f64=False):
    """Signed relaxed top-k mask (phi = |x|, paper Sec. 4 on the OWL norm): float64 results."""
    fn = lib().oracle_topk_signed_mask_f64 if f64 else lib().oracle_topk_signed_mask
    return _run(fn, x, k, p, lam, tangent, want_perm, want_block, f64)


def topk_masked_value(x, k, p, lam, tangent=None, f64=False):
    """x o mask_R(|x|), the alternative top-k in magnitude of the paper's Sec. 7."""
    fn = lib().oracle_topk_masked_value_f64 if f64 else lib().oracle_topk_masked_value
    return _run(fn, x, k, p, lam, tangent, False, False, f64)


def topk_mask_dykstra(theta, k, lam, iters) -> np.ndarray:
    """Relaxed top-k mask, p = 2, after ``iters`` iterations of Dykstra's algorithm (Alg. 1)."""
    x2 = _as_rows(theta)
    out = np.empty(x2.shape, dtype=np.float64)
    rc = lib().oracle_topk_mask_dykstra(_ptr(x2, ctypes.c_float), x2.shape[0], x2.shape[1], int(k),
                                        float(lam), int(iters), _ptr(out, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"oracle_topk_mask_dykstra failed: {rc}")
    return out.reshape(np.shape(theta))


def topk_general(x, w, p, lam, phi: str = "id", tangent=None, f64=False):
    """Relaxed operator y_{phi,R}(x, w) for non-increasing weights w ([n], or one row per row of
    x) and its JVP in x: dict with "out" (and "jvp"), float64."""
    dt, cty = (np.float64, ctypes.c_double) if f64 else (np.float32, ctypes.c_float)
    x2 = _as_rows(x, dt)
    rows, n = x2.shape
    w2 = np.ascontiguousarray(w, dtype=np.float32)
    assert w2.shape in ((n,), (rows, n))
    stride = 0 if w2.ndim == 1 else n
    t2 = None if tangent is None else _as_rows(tangent, dt)
    out = np.empty((rows, n), dtype=np.float64)
    jvp = np.empty((rows, n), dtype=np.float64) if t2 is not None else None
    fn = lib().oracle_topk_general_f64 if f64 else lib().oracle_topk_general
    rc = fn({"id": 0, "half_sq": 1}[phi], _ptr(x2, cty), _ptr(w2, ctypes.c_float), stride,
            _ptr(t2, cty), rows, n, p_code(p), float(lam), _ptr(out, ctypes.c_double),
            _ptr(jvp, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"oracle_topk_general failed: {rc}")
    res = {"out": out.reshape(np.shape(x))}
    if jvp is not None:
        res["jvp"] = jvp.reshape(np.shape(x))
    return res


def value(x, k, p, lam, phi: str = "id") -> np.ndarray:
    """f_{phi,R}(x, 1_k) of each row (paper Prop. 2, the minimisation form), float64."""
    x = np.atleast_2d(np.ascontiguousarray(x, dtype=np.float64))
    out = np.empty(x.shape[0], dtype=np.float64)
    rc = lib().oracle_topk_value({"id": 0, "half_sq": 1, "abs": 2}[phi], _ptr(x, ctypes.c_double), x.shape[0],
                                 x.shape[1], int(k), p_code(p), float(lam), _ptr(out, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"oracle_topk_value failed: {rc}")
    return out


def fenchel_young_loss(theta, target, k, p, lam):
    """Smooth top-k loss of the paper's Sec. 6: l(x, t) = f_{phi,R}(x, 1_k) - <x, t> with phi = id,
    and its gradient in x, y - t.  Returns (loss per row, gradient), float64."""
    theta = np.atleast_2d(np.asarray(theta))
    target = np.atleast_2d(np.asarray(target, dtype=np.float64))
    f = value(theta, k, p, lam, "id")
    y = topk_mask(theta, k, p, lam, f64=(theta.dtype == np.float64))["out"].reshape(theta.shape)
    return f - (theta.astype(np.float64) * target).sum(axis=1), y - target


def pav(s, w, phi: str, p, lam):
    """Isotonic solve on an already sorted float64 vector with arbitrary weights.

    Returns (v, block_start) where block_start[i] is the first index of i's block."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    v = np.empty_like(s)
    bid = np.empty(s.shape, dtype=np.int64)
    rc = lib().oracle_pav(_ptr(s, ctypes.c_double), _ptr(w, ctypes.c_double), s.shape[0],
                          {"id": 0, "half_sq": 1}[phi], p_code(p), float(lam),
                          _ptr(v, ctypes.c_double), _ptr(bid, ctypes.c_int64))
    if rc != 0:
        raise RuntimeError(f"oracle_pav failed: {rc}")
    return v, bid


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def set_threads(t: int) -> None:
    lib().oracle_set_threads(int(t))
