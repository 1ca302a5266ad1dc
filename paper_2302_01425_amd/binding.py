"""Thin ctypes binding over the C ABI of ``libsparse_topk.so`` (see ``include/sparse_topk.h``).

Argument marshalling only: torch supplies device memory and the current stream, every step of the
operators runs in the HIP kernels.  There is no fallback: if the library has not been built, or a
tensor is not a contiguous float32 tensor on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libsparse_topk.so")

(TOPK_OP_MASK_FWD, TOPK_OP_MASK_JVP, TOPK_OP_MAG_FWD, TOPK_OP_MAG_JVP, TOPK_OP_ARGSORT,
 TOPK_OP_SIGNED_MASK, TOPK_OP_MASKED_VALUE, TOPK_OP_GENERAL, TOPK_OP_MASK_SPARSE) = range(9)

EXPORTS = (
    "topk_mask_fwd", "topk_mask_jvp", "topk_mask_vjp", "topkmag_fwd", "topkmag_jvp", "topkmag_vjp",
    "topk_mask_sparse_fwd", "topk_general_fwd", "topk_general_jvp", "topk_mask_dykstra_fwd", "topk_signed_mask_fwd", "topk_signed_mask_jvp", "topk_masked_value_fwd", "topk_masked_value_jvp",
    "topk_mask_loss", "topk_argsort_desc", "topk_workspace_bytes", "topk_set_workspace",
    "topk_set_route", "topk_strerror", "topk_mask_jvp_static",
)

_lib = None


class TopkError(RuntimeError):
    pass


def load() -> ctypes.CDLL:
    """Load the shared library (built by ``paper_2302_01425_amd.build``); raise if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise TopkError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2302_01425_amd.build` "
            "(there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, dbl, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_double, ctypes.c_int
    L.topk_mask_fwd.argtypes = [vp, i64, i64, i64, dbl, dbl, vp, vp]
    L.topk_mask_jvp.argtypes = [vp, vp, i64, i64, i64, dbl, dbl, vp, vp, vp]
    L.topk_mask_jvp_static.argtypes = L.topk_mask_jvp.argtypes
    L.topk_mask_jvp_static.restype = ci
    L.topkmag_fwd.argtypes = [vp, i64, i64, i64, dbl, dbl, vp, vp]
    L.topkmag_jvp.argtypes = [vp, vp, i64, i64, i64, dbl, dbl, vp, vp, vp]
    for name in ("topk_signed_mask_fwd", "topk_masked_value_fwd"):
        getattr(L, name).argtypes = L.topk_mask_fwd.argtypes
        getattr(L, name).restype = ci
    for name in ("topk_signed_mask_jvp", "topk_masked_value_jvp"):
        getattr(L, name).argtypes = L.topk_mask_jvp.argtypes
        getattr(L, name).restype = ci
    L.topk_mask_sparse_fwd.argtypes = [vp, i64, i64, i64, dbl, dbl, i64, vp, vp, vp, vp]
    L.topk_mask_sparse_fwd.restype = ci
    L.topk_general_fwd.argtypes = [vp, vp, i64, i64, i64, ci, dbl, dbl, vp, vp]
    L.topk_general_fwd.restype = ci
    L.topk_general_jvp.argtypes = [vp, vp, i64, vp, i64, i64, ci, dbl, dbl, vp, vp, vp]
    L.topk_general_jvp.restype = ci
    L.topk_mask_dykstra_fwd.argtypes = [vp, i64, i64, i64, dbl, ci, vp, vp]
    L.topk_mask_dykstra_fwd.restype = ci
    L.topk_mask_vjp.argtypes = L.topk_mask_jvp.argtypes
    L.topkmag_vjp.argtypes = L.topkmag_jvp.argtypes
    L.topk_argsort_desc.argtypes = [vp, i64, i64, vp, vp]
    L.topk_mask_loss.argtypes = [vp, vp, i64, i64, i64, dbl, dbl, vp, vp, vp]
    L.topk_mask_loss.restype = ci
    for name in ("topk_mask_fwd", "topk_mask_jvp", "topk_mask_vjp", "topkmag_fwd", "topkmag_jvp",
                 "topkmag_vjp", "topk_argsort_desc"):
        getattr(L, name).restype = ci
    L.topk_workspace_bytes.argtypes = [ci, i64, i64, i64, dbl]
    L.topk_workspace_bytes.restype = ctypes.c_size_t
    L.topk_set_workspace.argtypes = [vp, ctypes.c_size_t]
    L.topk_set_workspace.restype = ci
    L.topk_set_route.argtypes = [ci, ci]
    L.topk_set_route.restype = ci
    L.topk_strerror.argtypes = [ci]
    L.topk_strerror.restype = ctypes.c_char_p
    _lib = L
    return L


def strerror(code: int) -> str:
    return load().topk_strerror(int(code)).decode()


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise TopkError(f"{what}: {strerror(rc)} (code {rc})")


def _dev_f32(t: torch.Tensor, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TopkError(f"{name} must be a tensor in GPU memory")
    if t.dtype != torch.float32 or not t.is_contiguous() or t.dim() != 2:
        raise TopkError(f"{name} must be a contiguous 2-D float32 tensor [rows, n]")
    return t


def _overlap(a: torch.Tensor, b: torch.Tensor) -> bool:
    a0, b0 = a.data_ptr(), b.data_ptr()
    return (a0 < b0 + b.numel() * b.element_size() and b0 < a0 + a.numel() * a.element_size()
            and a.numel() > 0 and b.numel() > 0)


def _like(t, ref: torch.Tensor, name: str, inputs=()) -> torch.Tensor:
    """A tensor the kernels read or write rows * n floats of: it must have the shape and the
    device of `ref` (the first input).  Outputs (`inputs` given) must not overlap any input."""
    t = _dev_f32(t, name)
    if tuple(t.shape) != tuple(ref.shape) or t.device != ref.device:
        raise TopkError(f"{name} must have the shape {tuple(ref.shape)} and the device {ref.device} "
                        f"of the first input (got {tuple(t.shape)} on {t.device})")
    for other in inputs:
        if _overlap(t, other):
            raise TopkError(f"{name} overlaps an input tensor (outputs must not alias inputs)")
    return t


def _out(t, ref: torch.Tensor, name: str, inputs) -> torch.Tensor:
    return torch.empty_like(ref) if t is None else _like(t, ref, name, inputs)


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


_ws_tensor = None
_ws_retired = []     # superseded workspaces, never freed (see ensure_workspace)


def workspace_bytes(op: int, rows: int, n: int, k: int, p: float) -> int:
    return int(load().topk_workspace_bytes(int(op), int(rows), int(n), int(k), float(p)))


def set_workspace(t: torch.Tensor | None) -> None:
    """Register a caller-owned uint8 GPU tensor as scratch memory (None unregisters).  The caller
    keeps it alive for as long as enqueued work or a captured graph may use it."""
    global _ws_tensor
    if t is None:
        _check(load().topk_set_workspace(None, 0), "topk_set_workspace")
        _ws_tensor = None
        return
    _check(load().topk_set_workspace(ctypes.c_void_p(t.data_ptr()), t.numel() * t.element_size()),
           "topk_set_workspace")
    _ws_tensor = t


def ensure_workspace(op: int, rows: int, n: int, k: int, p: float, device) -> None:
    """Allocate (once, growing) and register scratch memory large enough for this call.

    The library holds one raw pointer, and kernels already enqueued on any stream, as well as
    captured graphs, keep using the block that was registered when they were enqueued.  So a
    block that has been handed to the library is never freed: when a larger one is needed the
    device is synchronised first, the old block is retired (kept referenced until the process
    ends) and the new one registered.  During a stream capture nothing can be allocated or
    synchronised: size the workspace with one eager call of the same shape before capturing."""
    need = workspace_bytes(op, rows, n, k, p)
    if need == 0:
        return
    dev = torch.device(device)
    if dev.index is None:
        dev = torch.device("cuda", torch.cuda.current_device())
    if _ws_tensor is not None and _ws_tensor.numel() >= need and _ws_tensor.device == dev:
        return
    if torch.cuda.is_current_stream_capturing():
        raise TopkError("the workspace is too small for this call and cannot grow during a stream "
                        "capture: run the call once eagerly before capturing")
    torch.cuda.synchronize(dev)
    if _ws_tensor is not None:
        _ws_retired.append(_ws_tensor)
    set_workspace(torch.empty(need, dtype=torch.uint8, device=dev))


TOPK_ROUTE_LONG_ROWS, TOPK_ROUTE_SHORT_ROW_LANES, TOPK_ROUTE_SHORT_ROW_KERNEL = 0, 1, 2
TOPK_ROUTE_GENERAL_ROUNDS = 3
TOPK_SHORT_ROW_MAX, TOPK_GENERAL_ROW_MAX = 1024, 131072
(TOPK_LONG_ROWS_AUTO, TOPK_LONG_ROWS_SELECT, TOPK_LONG_ROWS_SORT, TOPK_LONG_ROWS_WIDE,
 TOPK_LONG_ROWS_ONE_LAUNCH_INDEXED) = range(5)
TOPK_SHORT_ROW_KERNEL_AUTO, TOPK_SHORT_ROW_KERNEL_INDEXED, TOPK_SHORT_ROW_KERNEL_GENERAL = 0, 1, 2


def set_route(which: int, value: int) -> None:
    """Test and tuning control of the library (see topk_set_route in the header)."""
    _check(load().topk_set_route(int(which), int(value)), "topk_set_route")


def topk_mask_fwd(theta, k, p, lam, out=None, stream=None):
    theta = _dev_f32(theta, "theta")
    rows, n = theta.shape
    out = _out(out, theta, "out", (theta,))
    ensure_workspace(TOPK_OP_MASK_FWD, rows, n, k, p, theta.device)
    _check(load().topk_mask_fwd(theta.data_ptr(), rows, n, int(k), float(p), float(lam),
                                out.data_ptr(), _stream(stream)), "topk_mask_fwd")
    return out


def topk_mask_jvp(theta, tangent, k, p, lam, out=None, jvp_out=None, want_out=True, stream=None):
    """Returns (out, jvp_out); out is None when want_out is False and no out tensor was given."""
    theta = _dev_f32(theta, "theta")
    tangent = _like(tangent, theta, "tangent")
    rows, n = theta.shape
    if out is not None or want_out:
        out = _out(out, theta, "out", (theta, tangent))
    jvp_out = _out(jvp_out, theta, "jvp_out", (theta, tangent))
    if out is not None and _overlap(out, jvp_out):
        raise TopkError("out and jvp_out overlap")
    ensure_workspace(TOPK_OP_MASK_JVP, rows, n, k, p, theta.device)
    _check(load().topk_mask_jvp(theta.data_ptr(), tangent.data_ptr(), rows, n, int(k), float(p),
                                float(lam), None if out is None else out.data_ptr(),
                                jvp_out.data_ptr(), _stream(stream)), "topk_mask_jvp")
    return out, jvp_out


def topk_mask_jvp_static(theta, tangent, k, p, lam, out, jvp_out, stream=None):
    """topk_mask_jvp on the library's static scratch: nothing is allocated here either, so every
    tensor (out may be None) comes from the caller.  Returns (out, jvp_out)."""
    theta = _dev_f32(theta, "theta")
    tangent = _like(tangent, theta, "tangent")
    rows, n = theta.shape
    if out is not None:
        out = _like(out, theta, "out", (theta, tangent))
    jvp_out = _like(jvp_out, theta, "jvp_out", (theta, tangent))
    if out is not None and _overlap(out, jvp_out):
        raise TopkError("out and jvp_out overlap")
    _check(load().topk_mask_jvp_static(theta.data_ptr(), tangent.data_ptr(), rows, n, int(k),
                                       float(p), float(lam),
                                       None if out is None else out.data_ptr(),
                                       jvp_out.data_ptr(), _stream(stream)),
           "topk_mask_jvp_static")
    return out, jvp_out


def topkmag_fwd(x, k, p, lam, out=None, stream=None):
    x = _dev_f32(x, "x")
    rows, n = x.shape
    out = _out(out, x, "out", (x,))
    ensure_workspace(TOPK_OP_MAG_FWD, rows, n, k, p, x.device)
    _check(load().topkmag_fwd(x.data_ptr(), rows, n, int(k), float(p), float(lam),
                              out.data_ptr(), _stream(stream)), "topkmag_fwd")
    return out


def topkmag_jvp(x, tangent, k, p, lam, out=None, jvp_out=None, want_out=True, stream=None):
    x = _dev_f32(x, "x")
    tangent = _like(tangent, x, "tangent")
    rows, n = x.shape
    if out is not None or want_out:
        out = _out(out, x, "out", (x, tangent))
    jvp_out = _out(jvp_out, x, "jvp_out", (x, tangent))
    if out is not None and _overlap(out, jvp_out):
        raise TopkError("out and jvp_out overlap")
    ensure_workspace(TOPK_OP_MAG_JVP, rows, n, k, p, x.device)
    _check(load().topkmag_jvp(x.data_ptr(), tangent.data_ptr(), rows, n, int(k), float(p),
                              float(lam), None if out is None else out.data_ptr(),
                              jvp_out.data_ptr(), _stream(stream)), "topkmag_jvp")
    return out, jvp_out


def _abs_variant(name, op, x, tangent, k, p, lam, out, jvp_out, stream):
    x = _dev_f32(x, "x")
    rows, n = x.shape
    out = _out(out, x, "out", (x,) if tangent is None else (x, _like(tangent, x, "tangent")))
    ensure_workspace(op, rows, n, k, p, x.device)
    if tangent is None:
        _check(getattr(load(), name + "_fwd")(x.data_ptr(), rows, n, int(k), float(p), float(lam),
                                              out.data_ptr(), _stream(stream)), name + "_fwd")
        return out
    jvp_out = _out(jvp_out, x, "jvp_out", (x, tangent))
    if _overlap(out, jvp_out):
        raise TopkError("out and jvp_out overlap")
    _check(getattr(load(), name + "_jvp")(x.data_ptr(), tangent.data_ptr(), rows, n, int(k),
                                          float(p), float(lam), out.data_ptr(), jvp_out.data_ptr(),
                                          _stream(stream)), name + "_jvp")
    return out, jvp_out


def topk_mask_sparse_fwd(theta, k, p, lam, max_nnz, idx_out=None, val_out=None, nnz_out=None,
                         stream=None):
    """Returns (idx [rows, max_nnz] int32, val [rows, max_nnz] float32, nnz [rows] int32); the three
    tensors may be passed in (contiguous, on the GPU, of those shapes and types)."""
    theta = _dev_f32(theta, "theta")
    rows, n = theta.shape
    shape = (rows, int(max_nnz))
    idx = torch.empty(shape, dtype=torch.int32, device=theta.device) if idx_out is None else idx_out
    val = torch.empty(shape, dtype=torch.float32, device=theta.device) if val_out is None else val_out
    nnz = torch.empty((rows,), dtype=torch.int32, device=theta.device) if nnz_out is None else nnz_out
    for t, dt, sh, name in ((idx, torch.int32, shape, "idx_out"), (val, torch.float32, shape, "val_out"),
                            (nnz, torch.int32, (rows,), "nnz_out")):
        if not isinstance(t, torch.Tensor) or not t.is_cuda or t.device != theta.device or \
                t.dtype != dt or tuple(t.shape) != sh or not t.is_contiguous():
            raise TopkError(f"{name} must be a contiguous {dt} tensor of shape {sh} on {theta.device}")
    ensure_workspace(TOPK_OP_MASK_SPARSE, rows, n, k, p, theta.device)
    _check(load().topk_mask_sparse_fwd(theta.data_ptr(), rows, n, int(k), float(p), float(lam),
                                       int(max_nnz), idx.data_ptr(), val.data_ptr(), nnz.data_ptr(),
                                       _stream(stream)), "topk_mask_sparse_fwd")
    return idx, val, nnz


TOPK_PHI_IDENTITY, TOPK_PHI_HALF_SQUARE = 0, 1


def _weights(w, rows, n, device):
    if not isinstance(w, torch.Tensor) or not w.is_cuda or w.dtype != torch.float32 or \
            not w.is_contiguous() or tuple(w.shape) not in ((n,), (rows, n)) or w.device != device:
        raise TopkError(f"w must be a contiguous float32 tensor of shape [n] or [rows, n] on {device}")
    return w, (0 if w.dim() == 1 else n)


def topk_general_fwd(x, w, phi, p, lam, out=None, stream=None):
    x = _dev_f32(x, "x")
    rows, n = x.shape
    w, stride = _weights(w, rows, n, x.device)
    out = _out(out, x, "out", (x, w))
    ensure_workspace(TOPK_OP_GENERAL, rows, n, 0, p, x.device)
    _check(load().topk_general_fwd(x.data_ptr(), w.data_ptr(), stride, rows, n, int(phi), float(p),
                                   float(lam), out.data_ptr(), _stream(stream)), "topk_general_fwd")
    return out


def topk_general_jvp(x, w, tangent, phi, p, lam, out=None, jvp_out=None, want_out=True, stream=None):
    """Returns (out, jvp_out); out is None when want_out is False and no out tensor was given."""
    x = _dev_f32(x, "x")
    tangent = _like(tangent, x, "tangent")
    rows, n = x.shape
    w, stride = _weights(w, rows, n, x.device)
    if out is not None or want_out:
        out = _out(out, x, "out", (x, w, tangent))
    jvp_out = _out(jvp_out, x, "jvp_out", (x, w, tangent))
    if out is not None and _overlap(out, jvp_out):
        raise TopkError("out and jvp_out overlap")
    ensure_workspace(TOPK_OP_GENERAL, rows, n, 0, p, x.device)
    _check(load().topk_general_jvp(x.data_ptr(), w.data_ptr(), stride, tangent.data_ptr(), rows, n,
                                   int(phi), float(p), float(lam),
                                   None if out is None else out.data_ptr(), jvp_out.data_ptr(),
                                   _stream(stream)), "topk_general_jvp")
    return out, jvp_out


def topk_mask_dykstra_fwd(theta, k, lam, iters, out=None, stream=None):
    theta = _dev_f32(theta, "theta")
    rows, n = theta.shape
    out = _out(out, theta, "out", (theta,))
    _check(load().topk_mask_dykstra_fwd(theta.data_ptr(), rows, n, int(k), float(lam), int(iters),
                                        out.data_ptr(), _stream(stream)), "topk_mask_dykstra_fwd")
    return out


def topk_signed_mask_fwd(x, k, p, lam, out=None, stream=None):
    return _abs_variant("topk_signed_mask", TOPK_OP_SIGNED_MASK, x, None, k, p, lam, out, None, stream)


def topk_signed_mask_jvp(x, tangent, k, p, lam, out=None, jvp_out=None, stream=None):
    """Returns (out, jvp_out)."""
    return _abs_variant("topk_signed_mask", TOPK_OP_SIGNED_MASK, x, tangent, k, p, lam, out, jvp_out,
                        stream)


def topk_masked_value_fwd(x, k, p, lam, out=None, stream=None):
    return _abs_variant("topk_masked_value", TOPK_OP_MASKED_VALUE, x, None, k, p, lam, out, None,
                        stream)


def topk_masked_value_jvp(x, tangent, k, p, lam, out=None, jvp_out=None, stream=None):
    """Returns (out, jvp_out)."""
    return _abs_variant("topk_masked_value", TOPK_OP_MASKED_VALUE, x, tangent, k, p, lam, out,
                        jvp_out, stream)


def topk_mask_vjp(theta, cotangent, k, p, lam, out=None, vjp_out=None, want_out=True, stream=None):
    """Returns (out, vjp_out); out is None when want_out is False and no out tensor was given."""
    theta = _dev_f32(theta, "theta")
    cotangent = _like(cotangent, theta, "cotangent")
    rows, n = theta.shape
    if out is not None or want_out:
        out = _out(out, theta, "out", (theta, cotangent))
    vjp_out = _out(vjp_out, theta, "vjp_out", (theta, cotangent))
    if out is not None and _overlap(out, vjp_out):
        raise TopkError("out and vjp_out overlap")
    ensure_workspace(TOPK_OP_MASK_JVP, rows, n, k, p, theta.device)
    _check(load().topk_mask_vjp(theta.data_ptr(), cotangent.data_ptr(), rows, n, int(k), float(p),
                                float(lam), None if out is None else out.data_ptr(),
                                vjp_out.data_ptr(), _stream(stream)), "topk_mask_vjp")
    return out, vjp_out


def topkmag_vjp(x, cotangent, k, p, lam, out=None, vjp_out=None, want_out=True, stream=None):
    x = _dev_f32(x, "x")
    cotangent = _like(cotangent, x, "cotangent")
    rows, n = x.shape
    if out is not None or want_out:
        out = _out(out, x, "out", (x, cotangent))
    vjp_out = _out(vjp_out, x, "vjp_out", (x, cotangent))
    if out is not None and _overlap(out, vjp_out):
        raise TopkError("out and vjp_out overlap")
    ensure_workspace(TOPK_OP_MAG_JVP, rows, n, k, p, x.device)
    _check(load().topkmag_vjp(x.data_ptr(), cotangent.data_ptr(), rows, n, int(k), float(p),
                              float(lam), None if out is None else out.data_ptr(),
                              vjp_out.data_ptr(), _stream(stream)), "topkmag_vjp")
    return out, vjp_out


def topk_mask_loss(theta, target, k, p, lam, loss_out=None, grad_out=None, stream=None):
    """Returns (loss [rows], grad [rows][n])."""
    theta = _dev_f32(theta, "theta")
    target = _like(target, theta, "target")
    rows, n = theta.shape
    if loss_out is None:
        loss_out = torch.empty(rows, dtype=torch.float32, device=theta.device)
    elif not isinstance(loss_out, torch.Tensor) or not loss_out.is_cuda or \
            loss_out.device != theta.device or loss_out.dtype != torch.float32 or \
            tuple(loss_out.shape) != (rows,) or not loss_out.is_contiguous():
        raise TopkError(f"loss_out must be a contiguous float32 tensor of shape ({rows},) on {theta.device}")
    grad_out = _out(grad_out, theta, "grad_out", (theta, target))
    ensure_workspace(TOPK_OP_MASK_FWD, rows, n, k, p, theta.device)
    _check(load().topk_mask_loss(theta.data_ptr(), target.data_ptr(), rows, n, int(k), float(p),
                                 float(lam), loss_out.data_ptr(), grad_out.data_ptr(),
                                 _stream(stream)), "topk_mask_loss")
    return loss_out, grad_out


def topk_argsort_desc(theta, perm_out=None, stream=None):
    theta = _dev_f32(theta, "theta")
    rows, n = theta.shape
    if perm_out is None:
        perm_out = torch.empty((rows, n), dtype=torch.int32, device=theta.device)
    elif not isinstance(perm_out, torch.Tensor) or not perm_out.is_cuda or \
            perm_out.device != theta.device or perm_out.dtype != torch.int32 or \
            tuple(perm_out.shape) != (rows, n) or not perm_out.is_contiguous():
        raise TopkError(f"perm_out must be a contiguous int32 tensor of shape ({rows}, {n}) on {theta.device}")
    ensure_workspace(TOPK_OP_ARGSORT, rows, n, 0, 2.0, theta.device)
    _check(load().topk_argsort_desc(theta.data_ptr(), rows, n, perm_out.data_ptr(),
                                    _stream(stream)), "topk_argsort_desc")
    return perm_out
