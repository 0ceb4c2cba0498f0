"""numpy front end of the plain-C fp64 MGLU oracle -- TEST INFRASTRUCTURE ONLY.

The arithmetic lives in ``mglu_oracle.c`` (Eq. 1-3 of the paper, written out);
this file only marshals numpy arrays into it.  Inputs of any float dtype are
widened exactly to fp64, so values already rounded to bf16 or fp32 enter the
oracle unchanged.
"""
import ctypes

import numpy as np

from . import build_oracle

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle.build(force=False))
        dp = ctypes.POINTER(ctypes.c_double)
        bp = ctypes.POINTER(ctypes.c_uint8)
        lib.mglu_oracle_forward.argtypes = [dp, dp, bp] + [ctypes.c_long] * 4 + [dp, dp, dp]
        lib.mglu_oracle_forward.restype = ctypes.c_int
        lib.swiglu_oracle_forward.argtypes = [dp, dp, dp] + [ctypes.c_long] * 3 + [dp]
        lib.swiglu_oracle_forward.restype = ctypes.c_int
        lib.mglu_oracle_forward_variant.argtypes = ([dp, dp, bp] + [ctypes.c_long] * 4
                                                    + [ctypes.c_int, ctypes.c_int, dp, dp])
        lib.mglu_oracle_forward_variant.restype = ctypes.c_int
        lib.mglu_oracle_route_topk.argtypes = [dp, dp] + [ctypes.c_long] * 4 + [dp]
        lib.mglu_oracle_route_topk.restype = ctypes.c_int
        lib.linear_oracle_forward.argtypes = [dp, dp] + [ctypes.c_long] * 3 + [dp]
        lib.linear_oracle_forward.restype = ctypes.c_int
        lib.mglu_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def threads():
    """Threads the oracle's parallel loops use (OMP_NUM_THREADS or all cores)."""
    return int(_load().mglu_oracle_threads())


def mglu_forward(x, W, masks, return_projections=False):
    """Eq. 3: ``sum_i swish(x (M_i*W)) * (x ((1-M_i)*W))``.

    x [T,h], W [h,d] (logical: reduction index first), masks [n_m,h,d] of 0/1.
    Returns out [T,d] fp64; with ``return_projections`` also gate and value,
    each [n_m,T,d].
    """
    x, W = _f64(x), _f64(W)
    M = np.ascontiguousarray(np.asarray(masks))
    if M.dtype == np.bool_:
        M = M.view(np.uint8)
    if M.dtype != np.uint8:
        raise TypeError("masks must be bool or uint8")
    if x.ndim != 2 or W.ndim != 2 or M.ndim != 3:
        raise ValueError("x [T,h], W [h,d], masks [n_m,h,d] expected")
    T, h = x.shape
    d = W.shape[1]
    n_m = M.shape[0]
    if W.shape[0] != h or M.shape[1:] != (h, d):
        raise ValueError("shape mismatch: x %s W %s masks %s" % (x.shape, W.shape, M.shape))
    if M.size and M.max() > 1:
        raise ValueError("mask bytes must be 0 or 1")
    out = np.empty((T, d), dtype=np.float64)
    gate = np.empty((n_m, T, d), dtype=np.float64) if return_projections else None
    value = np.empty((n_m, T, d), dtype=np.float64) if return_projections else None
    null = ctypes.POINTER(ctypes.c_double)()
    rc = _load().mglu_oracle_forward(
        _dptr(x), _dptr(W), M.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
        T, h, d, n_m, _dptr(out),
        _dptr(gate) if return_projections else null,
        _dptr(value) if return_projections else null)
    if rc != 0:
        raise RuntimeError("mglu_oracle_forward failed with code %d" % rc)
    return (out, gate, value) if return_projections else out


def swiglu_forward(x, Wg, Wv):
    """Eq. 1 with g = Swish: ``swish(x Wg) * (x Wv)``; x [T,h], Wg and Wv [h,d]."""
    x, Wg, Wv = _f64(x), _f64(Wg), _f64(Wv)
    T, h = x.shape
    d = Wg.shape[1]
    if Wg.shape != (h, d) or Wv.shape != (h, d):
        raise ValueError("shape mismatch")
    out = np.empty((T, d), dtype=np.float64)
    rc = _load().swiglu_oracle_forward(_dptr(x), _dptr(Wg), _dptr(Wv), T, h, d, _dptr(out))
    if rc != 0:
        raise RuntimeError("swiglu_oracle_forward failed with code %d" % rc)
    return out


GATE_FN = {"swish": 0, "gelu": 1, "relu": 2}
MASK_USE = {"both": 0, "dense_gate": 1, "dense_value": 2, "none": 3}


def _masks_u8(masks):
    M = np.ascontiguousarray(np.asarray(masks))
    if M.dtype == np.bool_:
        M = M.view(np.uint8)
    if M.dtype != np.uint8:
        raise TypeError("masks must be bool or uint8")
    return M


def mglu_forward_variant(x, W, masks, gate="swish", mask_use="both", route=None):
    """Eq. 3 with the appendix's variations: another gate function, the partial-mask ablations,
    per-token route weights (Top-K routing).  route: None or [T, n_m]."""
    x, W, M = _f64(x), _f64(W), _masks_u8(masks)
    T, h = x.shape
    d = W.shape[1]
    n_m = M.shape[0]
    if W.shape[0] != h or M.shape[1:] != (h, d):
        raise ValueError("shape mismatch")
    r = None
    if route is not None:
        r = _f64(route)
        if r.shape != (T, n_m):
            raise ValueError("route must be [T, n_m]")
    out = np.empty((T, d), dtype=np.float64)
    rc = _load().mglu_oracle_forward_variant(
        _dptr(x), _dptr(W), M.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), T, h, d, n_m,
        GATE_FN[gate], MASK_USE[mask_use], _dptr(r) if r is not None else ctypes.POINTER(ctypes.c_double)(),
        _dptr(out))
    if rc != 0:
        raise RuntimeError("mglu_oracle_forward_variant failed with code %d" % rc)
    return out


def route_topk(x, Wr, k):
    """Top-K router weights [T, n_m]: softmax over the k largest logits of x Wr, 0 elsewhere."""
    x, Wr = _f64(x), _f64(Wr)
    T, h = x.shape
    n_m = Wr.shape[1]
    if Wr.shape[0] != h:
        raise ValueError("shape mismatch")
    w = np.empty((T, n_m), dtype=np.float64)
    rc = _load().mglu_oracle_route_topk(_dptr(x), _dptr(Wr), T, h, n_m, int(k), _dptr(w))
    if rc != 0:
        raise RuntimeError("mglu_oracle_route_topk failed with code %d" % rc)
    return w


def linear_forward(a, W):
    """out = a W: a [T,K], W [K,N]."""
    a, W = _f64(a), _f64(W)
    T, K = a.shape
    if W.shape[0] != K:
        raise ValueError("shape mismatch")
    out = np.empty((T, W.shape[1]), dtype=np.float64)
    rc = _load().linear_oracle_forward(_dptr(a), _dptr(W), T, K, W.shape[1], _dptr(out))
    if rc != 0:
        raise RuntimeError("linear_oracle_forward failed with code %d" % rc)
    return out
