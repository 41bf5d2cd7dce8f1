"""CPU oracle for the conv2d hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end to conv2d_oracle.c (plain direct loops, fp64 sums; the
definitions follow the matrix-product reading of the paper's Sec. 4.2 "im2col"
passage).  Nothing on the product path may import this package; only tests, the
smoke check and the benchmark's CPU-baseline leg do.  It imports nothing from the
HIP package.

Every function takes C-contiguous fp32 numpy arrays (x NCHW, w KCRS, dy NKPQ) and
returns fp64 arrays.  `geom` is the 11-tuple
(N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w).
"""
from __future__ import annotations

import ctypes as C
from typing import Optional, Sequence, Tuple

import numpy as np

from .build import build as _build

_lib = None
_I = C.c_int
_FP = C.POINTER(C.c_float)
_DP = C.POINTER(C.c_double)
_LP = C.POINTER(C.c_int64)


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(_build())
        g = [_I] * 11
        lib.oracle_conv2d_output_dims.argtypes = g + [C.POINTER(_I), C.POINTER(_I)]
        lib.oracle_conv2d_fwd.argtypes = g + [_FP, _FP, _FP, _DP]
        lib.oracle_conv2d_bwd_data.argtypes = g + [_FP, _FP, _DP]
        lib.oracle_conv2d_bwd_weight.argtypes = g + [_FP, _FP, C.c_double, _DP, _DP]
        lib.oracle_conv2d_fwd_at.argtypes = g + [_FP, _FP, _FP, _LP, C.c_int64, _DP]
        lib.oracle_conv2d_bwd_data_at.argtypes = g + [_FP, _FP, _LP, C.c_int64, _DP]
        lib.oracle_conv2d_bwd_weight_at.argtypes = g + [_FP, _FP, C.c_double, _LP, C.c_int64, _DP]
        lib.oracle_num_threads.restype = _I
        _lib = lib
    return _lib


def _f(a: np.ndarray, shape) -> "C._Pointer":
    if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"] or tuple(a.shape) != tuple(shape):
        raise ValueError("expected C-contiguous float32 of shape %s, got %s %s"
                         % (tuple(shape), a.dtype, a.shape))
    return a.ctypes.data_as(_FP)


def _geom(geom: Sequence[int]):
    g = tuple(int(v) for v in geom)
    if len(g) != 11:
        raise ValueError("geom must have 11 entries")
    return g


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def output_dims(geom) -> Tuple[int, int]:
    g = _geom(geom)
    P, Q = _I(), _I()
    if _load().oracle_conv2d_output_dims(*g, C.byref(P), C.byref(Q)):
        raise ValueError("invalid geometry %s" % (g,))
    return P.value, Q.value


def fwd(geom, x, w, b: Optional[np.ndarray] = None) -> np.ndarray:
    g = _geom(geom)
    N, Cc, H, W, K, R, S = g[:7]
    P, Q = output_dims(g)
    y = np.empty((N, K, P, Q), dtype=np.float64)
    rc = _load().oracle_conv2d_fwd(*g, _f(x, (N, Cc, H, W)), _f(w, (K, Cc, R, S)),
                                   _f(b, (K,)) if b is not None else None,
                                   y.ctypes.data_as(_DP))
    if rc:
        raise ValueError("oracle fwd rc=%d" % rc)
    return y


def fwd_relu(geom, x, w, b: Optional[np.ndarray] = None) -> np.ndarray:
    """Forward followed by the rectifier layer the paper's Sec. 4.1 lists beside the
    convolutions (RELU): max(0, y) element by element on the fp64 forward result."""
    return np.maximum(fwd(geom, x, w, b), 0.0)


def fwd_relu_pool2(geom, x, w, b: Optional[np.ndarray] = None) -> np.ndarray:
    """fwd_relu followed by the 2x2 / stride-2 max pooling of the paper's Sec. 4.1 layer
    list: out[n,k,i,j] = max of the four rectified outputs (2i+a, 2j+b), a, b in {0,1}.
    P and Q must be even.  Written as explicit slices, one per window position."""
    y = fwd_relu(geom, x, w, b)
    if y.shape[2] % 2 or y.shape[3] % 2:
        raise ValueError("odd output size")
    out = y[:, :, 0::2, 0::2]
    for a_, b_ in ((0, 1), (1, 0), (1, 1)):
        out = np.maximum(out, y[:, :, a_::2, b_::2])
    return np.ascontiguousarray(out)


def bwd_data(geom, dy, w) -> np.ndarray:
    g = _geom(geom)
    N, Cc, H, W, K, R, S = g[:7]
    P, Q = output_dims(g)
    dx = np.empty((N, Cc, H, W), dtype=np.float64)
    rc = _load().oracle_conv2d_bwd_data(*g, _f(dy, (N, K, P, Q)), _f(w, (K, Cc, R, S)),
                                        dx.ctypes.data_as(_DP))
    if rc:
        raise ValueError("oracle bwd_data rc=%d" % rc)
    return dx


def bwd_weight(geom, x, dy, scale: float = 1.0, want_db: bool = True):
    g = _geom(geom)
    N, Cc, H, W, K, R, S = g[:7]
    P, Q = output_dims(g)
    dw = np.empty((K, Cc, R, S), dtype=np.float64)
    db = np.empty((K,), dtype=np.float64) if want_db else None
    rc = _load().oracle_conv2d_bwd_weight(*g, _f(x, (N, Cc, H, W)), _f(dy, (N, K, P, Q)),
                                          float(scale), dw.ctypes.data_as(_DP),
                                          db.ctypes.data_as(_DP) if want_db else None)
    if rc:
        raise ValueError("oracle bwd_weight rc=%d" % rc)
    return dw, db


def _idx(idx) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(idx, dtype=np.int64).ravel())


def fwd_at(geom, x, w, b, idx) -> np.ndarray:
    """y.ravel()[idx] computed element by element."""
    g = _geom(geom)
    N, Cc, H, W, K, R, S = g[:7]
    ii = _idx(idx)
    out = np.empty(ii.size, dtype=np.float64)
    rc = _load().oracle_conv2d_fwd_at(*g, _f(x, (N, Cc, H, W)), _f(w, (K, Cc, R, S)),
                                      _f(b, (K,)) if b is not None else None,
                                      ii.ctypes.data_as(_LP), ii.size, out.ctypes.data_as(_DP))
    if rc:
        raise ValueError("oracle fwd_at rc=%d" % rc)
    return out


def bwd_data_at(geom, dy, w, idx) -> np.ndarray:
    """dx.ravel()[idx] computed element by element (gather form)."""
    g = _geom(geom)
    N, Cc, H, W, K, R, S = g[:7]
    P, Q = output_dims(g)
    ii = _idx(idx)
    out = np.empty(ii.size, dtype=np.float64)
    rc = _load().oracle_conv2d_bwd_data_at(*g, _f(dy, (N, K, P, Q)), _f(w, (K, Cc, R, S)),
                                           ii.ctypes.data_as(_LP), ii.size,
                                           out.ctypes.data_as(_DP))
    if rc:
        raise ValueError("oracle bwd_data_at rc=%d" % rc)
    return out


def bwd_weight_at(geom, x, dy, idx, scale: float = 1.0) -> np.ndarray:
    """dw.ravel()[idx] computed element by element."""
    g = _geom(geom)
    N, Cc, H, W, K, R, S = g[:7]
    P, Q = output_dims(g)
    ii = _idx(idx)
    out = np.empty(ii.size, dtype=np.float64)
    rc = _load().oracle_conv2d_bwd_weight_at(*g, _f(x, (N, Cc, H, W)), _f(dy, (N, K, P, Q)),
                                             float(scale), ii.ctypes.data_as(_LP), ii.size,
                                             out.ctypes.data_as(_DP))
    if rc:
        raise ValueError("oracle bwd_weight_at rc=%d" % rc)
    return out


def apply_mul_add(x: np.ndarray, a: float, b: float) -> np.ndarray:
    """Per-element operation of the paper's Sec. 3.3 experiment (bandwidth of
    per-element kernels against tensor size; the paper does not say which
    operation it timed): y[i] = fl(fl(a * x[i]) + b), both operations rounded to
    fp32 separately (no fused multiply-add), as a Torch `mul` followed by `add`.
    Plain numpy; fp32 in, fp32 out (the precision is part of the definition)."""
    if x.dtype != np.float32:
        raise ValueError("expected float32")
    t = np.multiply(x, np.float32(a), dtype=np.float32)
    return np.add(t, np.float32(b), dtype=np.float32)
