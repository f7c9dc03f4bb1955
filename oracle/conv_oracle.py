"""ctypes front end of the C oracle (``conv_oracle.c``).  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file: the seven-loop forward convolution of the
paper's eq. 3 with the accessing function of eq. 2 (or its cross-correlation
variant), the output size of eq. 1, the alpha/beta accumulate form, and the two
backward forms (the transposes of the forward map with respect to the input and to
the filters).  This module only marshals numpy arrays and strides.
"""
import ctypes
import os

import numpy as np

from . import build as _build

CONVOLUTION = 0        # eq. 2: filter inverted
CROSS_CORRELATION = 1  # no inversion

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        lib = ctypes.CDLL(path)
        ll = ctypes.c_longlong
        lib.conv_oracle_output_dim.restype = ll
        lib.conv_oracle_output_dim.argtypes = [ll, ll, ll, ll]
        lib.conv_oracle_forward.restype = ctypes.c_int
        lib.conv_oracle_forward.argtypes = (
            [ctypes.c_void_p, ctypes.POINTER(ll)] + [ctypes.c_int] * 4
            + [ctypes.c_void_p] + [ctypes.c_int] * 3
            + [ctypes.c_int] * 5
            + [ctypes.c_double, ctypes.c_double]
            + [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ll)]
            + [ctypes.c_int] * 3)
        lib.conv_oracle_backward_data.restype = ctypes.c_int
        lib.conv_oracle_backward_data.argtypes = (
            [ctypes.c_void_p] + [ctypes.c_int] * 4
            + [ctypes.c_void_p, ctypes.POINTER(ll)] + [ctypes.c_int] * 3
            + [ctypes.c_int] * 5
            + [ctypes.c_double, ctypes.c_double]
            + [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ll)]
            + [ctypes.c_int] * 3)
        lib.conv_oracle_backward_filter.restype = ctypes.c_int
        lib.conv_oracle_backward_filter.argtypes = (
            [ctypes.c_void_p, ctypes.POINTER(ll)] + [ctypes.c_int] * 4
            + [ctypes.c_void_p, ctypes.POINTER(ll)] + [ctypes.c_int] * 3
            + [ctypes.c_int] * 5
            + [ctypes.c_double, ctypes.c_double]
            + [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 3)
        lib.conv_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def output_dim(H, R, u, pad):
    """Eq. 1: ceil((H - R + 1 + 2*pad) / u)."""
    return int(_load().conv_oracle_output_dim(H, R, u, pad))


def max_threads():
    return int(_load().conv_oracle_max_threads())


def _elem_strides(a):
    assert all(s % a.itemsize == 0 for s in a.strides)
    return [s // a.itemsize for s in a.strides]


def conv_forward(x, w, pad=(0, 0), stride=(1, 1), mode=CROSS_CORRELATION,
                 alpha=1.0, beta=0.0, y_old=None, y_layout="NCHW", nthreads=0):
    """y = alpha * conv(x, w) + beta * y_old, all as float64, logical shape (N,K,P,Q).

    ``x``: float32 array, logical shape (N,C,H,W), any (non-negative) strides - a
    transposed or sliced view is read in place through its strides.  ``w``: float32
    (K,C,R,S).  ``y_old``: logical (N,K,P,Q) array or None.  ``y_layout`` chooses the
    memory order of the oracle's own output buffer ("NCHW" or "NHWC"); the returned
    array is always indexed logically, so the choice only exercises the strided store.
    """
    x = np.asarray(x)
    assert x.dtype == np.float32 and x.ndim == 4
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert w.ndim == 4 and w.shape[1] == x.shape[1]
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = output_dim(H, R, stride[0], pad[0])
    Q = output_dim(W, S, stride[1], pad[1])
    if P < 1 or Q < 1:
        raise ValueError("no output: P=%d Q=%d" % (P, Q))
    if y_layout == "NCHW":
        y = np.empty((N, K, P, Q), dtype=np.float64)
    elif y_layout == "NHWC":
        y = np.empty((N, P, Q, K), dtype=np.float64).transpose(0, 3, 1, 2)
    else:
        raise ValueError(y_layout)
    yo_ptr = None
    if y_old is not None:
        yo = np.empty_like(y)  # same strides as y
        yo[...] = np.asarray(y_old, dtype=np.float64)
        assert yo.strides == y.strides
        yo_ptr = yo.ctypes.data
    elif beta != 0.0:
        raise ValueError("beta != 0 needs y_old")
    ll4 = ctypes.c_longlong * 4
    rc = _load().conv_oracle_forward(
        x.ctypes.data, ll4(*_elem_strides(x)), N, C, H, W,
        w.ctypes.data, K, R, S,
        pad[0], pad[1], stride[0], stride[1], mode,
        float(alpha), float(beta),
        yo_ptr, y.ctypes.data, ll4(*_elem_strides(y)), P, Q, nthreads)
    if rc != 0:
        raise ValueError("conv_oracle_forward rejected the problem: %d" % rc)
    return y


def _strided_f64(shape, layout):
    if layout == "NCHW":
        return np.empty(shape, dtype=np.float64)
    if layout == "NHWC":
        n, c, h, w = shape
        return np.empty((n, h, w, c), dtype=np.float64).transpose(0, 3, 1, 2)
    raise ValueError(layout)


def conv_backward_data(dy, w, hw, pad=(0, 0), stride=(1, 1), mode=CROSS_CORRELATION,
                       alpha=1.0, beta=0.0, dx_old=None, dx_layout="NCHW", nthreads=0):
    """dx = alpha * (transpose of the forward map w.r.t. x applied to dy) + beta * dx_old,
    float64, logical shape (N,C,H,W) with ``hw = (H, W)`` the input size of the forward
    problem (eq. 1 does not determine it from P, Q when the stride is above 1).

    ``dy``: float32, logical (N,K,P,Q), any non-negative strides.  ``w``: float32 (K,C,R,S).
    """
    dy = np.asarray(dy)
    assert dy.dtype == np.float32 and dy.ndim == 4
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, K, P, Q = dy.shape
    assert w.ndim == 4 and w.shape[0] == K
    _, C, R, S = w.shape
    H, W = hw
    dx = _strided_f64((N, C, H, W), dx_layout)
    old_ptr = None
    if dx_old is not None:
        old = np.empty_like(dx)
        old[...] = np.asarray(dx_old, dtype=np.float64)
        assert old.strides == dx.strides
        old_ptr = old.ctypes.data
    elif beta != 0.0:
        raise ValueError("beta != 0 needs dx_old")
    ll4 = ctypes.c_longlong * 4
    rc = _load().conv_oracle_backward_data(
        w.ctypes.data, K, C, R, S,
        dy.ctypes.data, ll4(*_elem_strides(dy)), N, P, Q,
        pad[0], pad[1], stride[0], stride[1], mode,
        float(alpha), float(beta),
        old_ptr, dx.ctypes.data, ll4(*_elem_strides(dx)), H, W, nthreads)
    if rc != 0:
        raise ValueError("conv_oracle_backward_data rejected the problem: %d" % rc)
    return dx


def conv_backward_filter(x, dy, rs, pad=(0, 0), stride=(1, 1), mode=CROSS_CORRELATION,
                         alpha=1.0, beta=0.0, dw_old=None, nthreads=0):
    """dw = alpha * (transpose of the forward map w.r.t. w applied to dy) + beta * dw_old,
    float64, shape (K,C,R,S) with ``rs = (R, S)`` the filter size.

    ``x``: float32 logical (N,C,H,W); ``dy``: float32 logical (N,K,P,Q); any non-negative strides.
    """
    x = np.asarray(x)
    dy = np.asarray(dy)
    assert x.dtype == np.float32 and x.ndim == 4 and dy.dtype == np.float32 and dy.ndim == 4
    N, C, H, W = x.shape
    assert dy.shape[0] == N
    _, K, P, Q = dy.shape
    R, S = rs
    dw = np.empty((K, C, R, S), dtype=np.float64)
    old_ptr = None
    if dw_old is not None:
        old = np.ascontiguousarray(dw_old, dtype=np.float64)
        assert old.shape == dw.shape
        old_ptr = old.ctypes.data
    elif beta != 0.0:
        raise ValueError("beta != 0 needs dw_old")
    ll4 = ctypes.c_longlong * 4
    rc = _load().conv_oracle_backward_filter(
        x.ctypes.data, ll4(*_elem_strides(x)), N, C, H, W,
        dy.ctypes.data, ll4(*_elem_strides(dy)), K, P, Q,
        pad[0], pad[1], stride[0], stride[1], mode,
        float(alpha), float(beta),
        old_ptr, dw.ctypes.data, R, S, nthreads)
    if rc != 0:
        raise ValueError("conv_oracle_backward_filter rejected the problem: %d" % rc)
    return dw
