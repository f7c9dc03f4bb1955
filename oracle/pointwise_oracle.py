"""ctypes front end of the C oracle for the library's other functions
(``pointwise_oracle.c``: activations, softmax, pooling, tensor addition with
broadcasting and its transpose, the bias gradient).  TEST INFRASTRUCTURE ONLY.  The arithmetic lives in the C file; this
module only marshals numpy arrays and strides."""
import ctypes
import os

import numpy as np

from . import build as _build

SIGMOID, RELU, TANH = 0, 1, 2
SOFTMAX_INSTANCE, SOFTMAX_CHANNEL = 0, 1   # over (c,h,w) of an image / over c at each (n,h,w)
POOL_MAX, POOL_AVERAGE = 0, 1

_lib = None
_ll4 = ctypes.c_longlong * 4


def _load():
    global _lib
    if _lib is None:
        path = _build.POINTWISE_LIB if os.path.exists(_build.POINTWISE_LIB) else _build.build_pointwise()
        _lib = ctypes.CDLL(path)
    return _lib


def _strides(a):
    assert all(s % a.itemsize == 0 for s in a.strides)
    return _ll4(*[s // a.itemsize for s in a.strides])


def _f32(a):
    """A 4-D input array: float32, or float64 for the double-precision form of a function."""
    a = np.asarray(a)
    assert a.dtype in (np.float32, np.float64) and a.ndim == 4
    return a


def _fn(name, *arrays):
    """The library entry for the arrays' common element type."""
    dt = arrays[0].dtype
    assert all(a.dtype == dt for a in arrays), "all inputs of a call share one element type"
    return getattr(_load(), ("pointwise_oracle_f64_" if dt == np.float64 else "pointwise_oracle_") + name)


def _out(shape, layout, old, beta):
    if layout == "NCHW":
        y = np.empty(shape, dtype=np.float64)
    elif layout == "NHWC":
        n, c, h, w = shape
        y = np.empty((n, h, w, c), dtype=np.float64).transpose(0, 3, 1, 2)
    else:
        raise ValueError(layout)
    old_ptr = None
    keep = None
    if old is not None:
        keep = np.empty_like(y)
        keep[...] = np.asarray(old, dtype=np.float64)
        assert keep.strides == y.strides
        old_ptr = keep.ctypes.data
    elif beta != 0.0:
        raise ValueError("beta != 0 needs the old output")
    return y, old_ptr, keep


def _check(rc, what):
    if rc != 0:
        raise ValueError("%s rejected the problem: %d" % (what, rc))


def activation_forward(mode, x, alpha=1.0, beta=0.0, y_old=None, layout="NCHW"):
    x = _f32(x)
    y, old_ptr, _keep = _out(x.shape, layout, y_old, beta)
    _check(_fn("activation_forward", x)(
        ctypes.c_int(mode), ctypes.c_void_p(x.ctypes.data), _strides(x), *[ctypes.c_int(d) for d in x.shape],
        ctypes.c_double(alpha), ctypes.c_double(beta), ctypes.c_void_p(old_ptr), ctypes.c_void_p(y.ctypes.data),
        _strides(y)), "activation_forward")
    return y


def activation_backward(mode, y, dy, x, alpha=1.0, beta=0.0, dx_old=None, layout="NCHW"):
    y, dy, x = _f32(y), _f32(dy), _f32(x)
    assert y.shape == dy.shape == x.shape
    dx, old_ptr, _keep = _out(x.shape, layout, dx_old, beta)
    _check(_fn("activation_backward", y, dy, x)(
        ctypes.c_int(mode), ctypes.c_void_p(y.ctypes.data), _strides(y), ctypes.c_void_p(dy.ctypes.data), _strides(dy),
        ctypes.c_void_p(x.ctypes.data), _strides(x), *[ctypes.c_int(d) for d in x.shape],
        ctypes.c_double(alpha), ctypes.c_double(beta), ctypes.c_void_p(old_ptr), ctypes.c_void_p(dx.ctypes.data),
        _strides(dx)), "activation_backward")
    return dx


def add_tensor(b, shape, alpha=1.0, beta=0.0, y_old=None, layout="NCHW"):
    """alpha * b (broadcast along its size-1 dimensions to ``shape``) + beta * y_old."""
    b = _f32(b)
    y, old_ptr, _keep = _out(tuple(shape), layout, y_old, beta)
    _check(_fn("add_tensor", b)(
        ctypes.c_void_p(b.ctypes.data), _strides(b), *[ctypes.c_int(d) for d in b.shape],
        *[ctypes.c_int(d) for d in shape], ctypes.c_double(alpha), ctypes.c_double(beta),
        ctypes.c_void_p(old_ptr), ctypes.c_void_p(y.ctypes.data), _strides(y)), "add_tensor")
    return y


def bias_backward(dy, alpha=1.0, beta=0.0, db_old=None):
    """alpha * (sum of dy over n, h, w per feature map) + beta * db_old: C values as float64."""
    dy = _f32(dy)
    db = np.empty(dy.shape[1], dtype=np.float64)
    keep = None
    if db_old is not None:
        keep = np.ascontiguousarray(np.asarray(db_old, dtype=np.float64).reshape(-1))
        assert keep.shape == db.shape
    elif beta != 0.0:
        raise ValueError("beta != 0 needs the old output")
    _check(_fn("bias_backward", dy)(
        ctypes.c_void_p(dy.ctypes.data), _strides(dy), *[ctypes.c_int(d) for d in dy.shape],
        ctypes.c_double(alpha), ctypes.c_double(beta), ctypes.c_void_p(keep.ctypes.data if keep is not None else None),
        ctypes.c_void_p(db.ctypes.data)), "bias_backward")
    return db


def softmax_forward(mode, x, alpha=1.0, beta=0.0, y_old=None, layout="NCHW"):
    x = _f32(x)
    y, old_ptr, _keep = _out(x.shape, layout, y_old, beta)
    _check(_fn("softmax_forward", x)(
        ctypes.c_int(mode), ctypes.c_void_p(x.ctypes.data), _strides(x), *[ctypes.c_int(d) for d in x.shape],
        ctypes.c_double(alpha), ctypes.c_double(beta), ctypes.c_void_p(old_ptr), ctypes.c_void_p(y.ctypes.data),
        _strides(y)), "softmax_forward")
    return y


def pooling_output_dim(H, win, pad, u):
    return (H + 2 * pad - win) // u + 1


def pooling_forward(mode, x, window, pad=(0, 0), stride=(1, 1), alpha=1.0, beta=0.0, y_old=None, layout="NCHW"):
    x = _f32(x)
    N, C, H, W = x.shape
    P = pooling_output_dim(H, window[0], pad[0], stride[0])
    Q = pooling_output_dim(W, window[1], pad[1], stride[1])
    if P < 1 or Q < 1:
        raise ValueError("no output")
    y, old_ptr, _keep = _out((N, C, P, Q), layout, y_old, beta)
    _check(_fn("pooling_forward", x)(
        ctypes.c_int(mode), ctypes.c_void_p(x.ctypes.data), _strides(x), *[ctypes.c_int(d) for d in x.shape],
        ctypes.c_int(window[0]), ctypes.c_int(window[1]), ctypes.c_int(pad[0]), ctypes.c_int(pad[1]),
        ctypes.c_int(stride[0]), ctypes.c_int(stride[1]), ctypes.c_double(alpha), ctypes.c_double(beta),
        ctypes.c_void_p(old_ptr), ctypes.c_void_p(y.ctypes.data), _strides(y), ctypes.c_int(P), ctypes.c_int(Q)),
        "pooling_forward")
    return y


def softmax_backward(mode, y, dy, alpha=1.0, beta=0.0, dx_old=None, layout="NCHW"):
    y, dy = _f32(y), _f32(dy)
    assert y.shape == dy.shape
    dx, old_ptr, _keep = _out(y.shape, layout, dx_old, beta)
    _check(_fn("softmax_backward", y, dy)(
        ctypes.c_int(mode), ctypes.c_void_p(y.ctypes.data), _strides(y), ctypes.c_void_p(dy.ctypes.data), _strides(dy),
        *[ctypes.c_int(d) for d in y.shape], ctypes.c_double(alpha), ctypes.c_double(beta), ctypes.c_void_p(old_ptr),
        ctypes.c_void_p(dx.ctypes.data), _strides(dx)), "softmax_backward")
    return dx


def pooling_backward(mode, x, dy, window, pad=(0, 0), stride=(1, 1), alpha=1.0, beta=0.0, dx_old=None, layout="NCHW"):
    x, dy = _f32(x), _f32(dy)
    N, C, H, W = x.shape
    P = pooling_output_dim(H, window[0], pad[0], stride[0])
    Q = pooling_output_dim(W, window[1], pad[1], stride[1])
    assert dy.shape == (N, C, P, Q)
    dx, old_ptr, _keep = _out((N, C, H, W), layout, dx_old, beta)
    scratch = np.empty(N * C * H * W, dtype=np.float64)
    _check(_fn("pooling_backward", x, dy)(
        ctypes.c_int(mode), ctypes.c_void_p(x.ctypes.data), _strides(x), ctypes.c_void_p(dy.ctypes.data), _strides(dy),
        *[ctypes.c_int(d) for d in x.shape],
        ctypes.c_int(window[0]), ctypes.c_int(window[1]), ctypes.c_int(pad[0]), ctypes.c_int(pad[1]),
        ctypes.c_int(stride[0]), ctypes.c_int(stride[1]), ctypes.c_double(alpha), ctypes.c_double(beta),
        ctypes.c_void_p(old_ptr), ctypes.c_void_p(dx.ctypes.data), _strides(dx), ctypes.c_int(P), ctypes.c_int(Q),
        ctypes.c_void_p(scratch.ctypes.data)), "pooling_backward")
    return dx
