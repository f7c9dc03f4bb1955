"""Run the library on numpy inputs through its C ABI: device buffers, descriptors, launches.

Used by the GPU tests, ``bench.py`` and the smoke check.  PyTorch serves for device memory
and streams only; every arithmetic step runs in the library's kernels.  Output buffers are
surrounded by guard bands so that a store outside a tensor's extent is caught.
"""
import numpy as np
import torch

from . import binding as ig

GUARD = 4096          # elements of guard band before and after y
GUARD_VALUE = 777.25


def _dt(dtype):
    return {"f32": ig.IGC_DATA_FLOAT, "bf16": ig.IGC_DATA_BFLOAT16, "f64": ig.IGC_DATA_DOUBLE}[dtype]


def _out_torch(dtype):
    return torch.float64 if dtype == "f64" else torch.float32


def elem_strides(a):
    return [s // a.itemsize for s in a.strides]


def extent(shape, strides):
    return 1 + sum((d - 1) * s for d, s in zip(shape, strides))


def to_device_strided(a, dtype):
    """Copy a (possibly strided) numpy array's memory span to the GPU; returns
    (tensor holding the span, element strides).  bf16: values must be representable."""
    strides = elem_strides(a)
    n = extent(a.shape, strides)
    flat = np.lib.stride_tricks.as_strided(a, shape=(n,), strides=(a.itemsize,))
    t = torch.from_numpy(np.ascontiguousarray(flat))
    assert (a.dtype == np.float64) == (dtype == "f64")
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
        assert torch.equal(t.float(), torch.from_numpy(np.ascontiguousarray(flat)))
    return t.cuda(), strides


class GpuConv:
    """One problem set up on the GPU through the C ABI."""

    def __init__(self, x, w, pad, stride, mode, dtype="f32", y_layout="NCHW", y_strides=None,
                 y_extent=None, handle=None):
        self.handle = handle or ig.Handle()
        N, C, H, W = x.shape
        K, _, R, S = w.shape
        dt = _dt(dtype)
        self.esize = 8 if dtype == "f64" else 4
        self.x_dev, xs = to_device_strided(x, dtype)
        self.w_dev, _ = to_device_strided(np.ascontiguousarray(w), dtype)
        self.xdesc = ig.TensorDescriptor().set(dt, N, C, H, W, xs)
        self.wdesc = ig.FilterDescriptor().set(dt, K, C, R, S)
        self.conv = ig.ConvolutionDescriptor().set(pad[0], pad[1], stride[0], stride[1], mode)
        n, k, p, q = ig.get_output_dim(self.conv, self.xdesc, self.wdesc)
        self.yshape = (n, k, p, q)
        if y_strides is None:
            if y_layout == "NCHW":
                y_strides = (k * p * q, p * q, q, 1)
            elif y_layout == "NHWC":
                y_strides = (p * q * k, 1, q * k, k)
            else:
                raise ValueError(y_layout)
        self.ystrides = tuple(y_strides)
        self.yext = y_extent or extent(self.yshape, self.ystrides)
        self.ydesc = ig.TensorDescriptor().set(ig.IGC_DATA_DOUBLE if dtype == "f64" else ig.IGC_DATA_FLOAT, n, k, p, q, self.ystrides)
        self.ybuf = torch.full((self.yext + 2 * GUARD,), GUARD_VALUE, dtype=_out_torch(dtype), device="cuda")
        self.flops = 2 * n * k * p * q * C * R * S

    @property
    def y_ptr(self):
        return self.ybuf.data_ptr() + self.esize * GUARD

    def y_view(self):
        """Logical (N,K,P,Q) view of the device output."""
        return torch.as_strided(self.ybuf, self.yshape, self.ystrides, storage_offset=GUARD)

    def prefill(self, y0=None, value=None):
        inner = self.ybuf[GUARD:GUARD + self.yext]
        if y0 is not None:
            inner.fill_(float("nan"))
            self.y_view().copy_(torch.from_numpy(np.ascontiguousarray(y0)).cuda().to(self.ybuf.dtype))
        else:
            inner.fill_(value)

    def plan(self):
        return ig.get_plan(self.handle, self.xdesc, self.wdesc, self.conv, self.ydesc)

    def launch(self, alpha=1.0, beta=0.0):
        self.handle.set_stream(torch.cuda.current_stream().cuda_stream)
        ws = getattr(self, "ws", None)
        st = ig.convolution_forward(self.handle, alpha, self.xdesc, self.x_dev.data_ptr(), self.wdesc,
                                    self.w_dev.data_ptr(), self.conv, beta, self.ydesc, self.y_ptr,
                                    ws.ptr if ws is not None else 0, self.ws_bytes if ws is not None else 0)
        ig.check(st, "igcConvolutionForward")

    def lend_workspace(self, nbytes=None):
        """Give later launches a workspace (default: the size the library reports as useful);
        returns that reported size."""
        asked = ig.get_optional_workspace_size(self.handle, self.xdesc, self.wdesc, self.conv, self.ydesc)
        self.ws_bytes = asked if nbytes is None else int(nbytes)
        self.ws = GuardedOutput((1, 1, 1, max(self.ws_bytes // 4, 1)), (0, 0, 0, 1)) if self.ws_bytes else None
        if self.ws is not None:
            self.ws.prefill(value=float("nan"))
        return asked

    def launch_fused(self, alpha, beta, bias, activation):
        """y = f(alpha*conv + beta*y + bias[k]); bias a float32 vector of K values or None."""
        self.handle.set_stream(torch.cuda.current_stream().cuda_stream)
        self.bias_dev = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda()
        ws = getattr(self, "ws", None)
        st = ig.convolution_bias_activation_forward(
            self.handle, alpha, self.xdesc, self.x_dev.data_ptr(), self.wdesc, self.w_dev.data_ptr(), self.conv, beta,
            0 if bias is None else self.bias_dev.data_ptr(), activation, self.ydesc, self.y_ptr,
            ws.ptr if ws is not None else 0, self.ws_bytes if ws is not None else 0)
        ig.check(st, "igcConvolutionBiasActivationForward")

    def result(self):
        torch.cuda.synchronize()
        g = self.ybuf.cpu().numpy()
        assert np.all(g[:GUARD] == GUARD_VALUE) and np.all(g[GUARD + self.yext:] == GUARD_VALUE), \
            "store outside y's extent"
        return self.y_view().cpu().numpy().astype(np.float64)


def run(x, w, pad=(0, 0), stride=(1, 1), mode=ig.IGC_CROSS_CORRELATION, alpha=1.0, beta=0.0, y0=None,
        dtype="f32", y_layout="NCHW", kernel=None):
    """One forward call; returns (y as float64 logical NCHW, plan)."""
    g = GpuConv(x, w, pad, stride, mode, dtype=dtype, y_layout=y_layout)
    if kernel is not None:
        g.handle.set_kernel_override(kernel)
    if y0 is not None:
        g.prefill(y0=y0)
    else:
        g.prefill(value=float("nan"))   # beta == 0 must overwrite, never read
    g.launch(alpha, beta)
    return g.result(), g.plan()


def rel_err(got, want):
    """The parity measure: max|got - want| / max|want|."""
    return float(np.max(np.abs(got - want)) / max(np.max(np.abs(want)), 1e-30))


def _device_tensor(a, dtype):
    """(device tensor holding a's memory span, element strides, byte offset 0)."""
    return to_device_strided(a, dtype)


class GuardedOutput:
    """A float32 device buffer for a strided logical 4-D tensor, with guard bands."""

    def __init__(self, shape, strides, dtype="f32"):
        self.shape, self.strides = tuple(shape), tuple(strides)
        self.ext = extent(self.shape, self.strides)
        self.buf = torch.full((self.ext + 2 * GUARD,), GUARD_VALUE, dtype=_out_torch(dtype), device="cuda")

    @property
    def ptr(self):
        return self.buf.data_ptr() + self.buf.element_size() * GUARD

    def view(self):
        return torch.as_strided(self.buf, self.shape, self.strides, storage_offset=GUARD)

    def prefill(self, old=None, value=None):
        inner = self.buf[GUARD:GUARD + self.ext]
        if old is not None:
            inner.fill_(float("nan"))
            self.view().copy_(torch.from_numpy(np.ascontiguousarray(old)).cuda().to(self.buf.dtype))
        else:
            inner.fill_(value)

    def result(self):
        torch.cuda.synchronize()
        g = self.buf.cpu().numpy()
        assert np.all(g[:GUARD] == GUARD_VALUE) and np.all(g[GUARD + self.ext:] == GUARD_VALUE), \
            "store outside the output's extent"
        return self.view().cpu().numpy().astype(np.float64)


def layout_strides(shape, layout):
    n, c, h, w = shape
    if layout == "NCHW":
        return (c * h * w, h * w, w, 1)
    if layout == "NHWC":
        return (h * w * c, 1, w * c, c)
    raise ValueError(layout)


class GpuBackwardData:
    """One backward-data problem set up on the GPU through the C ABI.  ``workspace``: "full"
    (what the library asks for), "none", or a number of bytes."""

    def __init__(self, dy, w, hw, pad, stride, mode, dtype="f32", dx_layout="NCHW", workspace="full"):
        self.handle = ig.Handle()
        N, K, P, Q = dy.shape
        _, C, R, S = w.shape
        dt = _dt(dtype)
        self.dy_dev, dys = to_device_strided(dy, dtype)
        self.w_dev, _ = to_device_strided(np.ascontiguousarray(w), dtype)
        self.dydesc = ig.TensorDescriptor().set(dt, N, K, P, Q, dys)
        self.wdesc = ig.FilterDescriptor().set(dt, K, C, R, S)
        self.conv = ig.ConvolutionDescriptor().set(pad[0], pad[1], stride[0], stride[1], mode)
        shape = (N, C, hw[0], hw[1])
        self.out = GuardedOutput(shape, layout_strides(shape, dx_layout), dtype)
        self.dxdesc = ig.TensorDescriptor().set(ig.IGC_DATA_DOUBLE if dtype == "f64" else ig.IGC_DATA_FLOAT, *shape, self.out.strides)
        self.asked = ig.get_backward_data_workspace_size(self.handle, self.wdesc, self.dydesc, self.conv, self.dxdesc)
        self.ws_bytes = self.asked if workspace == "full" else (0 if workspace == "none" else int(workspace))
        self.ws = GuardedOutput((1, 1, 1, max((self.ws_bytes + 3) // 4, 1)), (0, 0, 0, 1))
        self.ws.prefill(value=float("nan"))

    def launch(self, alpha=1.0, beta=0.0):
        self.handle.set_stream(torch.cuda.current_stream().cuda_stream)
        st = ig.convolution_backward_data(self.handle, alpha, self.wdesc, self.w_dev.data_ptr(), self.dydesc,
                                          self.dy_dev.data_ptr(), self.conv, beta, self.dxdesc, self.out.ptr,
                                          self.ws.ptr if self.ws_bytes else 0, self.ws_bytes)
        ig.check(st, "igcConvolutionBackwardData")


def run_backward_data(dy, w, hw, pad=(0, 0), stride=(1, 1), mode=ig.IGC_CROSS_CORRELATION, alpha=1.0, beta=0.0,
                      dx_old=None, dtype="f32", dx_layout="NCHW", workspace="full", asked=None):
    """One igcConvolutionBackwardData call; returns dx as float64, logical (N,C,H,W).  ``asked``:
    a list that receives the workspace size the library asked for."""
    g = GpuBackwardData(dy, w, hw, pad, stride, mode, dtype, dx_layout, workspace)
    if asked is not None:
        asked.append(g.asked)
    if dx_old is not None:
        g.out.prefill(old=dx_old)
    else:
        g.out.prefill(value=float("nan"))
    g.launch(alpha, beta)
    g.ws.result()   # (guard bands of the workspace)
    return g.out.result()


class GpuBackwardFilter:
    """One backward-filter problem set up on the GPU through the C ABI.  ``workspace``: "full"
    (what the library asks for), "none", or a number of bytes."""

    def __init__(self, x, dy, rs, pad, stride, mode, dtype="f32", workspace="full"):
        self.handle = ig.Handle()
        N, C, H, W = x.shape
        _, K, P, Q = dy.shape
        R, S = rs
        dt = _dt(dtype)
        self.x_dev, xs = to_device_strided(x, dtype)
        self.dy_dev, dys = to_device_strided(dy, dtype)
        self.xdesc = ig.TensorDescriptor().set(dt, N, C, H, W, xs)
        self.dydesc = ig.TensorDescriptor().set(dt, N, K, P, Q, dys)
        self.dwdesc = ig.FilterDescriptor().set(ig.IGC_DATA_DOUBLE if dtype == "f64" else ig.IGC_DATA_FLOAT, K, C, R, S)
        self.conv = ig.ConvolutionDescriptor().set(pad[0], pad[1], stride[0], stride[1], mode)
        self.out = GuardedOutput((K, C, R, S), (C * R * S, R * S, S, 1), dtype)
        self.asked = ig.get_backward_filter_workspace_size(self.handle, self.xdesc, self.dydesc, self.conv, self.dwdesc)
        self.ws_bytes = self.asked if workspace == "full" else (0 if workspace == "none" else int(workspace))
        es = 8 if dtype == "f64" else 4
        self.ws = GuardedOutput((1, 1, 1, max(self.ws_bytes // es, 1)), (0, 0, 0, 1), dtype)
        self.ws.prefill(value=float("nan"))

    def launch(self, alpha=1.0, beta=0.0):
        self.handle.set_stream(torch.cuda.current_stream().cuda_stream)
        st = ig.convolution_backward_filter(self.handle, alpha, self.xdesc, self.x_dev.data_ptr(), self.dydesc,
                                            self.dy_dev.data_ptr(), self.conv, beta, self.dwdesc, self.out.ptr,
                                            self.ws.ptr if self.ws_bytes else 0, self.ws_bytes)
        ig.check(st, "igcConvolutionBackwardFilter")


def run_backward_filter(x, dy, rs, pad=(0, 0), stride=(1, 1), mode=ig.IGC_CROSS_CORRELATION, alpha=1.0, beta=0.0,
                        dw_old=None, dtype="f32", workspace="full"):
    """One igcConvolutionBackwardFilter call; returns (dw as float64 (K,C,R,S), workspace
    bytes the library asked for)."""
    g = GpuBackwardFilter(x, dy, rs, pad, stride, mode, dtype, workspace)
    if dw_old is not None:
        g.out.prefill(old=dw_old)
    else:
        g.out.prefill(value=float("nan"))
    g.launch(alpha, beta)
    res = g.out.result()
    g.ws.result()   # guard bands of the workspace
    return res, g.asked


# ---------------------------------------------------------------- other functions
def _desc_for(a):
    """(device tensor, descriptor) of a float32 or float64 numpy array read through its strides."""
    dtype = "f64" if a.dtype == np.float64 else "f32"
    dev, strides = to_device_strided(a, dtype)
    return dev, ig.TensorDescriptor().set(_dt(dtype), *a.shape, strides)


def _handle():
    h = ig.Handle()
    h.set_stream(torch.cuda.current_stream().cuda_stream)
    return h


def _output(shape, layout, old, like=None):
    """Guarded output tensor of the element type of the array ``like`` (default float32)."""
    dtype = "f64" if like is not None and like.dtype == np.float64 else "f32"
    out = GuardedOutput(shape, layout_strides(shape, layout), dtype)
    if old is not None:
        out.prefill(old=old)
    else:
        out.prefill(value=float("nan"))
    return out, ig.TensorDescriptor().set(_dt(dtype), *shape, out.strides)


def run_activation_forward(mode, x, alpha=1.0, beta=0.0, y_old=None, layout="NCHW"):
    xd, xdesc = _desc_for(x)
    out, ydesc = _output(x.shape, layout, y_old, x)
    ig.check(ig.activation_forward(_handle(), mode, alpha, xdesc, xd.data_ptr(), beta, ydesc, out.ptr), "igcActivationForward")
    return out.result()


def run_activation_backward(mode, y, dy, x, alpha=1.0, beta=0.0, dx_old=None, layout="NCHW"):
    yd, ydesc = _desc_for(y)
    dyd, dydesc = _desc_for(dy)
    xd, xdesc = _desc_for(x)
    out, dxdesc = _output(x.shape, layout, dx_old, x)
    ig.check(ig.activation_backward(_handle(), mode, alpha, ydesc, yd.data_ptr(), dydesc, dyd.data_ptr(), xdesc,
                                    xd.data_ptr(), beta, dxdesc, out.ptr), "igcActivationBackward")
    return out.result()


def run_add_tensor(b, shape, alpha=1.0, beta=0.0, y_old=None, layout="NCHW"):
    bd, bdesc = _desc_for(b)
    out, ydesc = _output(tuple(shape), layout, y_old, b)
    ig.check(ig.add_tensor(_handle(), alpha, bdesc, bd.data_ptr(), beta, ydesc, out.ptr), "igcAddTensor")
    return out.result()


def run_backward_bias(dy, alpha=1.0, beta=0.0, db_old=None, dtype=None, workspace="full", db_stride=1, asked=None):
    """One igcConvolutionBackwardBias call; returns db (C values) as float64.  ``dtype``: "bf16" sends dy as bfloat16
    (default: dy's own float32 / float64); ``workspace``: "full" (what the library asks for), "none", or a number of
    bytes; ``db_stride``: element stride between db's feature maps; ``asked``: a list that receives the size asked for."""
    if dtype is None:
        dtype = "f64" if dy.dtype == np.float64 else "f32"
    dev, strides = to_device_strided(dy, dtype)
    dydesc = ig.TensorDescriptor().set(_dt(dtype), *dy.shape, strides)
    C = dy.shape[1]
    out_dtype = "f64" if dtype == "f64" else "f32"
    out = GuardedOutput((1, C, 1, 1), (C * db_stride, db_stride, 1, 1), out_dtype)
    if db_old is not None:
        out.prefill(old=np.asarray(db_old).reshape(1, C, 1, 1))
    else:
        out.prefill(value=float("nan"))
    dbdesc = ig.TensorDescriptor().set(_dt(out_dtype), 1, C, 1, 1, out.strides)
    h = _handle()
    want = ig.get_backward_bias_workspace_size(h, dydesc, dbdesc)
    if asked is not None:
        asked.append(want)
    ws_bytes = want if workspace == "full" else (0 if workspace == "none" else int(workspace))
    ws = GuardedOutput((1, 1, 1, max(ws_bytes // 8, 1)), (0, 0, 0, 1), "f64")
    ws.prefill(value=float("nan"))
    ig.check(ig.convolution_backward_bias(h, alpha, dydesc, dev.data_ptr(), beta, dbdesc, out.ptr, ws.ptr if ws_bytes else 0, ws_bytes),
             "igcConvolutionBackwardBias")
    res = out.result().reshape(C)
    ws.result()   # (guard bands of the workspace)
    return res


def run_softmax_forward(mode, x, alpha=1.0, beta=0.0, y_old=None, layout="NCHW"):
    xd, xdesc = _desc_for(x)
    out, ydesc = _output(x.shape, layout, y_old, x)
    ig.check(ig.softmax_forward(_handle(), mode, alpha, xdesc, xd.data_ptr(), beta, ydesc, out.ptr), "igcSoftmaxForward")
    return out.result()


def run_pooling_forward(mode, x, window, pad=(0, 0), stride=(1, 1), alpha=1.0, beta=0.0, y_old=None, layout="NCHW"):
    xd, xdesc = _desc_for(x)
    pool = ig.PoolingDescriptor().set(mode, window[0], window[1], pad[0], pad[1], stride[0], stride[1])
    shape = ig.get_pooling_output_dim(pool, xdesc)
    out, ydesc = _output(shape, layout, y_old, x)
    ig.check(ig.pooling_forward(_handle(), pool, alpha, xdesc, xd.data_ptr(), beta, ydesc, out.ptr), "igcPoolingForward")
    return out.result()


def run_softmax_backward(mode, y, dy, alpha=1.0, beta=0.0, dx_old=None, layout="NCHW"):
    yd, ydesc = _desc_for(y)
    dyd, dydesc = _desc_for(dy)
    out, dxdesc = _output(y.shape, layout, dx_old, y)
    ig.check(ig.softmax_backward(_handle(), mode, alpha, ydesc, yd.data_ptr(), dydesc, dyd.data_ptr(), beta, dxdesc, out.ptr),
             "igcSoftmaxBackward")
    return out.result()


def run_pooling_backward(mode, x, dy, window, pad=(0, 0), stride=(1, 1), alpha=1.0, beta=0.0, dx_old=None, layout="NCHW"):
    xd, xdesc = _desc_for(x)
    dyd, dydesc = _desc_for(dy)
    pool = ig.PoolingDescriptor().set(mode, window[0], window[1], pad[0], pad[1], stride[0], stride[1])
    out, dxdesc = _output(x.shape, layout, dx_old, x)
    ig.check(ig.pooling_backward(_handle(), pool, alpha, dydesc, dyd.data_ptr(), xdesc, xd.data_ptr(), beta, dxdesc, out.ptr),
             "igcPoolingBackward")
    return out.result()


def run_transform_tensor(x, alpha=1.0, beta=0.0, y_old=None, layout="NCHW", y_strides=None):
    """igcTransformTensor from x (read through its numpy strides) into a tensor of the given
    layout (or explicit element strides)."""
    xd, xdesc = _desc_for(x)
    if y_strides is None:
        out, ydesc = _output(x.shape, layout, y_old, x)
    else:
        dtype = "f64" if x.dtype == np.float64 else "f32"
        out = GuardedOutput(x.shape, y_strides, dtype)
        out.prefill(old=y_old) if y_old is not None else out.prefill(value=float("nan"))
        ydesc = ig.TensorDescriptor().set(_dt(dtype), *x.shape, out.strides)
    ig.check(ig.transform_tensor(_handle(), alpha, xdesc, xd.data_ptr(), beta, ydesc, out.ptr), "igcTransformTensor")
    return out.result()
