"""ctypes binding of the C ABI in ``include/igconv.h`` - same names, same arguments.

Argument marshalling only.  ``lib()`` loads the in-tree ``libigconv.so`` and raises
if it is absent (run ``python -c "import __graft_entry__ as g; g.build()"`` or
``python paper_1410_0759_amd/build.py`` first); nothing here computes anything.
"""
import ctypes
import os

__all__ = [
    "lib", "IgcError", "check",
    "IGC_STATUS_SUCCESS", "IGC_STATUS_BAD_PARAM", "IGC_STATUS_NOT_SUPPORTED",
    "IGC_STATUS_NOT_INITIALIZED", "IGC_STATUS_ALLOC_FAILED", "IGC_STATUS_EXECUTION_FAILED",
    "IGC_DATA_FLOAT", "IGC_DATA_BFLOAT16", "IGC_DATA_DOUBLE", "IGC_CONVOLUTION", "IGC_CROSS_CORRELATION",
    "igcConvolutionForwardPlan", "DECLARED_SYMBOLS",
    "Handle", "TensorDescriptor", "FilterDescriptor", "ConvolutionDescriptor",
    "get_output_dim", "get_workspace_size", "get_optional_workspace_size", "get_plan", "convolution_forward",
    "get_backward_data_workspace_size", "convolution_backward_data",
    "get_backward_filter_workspace_size", "convolution_backward_filter",
    "PoolingDescriptor", "get_pooling_output_dim", "activation_forward", "activation_backward", "add_tensor",
    "softmax_forward", "pooling_forward", "softmax_backward", "pooling_backward", "transform_tensor", "convolution_bias_activation_forward", "IGC_ACTIVATION_IDENTITY",
    "IGC_ACTIVATION_SIGMOID", "IGC_ACTIVATION_RELU", "IGC_ACTIVATION_TANH", "IGC_SOFTMAX_MODE_INSTANCE",
    "IGC_SOFTMAX_MODE_CHANNEL", "IGC_POOLING_MAX", "IGC_POOLING_AVERAGE",
    "kernel_names", "magic_divisor", "magic_divide", "tensor_descriptor_for",
    "get_device_properties", "measure_matrix_rate", "measure_matrix_rate_operands", "convolution_backward_filter_no_alloc", "NOALLOC_SCRATCH_BYTES",
    "get_backward_bias_workspace_size", "convolution_backward_bias", "set_compute_units", "get_compute_units", "get_forward_address_reach", "get_backward_data_address_reach",
]

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libigconv.so")

(IGC_STATUS_SUCCESS, IGC_STATUS_BAD_PARAM, IGC_STATUS_NOT_SUPPORTED,
 IGC_STATUS_NOT_INITIALIZED, IGC_STATUS_ALLOC_FAILED, IGC_STATUS_EXECUTION_FAILED) = range(6)
IGC_DATA_FLOAT, IGC_DATA_BFLOAT16, IGC_DATA_DOUBLE = 0, 1, 2
IGC_CONVOLUTION, IGC_CROSS_CORRELATION = 0, 1
IGC_ACTIVATION_SIGMOID, IGC_ACTIVATION_RELU, IGC_ACTIVATION_TANH = 0, 1, 2
IGC_ACTIVATION_IDENTITY = -1
IGC_SOFTMAX_MODE_INSTANCE, IGC_SOFTMAX_MODE_CHANNEL = 0, 1
IGC_POOLING_MAX, IGC_POOLING_AVERAGE = 0, 1


class igcConvolutionForwardPlan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in (
        "kernelId", "tileM", "tileN", "tileK", "gridX", "kSteps", "threads", "ldsBytes",
        "swapOperands", "vecFilterLoads", "gatherMode")]


_vp, _i, _ll, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_size_t
_P = ctypes.POINTER

# name -> (restype, argtypes): every symbol include/igconv.h declares
DECLARED_SYMBOLS = {
    "igcGetErrorString": (ctypes.c_char_p, [_i]),
    "igcCreate": (_i, [_P(_vp)]),
    "igcDestroy": (_i, [_vp]),
    "igcSetStream": (_i, [_vp, _vp]),
    "igcGetStream": (_i, [_vp, _P(_vp)]),
    "igcCreateTensorDescriptor": (_i, [_P(_vp)]),
    "igcDestroyTensorDescriptor": (_i, [_vp]),
    "igcSetTensor4dDescriptor": (_i, [_vp, _i, _i, _i, _i, _i, _ll, _ll, _ll, _ll]),
    "igcGetTensor4dDescriptor": (_i, [_vp, _P(_i), _P(_i), _P(_i), _P(_i), _P(_i),
                                      _P(_ll), _P(_ll), _P(_ll), _P(_ll)]),
    "igcCreateFilterDescriptor": (_i, [_P(_vp)]),
    "igcDestroyFilterDescriptor": (_i, [_vp]),
    "igcSetFilter4dDescriptor": (_i, [_vp, _i, _i, _i, _i, _i]),
    "igcGetFilter4dDescriptor": (_i, [_vp, _P(_i), _P(_i), _P(_i), _P(_i), _P(_i)]),
    "igcCreateConvolutionDescriptor": (_i, [_P(_vp)]),
    "igcDestroyConvolutionDescriptor": (_i, [_vp]),
    "igcSetConvolution2dDescriptor": (_i, [_vp, _i, _i, _i, _i, _i]),
    "igcGetConvolution2dDescriptor": (_i, [_vp, _P(_i), _P(_i), _P(_i), _P(_i), _P(_i)]),
    "igcGetConvolution2dForwardOutputDim": (_i, [_vp, _vp, _vp, _P(_i), _P(_i), _P(_i), _P(_i)]),
    "igcGetConvolutionForwardWorkspaceSize": (_i, [_vp, _vp, _vp, _vp, _vp, _P(_sz)]),
    "igcGetConvolutionForwardOptionalWorkspaceSize": (_i, [_vp, _vp, _vp, _vp, _vp, _P(_sz)]),
    "igcConvolutionForward": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp, _vp]),
    "igcGetConvolutionBackwardDataWorkspaceSize": (_i, [_vp, _vp, _vp, _vp, _vp, _P(_sz)]),
    "igcConvolutionBackwardData": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp, _vp]),
    "igcGetConvolutionBackwardFilterWorkspaceSize": (_i, [_vp, _vp, _vp, _vp, _vp, _P(_sz)]),
    "igcConvolutionBackwardFilter": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp, _vp]),
    "igcActivationForward": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcActivationBackward": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcAddTensor": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcGetConvolutionBackwardBiasWorkspaceSize": (_i, [_vp, _vp, _vp, _P(_sz)]),
    "igcConvolutionBackwardBias": (_i, [_vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp, _vp]),
    "igcSoftmaxForward": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcCreatePoolingDescriptor": (_i, [_P(_vp)]),
    "igcDestroyPoolingDescriptor": (_i, [_vp]),
    "igcSetPooling2dDescriptor": (_i, [_vp, _i, _i, _i, _i, _i, _i, _i]),
    "igcGetPooling2dDescriptor": (_i, [_vp] + [_P(_i)] * 7),
    "igcGetPooling2dForwardOutputDim": (_i, [_vp, _vp, _P(_i), _P(_i), _P(_i), _P(_i)]),
    "igcPoolingForward": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcSoftmaxBackward": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcTransformTensor": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcPoolingBackward": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcConvolutionBiasActivationForward": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp, _i, _vp, _vp]),
    "igcGetConvolutionForwardPlan": (_i, [_vp, _vp, _vp, _vp, _vp, _P(igcConvolutionForwardPlan)]),
    "igcGetKernelCount": (_i, []),
    "igcGetKernelName": (ctypes.c_char_p, [_i]),
    "igcSetKernelOverride": (_i, [_vp, _i]),
    "igcMagicDivisor": (_i, [ctypes.c_uint, _P(ctypes.c_uint), _P(ctypes.c_uint)]),
    "igcMagicDivide": (ctypes.c_uint, [ctypes.c_uint, ctypes.c_uint, ctypes.c_uint]),
    "igcConvolutionBackwardFilterNoAlloc": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "igcGetDeviceProperties": (_i, [_vp, _P(_i), _P(_i)]),
    "igcMeasureMatrixRate": (_i, [_vp, _i, _i, _P(ctypes.c_double)]),
    "igcMeasureMatrixRateOperands": (_i, [_vp, _i, _i, _i, _P(ctypes.c_double)]),
    "igcSetComputeUnits": (_i, [_vp, _i]),
    "igcGetComputeUnits": (_i, [_vp, _P(_i)]),
    "igcGetConvolutionForwardAddressReach": (_i, [_vp, _vp, _vp, _vp, _vp, _P(ctypes.c_longlong), _P(ctypes.c_longlong)]),
    "igcGetConvolutionBackwardDataAddressReach": (_i, [_vp, _vp, _vp, _vp, _vp, _P(ctypes.c_longlong), _P(ctypes.c_longlong)]),
}

_lib = None


def lib():
    """The loaded shared library with argument types set; raises if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libigconv.so is not built (%s); build it with paper_1410_0759_amd/build.py. "
                "There is no fallback path." % LIB_PATH)
        # A process may hold one HIP runtime only.  PyTorch-ROCm ships its own copy; when the
        # caller is going to use PyTorch for device memory and streams, that copy has to be
        # the one loaded first (libigconv.so then binds to it).  Loaded the other way round,
        # the two runtimes conflict and every launch reports that no device is present.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in DECLARED_SYMBOLS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


class IgcError(RuntimeError):
    def __init__(self, status, where=""):
        self.status = status
        name = lib().igcGetErrorString(status).decode()
        super().__init__("%s%s" % (name, " in " + where if where else ""))


def check(status, where=""):
    if status != IGC_STATUS_SUCCESS:
        raise IgcError(status, where)


class _Owned:
    _create = _destroy = None

    def __init__(self):
        self.ptr = _vp()
        check(getattr(lib(), self._create)(ctypes.byref(self.ptr)), self._create)

    def close(self):
        if self.ptr:
            getattr(lib(), self._destroy)(self.ptr)
            self.ptr = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Handle(_Owned):
    _create, _destroy = "igcCreate", "igcDestroy"

    def set_stream(self, stream_ptr):
        """``stream_ptr``: integer value of a hipStream_t (e.g. torch's ``cuda_stream``), 0 = default."""
        check(lib().igcSetStream(self.ptr, _vp(stream_ptr)), "igcSetStream")

    def get_stream(self):
        out = _vp()
        check(lib().igcGetStream(self.ptr, ctypes.byref(out)), "igcGetStream")
        return out.value or 0

    def set_kernel_override(self, kernel_id):
        check(lib().igcSetKernelOverride(self.ptr, kernel_id), "igcSetKernelOverride")


def _scalars(out_desc, alpha, beta):
    """alpha and beta as the host scalars the library expects: doubles for double-precision
    problems (told by the output's descriptor), floats otherwise."""
    dt = getattr(out_desc, "dtype", None)      # (remembered by set(): no library call on the launch path)
    if dt is None:
        dt = out_desc.get()[0]
    t = ctypes.c_double if dt == IGC_DATA_DOUBLE else ctypes.c_float
    return t(alpha), t(beta)


class TensorDescriptor(_Owned):
    _create, _destroy = "igcCreateTensorDescriptor", "igcDestroyTensorDescriptor"

    def set(self, dtype, n, c, h, w, strides):
        check(lib().igcSetTensor4dDescriptor(self.ptr, dtype, n, c, h, w, *[int(s) for s in strides]),
              "igcSetTensor4dDescriptor")
        self.dtype = dtype
        return self

    def get(self):
        dt, d = _i(), [_i() for _ in range(4)]
        s = [_ll() for _ in range(4)]
        check(lib().igcGetTensor4dDescriptor(self.ptr, ctypes.byref(dt), *[ctypes.byref(v) for v in d + s]),
              "igcGetTensor4dDescriptor")
        return dt.value, tuple(v.value for v in d), tuple(v.value for v in s)


class FilterDescriptor(_Owned):
    _create, _destroy = "igcCreateFilterDescriptor", "igcDestroyFilterDescriptor"

    def set(self, dtype, k, c, r, s):
        check(lib().igcSetFilter4dDescriptor(self.ptr, dtype, k, c, r, s), "igcSetFilter4dDescriptor")
        self.dtype = dtype
        return self

    def get(self):
        v = [_i() for _ in range(5)]
        check(lib().igcGetFilter4dDescriptor(self.ptr, *[ctypes.byref(a) for a in v]), "igcGetFilter4dDescriptor")
        return tuple(a.value for a in v)


class ConvolutionDescriptor(_Owned):
    _create, _destroy = "igcCreateConvolutionDescriptor", "igcDestroyConvolutionDescriptor"

    def set(self, pad_h, pad_w, u, v, mode):
        check(lib().igcSetConvolution2dDescriptor(self.ptr, pad_h, pad_w, u, v, mode),
              "igcSetConvolution2dDescriptor")
        return self

    def get(self):
        v = [_i() for _ in range(5)]
        check(lib().igcGetConvolution2dDescriptor(self.ptr, *[ctypes.byref(a) for a in v]),
              "igcGetConvolution2dDescriptor")
        return tuple(a.value for a in v)


class PoolingDescriptor(_Owned):
    _create, _destroy = "igcCreatePoolingDescriptor", "igcDestroyPoolingDescriptor"

    def set(self, mode, win_h, win_w, pad_h, pad_w, u, v):
        check(lib().igcSetPooling2dDescriptor(self.ptr, mode, win_h, win_w, pad_h, pad_w, u, v),
              "igcSetPooling2dDescriptor")
        return self

    def get(self):
        v = [_i() for _ in range(7)]
        check(lib().igcGetPooling2dDescriptor(self.ptr, *[ctypes.byref(a) for a in v]), "igcGetPooling2dDescriptor")
        return tuple(a.value for a in v)


def get_pooling_output_dim(pool, xdesc):
    v = [_i() for _ in range(4)]
    check(lib().igcGetPooling2dForwardOutputDim(pool.ptr, xdesc.ptr, *[ctypes.byref(a) for a in v]),
          "igcGetPooling2dForwardOutputDim")
    return tuple(a.value for a in v)


def activation_forward(handle, mode, alpha, xdesc, x_ptr, beta, ydesc, y_ptr):
    a, b = _scalars(ydesc, alpha, beta)
    return lib().igcActivationForward(handle.ptr, mode, ctypes.byref(a), xdesc.ptr, _vp(x_ptr), ctypes.byref(b),
                                      ydesc.ptr, _vp(y_ptr))


def activation_backward(handle, mode, alpha, ydesc, y_ptr, dydesc, dy_ptr, xdesc, x_ptr, beta, dxdesc, dx_ptr):
    a, b = _scalars(dxdesc, alpha, beta)
    return lib().igcActivationBackward(handle.ptr, mode, ctypes.byref(a), ydesc.ptr, _vp(y_ptr), dydesc.ptr, _vp(dy_ptr),
                                       xdesc.ptr, _vp(x_ptr), ctypes.byref(b), dxdesc.ptr, _vp(dx_ptr))


def add_tensor(handle, alpha, bdesc, b_ptr, beta, ydesc, y_ptr):
    a, b = _scalars(ydesc, alpha, beta)
    return lib().igcAddTensor(handle.ptr, ctypes.byref(a), bdesc.ptr, _vp(b_ptr), ctypes.byref(b), ydesc.ptr, _vp(y_ptr))


def get_backward_bias_workspace_size(handle, dydesc, dbdesc):
    out = _sz()
    check(lib().igcGetConvolutionBackwardBiasWorkspaceSize(handle.ptr, dydesc.ptr, dbdesc.ptr, ctypes.byref(out)),
          "igcGetConvolutionBackwardBiasWorkspaceSize")
    return out.value


def convolution_backward_bias(handle, alpha, dydesc, dy_ptr, beta, dbdesc, db_ptr, workspace_ptr=0, workspace_bytes=0):
    a, b = _scalars(dbdesc, alpha, beta)
    return lib().igcConvolutionBackwardBias(handle.ptr, ctypes.byref(a), dydesc.ptr, _vp(dy_ptr), _vp(workspace_ptr), workspace_bytes,
                                            ctypes.byref(b), dbdesc.ptr, _vp(db_ptr))


def softmax_forward(handle, mode, alpha, xdesc, x_ptr, beta, ydesc, y_ptr):
    a, b = _scalars(ydesc, alpha, beta)
    return lib().igcSoftmaxForward(handle.ptr, mode, ctypes.byref(a), xdesc.ptr, _vp(x_ptr), ctypes.byref(b),
                                   ydesc.ptr, _vp(y_ptr))


def pooling_forward(handle, pool, alpha, xdesc, x_ptr, beta, ydesc, y_ptr):
    a, b = _scalars(ydesc, alpha, beta)
    return lib().igcPoolingForward(handle.ptr, pool.ptr, ctypes.byref(a), xdesc.ptr, _vp(x_ptr), ctypes.byref(b),
                                   ydesc.ptr, _vp(y_ptr))


def transform_tensor(handle, alpha, xdesc, x_ptr, beta, ydesc, y_ptr):
    a, b = _scalars(ydesc, alpha, beta)
    return lib().igcTransformTensor(handle.ptr, ctypes.byref(a), xdesc.ptr, _vp(x_ptr), ctypes.byref(b), ydesc.ptr, _vp(y_ptr))


def softmax_backward(handle, mode, alpha, ydesc, y_ptr, dydesc, dy_ptr, beta, dxdesc, dx_ptr):
    a, b = _scalars(dxdesc, alpha, beta)
    return lib().igcSoftmaxBackward(handle.ptr, mode, ctypes.byref(a), ydesc.ptr, _vp(y_ptr), dydesc.ptr, _vp(dy_ptr),
                                    ctypes.byref(b), dxdesc.ptr, _vp(dx_ptr))


def pooling_backward(handle, pool, alpha, dydesc, dy_ptr, xdesc, x_ptr, beta, dxdesc, dx_ptr):
    a, b = _scalars(dxdesc, alpha, beta)
    return lib().igcPoolingBackward(handle.ptr, pool.ptr, ctypes.byref(a), dydesc.ptr, _vp(dy_ptr), xdesc.ptr, _vp(x_ptr),
                                    ctypes.byref(b), dxdesc.ptr, _vp(dx_ptr))


def get_output_dim(conv, xdesc, wdesc):
    v = [_i() for _ in range(4)]
    check(lib().igcGetConvolution2dForwardOutputDim(conv.ptr, xdesc.ptr, wdesc.ptr, *[ctypes.byref(a) for a in v]),
          "igcGetConvolution2dForwardOutputDim")
    return tuple(a.value for a in v)


def get_workspace_size(handle, xdesc, wdesc, conv, ydesc):
    out = _sz(12345)
    check(lib().igcGetConvolutionForwardWorkspaceSize(handle.ptr, xdesc.ptr, wdesc.ptr, conv.ptr, ydesc.ptr,
                                                      ctypes.byref(out)), "igcGetConvolutionForwardWorkspaceSize")
    return out.value


def get_optional_workspace_size(handle, xdesc, wdesc, conv, ydesc):
    out = _sz(12345)
    check(lib().igcGetConvolutionForwardOptionalWorkspaceSize(handle.ptr, xdesc.ptr, wdesc.ptr, conv.ptr, ydesc.ptr,
                                                              ctypes.byref(out)),
          "igcGetConvolutionForwardOptionalWorkspaceSize")
    return out.value


def get_plan(handle, xdesc, wdesc, conv, ydesc):
    plan = igcConvolutionForwardPlan()
    check(lib().igcGetConvolutionForwardPlan(handle.ptr, xdesc.ptr, wdesc.ptr, conv.ptr, ydesc.ptr,
                                             ctypes.byref(plan)), "igcGetConvolutionForwardPlan")
    return plan


def convolution_forward(handle, alpha, xdesc, x_ptr, wdesc, w_ptr, conv, beta, ydesc, y_ptr,
                        workspace_ptr=0, workspace_bytes=0):
    """igcConvolutionForward with device pointers given as integers; returns the status."""
    a, b = _scalars(ydesc, alpha, beta)
    return lib().igcConvolutionForward(
        handle.ptr, ctypes.byref(a), xdesc.ptr, _vp(x_ptr), wdesc.ptr, _vp(w_ptr), conv.ptr,
        _vp(workspace_ptr), workspace_bytes, ctypes.byref(b), ydesc.ptr, _vp(y_ptr))


def get_backward_data_workspace_size(handle, wdesc, dydesc, conv, dxdesc):
    out = _sz(12345)
    check(lib().igcGetConvolutionBackwardDataWorkspaceSize(handle.ptr, wdesc.ptr, dydesc.ptr, conv.ptr, dxdesc.ptr,
                                                           ctypes.byref(out)),
          "igcGetConvolutionBackwardDataWorkspaceSize")
    return out.value


def convolution_backward_data(handle, alpha, wdesc, w_ptr, dydesc, dy_ptr, conv, beta, dxdesc, dx_ptr,
                              workspace_ptr=0, workspace_bytes=0):
    """igcConvolutionBackwardData with device pointers given as integers; returns the status."""
    a, b = _scalars(dxdesc, alpha, beta)
    return lib().igcConvolutionBackwardData(
        handle.ptr, ctypes.byref(a), wdesc.ptr, _vp(w_ptr), dydesc.ptr, _vp(dy_ptr), conv.ptr,
        _vp(workspace_ptr), workspace_bytes, ctypes.byref(b), dxdesc.ptr, _vp(dx_ptr))


def get_backward_filter_workspace_size(handle, xdesc, dydesc, conv, dwdesc):
    out = _sz(12345)
    check(lib().igcGetConvolutionBackwardFilterWorkspaceSize(handle.ptr, xdesc.ptr, dydesc.ptr, conv.ptr, dwdesc.ptr,
                                                             ctypes.byref(out)),
          "igcGetConvolutionBackwardFilterWorkspaceSize")
    return out.value


def convolution_backward_filter(handle, alpha, xdesc, x_ptr, dydesc, dy_ptr, conv, beta, dwdesc, dw_ptr,
                                workspace_ptr=0, workspace_bytes=0):
    """igcConvolutionBackwardFilter with device pointers given as integers; returns the status."""
    a, b = _scalars(dwdesc, alpha, beta)
    return lib().igcConvolutionBackwardFilter(
        handle.ptr, ctypes.byref(a), xdesc.ptr, _vp(x_ptr), dydesc.ptr, _vp(dy_ptr), conv.ptr,
        _vp(workspace_ptr), workspace_bytes, ctypes.byref(b), dwdesc.ptr, _vp(dw_ptr))


NOALLOC_SCRATCH_BYTES = 64 << 20   # IGC_NOALLOC_SCRATCH_BYTES of include/igconv.h


def convolution_backward_filter_no_alloc(handle, alpha, xdesc, x_ptr, dydesc, dy_ptr, conv, beta, dwdesc, dw_ptr):
    """igcConvolutionBackwardFilterNoAlloc (no workspace argument: the library's own scratch array); returns the status."""
    a, b = _scalars(dwdesc, alpha, beta)
    return lib().igcConvolutionBackwardFilterNoAlloc(
        handle.ptr, ctypes.byref(a), xdesc.ptr, _vp(x_ptr), dydesc.ptr, _vp(dy_ptr), conv.ptr,
        ctypes.byref(b), dwdesc.ptr, _vp(dw_ptr))


def convolution_bias_activation_forward(handle, alpha, xdesc, x_ptr, wdesc, w_ptr, conv, beta, bias_ptr, activation,
                                        ydesc, y_ptr, ws_ptr=0, ws_bytes=0):
    """igcConvolutionBiasActivationForward; bias_ptr 0 for no bias, activation -1 for none."""
    a, b = _scalars(ydesc, alpha, beta)
    return lib().igcConvolutionBiasActivationForward(
        handle.ptr, ctypes.byref(a), xdesc.ptr, _vp(x_ptr), wdesc.ptr, _vp(w_ptr), conv.ptr, _vp(ws_ptr) if ws_ptr else None,
        ws_bytes, ctypes.byref(b), _vp(bias_ptr), activation, ydesc.ptr, _vp(y_ptr))


def kernel_names():
    L = lib()
    return [L.igcGetKernelName(i).decode() for i in range(L.igcGetKernelCount())]


def get_device_properties(handle):
    """(compute units, engine clock in kHz) of the current device."""
    cus, khz = _i(), _i()
    check(lib().igcGetDeviceProperties(handle.ptr, ctypes.byref(cus), ctypes.byref(khz)), "igcGetDeviceProperties")
    return cus.value, khz.value


def measure_matrix_rate(handle, dtype, milliseconds=50):
    """TFLOP/s of a register-only loop of the data type's matrix instruction (waits for the GPU)."""
    out = ctypes.c_double()
    check(lib().igcMeasureMatrixRate(handle.ptr, dtype, milliseconds, ctypes.byref(out)), "igcMeasureMatrixRate")
    return out.value


def measure_matrix_rate_operands(handle, dtype, milliseconds=50, random_operands=1):
    """The same with a choice of operand values: 0 uniform (as measure_matrix_rate), 1 pseudo-random, changing with every instruction."""
    out = ctypes.c_double()
    check(lib().igcMeasureMatrixRateOperands(handle.ptr, dtype, milliseconds, random_operands, ctypes.byref(out)), "igcMeasureMatrixRateOperands")
    return out.value


def set_compute_units(handle, compute_units):
    check(lib().igcSetComputeUnits(handle.ptr, compute_units), "igcSetComputeUnits")


def get_compute_units(handle):
    out = _i()
    check(lib().igcGetComputeUnits(handle.ptr, ctypes.byref(out)), "igcGetComputeUnits")
    return out.value


def get_forward_address_reach(handle, xdesc, wdesc, conv, ydesc):
    """((reach of x, w, y), (extent of x, w, y)) in bytes for the forward pass."""
    reach, extent = (ctypes.c_longlong * 3)(), (ctypes.c_longlong * 3)()
    check(lib().igcGetConvolutionForwardAddressReach(handle.ptr, xdesc.ptr, wdesc.ptr, conv.ptr, ydesc.ptr, reach, extent),
          "igcGetConvolutionForwardAddressReach")
    return tuple(reach), tuple(extent)


def get_backward_data_address_reach(handle, wdesc, dydesc, conv, dxdesc):
    """((reach of dy, w, dx), (extent of dy, w, dx)) in bytes for backward data."""
    reach, extent = (ctypes.c_longlong * 3)(), (ctypes.c_longlong * 3)()
    check(lib().igcGetConvolutionBackwardDataAddressReach(handle.ptr, wdesc.ptr, dydesc.ptr, conv.ptr, dxdesc.ptr, reach, extent),
          "igcGetConvolutionBackwardDataAddressReach")
    return tuple(reach), tuple(extent)


def magic_divisor(d):
    mul, shift = ctypes.c_uint(), ctypes.c_uint()
    check(lib().igcMagicDivisor(d, ctypes.byref(mul), ctypes.byref(shift)), "igcMagicDivisor")
    return mul.value, shift.value


def magic_divide(n, mul, shift):
    return lib().igcMagicDivide(n, mul, shift)


def tensor_descriptor_for(t, dtype=None):
    """Descriptor for a logically-NCHW 4-D torch tensor or numpy array, read from its
    shape and strides (any memory order)."""
    if hasattr(t, "element_size"):  # torch
        strides = t.stride()
        is_bf16 = "bfloat16" in str(t.dtype)
    else:  # numpy
        strides = [s // t.itemsize for s in t.strides]
        is_bf16 = False
    if dtype is None:
        dtype = IGC_DATA_BFLOAT16 if is_bf16 else (IGC_DATA_DOUBLE if "float64" in str(t.dtype) else IGC_DATA_FLOAT)
    n, c, h, w = t.shape
    return TensorDescriptor().set(dtype, n, c, h, w, strides)
