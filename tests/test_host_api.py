"""CPU-only tests of the C-ABI library: it loads, exports every declared symbol, and
its host logic (validation, output size, plan, magic division) behaves as the header
says.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1410_0759_amd as ig
from oracle import conv_oracle as oc
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "igconv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(igc[A-Z]\w*)\s*\(", header))
    assert declared, "no declarations found"
    L = ig.lib()
    for name in declared:
        assert hasattr(L, name), "library lacks %s" % name
    assert declared == set(ig.DECLARED_SYMBOLS), declared ^ set(ig.DECLARED_SYMBOLS)


def test_error_strings():
    L = ig.lib()
    names = {L.igcGetErrorString(i).decode() for i in range(6)}
    assert len(names) == 6 and all(n.startswith("IGC_STATUS_") for n in names)
    assert L.igcGetErrorString(99) is not None


def _descs(N=2, C=3, H=8, W=8, K=4, R=3, S=3, pad=(1, 1), stride=(1, 1), mode=1, dt=0,
           xs=None, ys=None, ydims=None, ydt=0):
    x = ig.TensorDescriptor().set(dt, N, C, H, W, xs or (C * H * W, H * W, W, 1))
    w = ig.FilterDescriptor().set(dt, K, C, R, S)
    c = ig.ConvolutionDescriptor().set(pad[0], pad[1], stride[0], stride[1], mode)
    n, k, p, q = ydims or ig.get_output_dim(c, x, w)
    y = ig.TensorDescriptor().set(ydt, n, k, p, q, ys or (k * p * q, p * q, q, 1))
    return x, w, c, y


def test_descriptor_roundtrip():
    x, w, c, y = _descs()
    assert x.get() == (0, (2, 3, 8, 8), (192, 64, 8, 1))
    assert w.get() == (0, 4, 3, 3, 3)
    assert c.get() == (1, 1, 1, 1, 1)


def test_output_dim_matches_eq1():
    rng = np.random.default_rng(0)
    for _ in range(300):
        H, W = int(rng.integers(1, 60)), int(rng.integers(1, 60))
        R, S = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        pad = (int(rng.integers(0, 4)), int(rng.integers(0, 4)))
        st = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        x = ig.TensorDescriptor().set(0, 2, 3, H, W, (3 * H * W, H * W, W, 1))
        w = ig.FilterDescriptor().set(0, 5, 3, R, S)
        c = ig.ConvolutionDescriptor().set(pad[0], pad[1], st[0], st[1], 0)
        P, Q = oc.output_dim(H, R, st[0], pad[0]), oc.output_dim(W, S, st[1], pad[1])
        if P < 1 or Q < 1:
            with pytest.raises(ig.IgcError) as e:
                ig.get_output_dim(c, x, w)
            assert e.value.status == ig.IGC_STATUS_BAD_PARAM
        else:
            assert ig.get_output_dim(c, x, w) == (2, 5, P, Q)


def test_workload_dims_and_plans():
    h = ig.Handle()
    for w_ in wl.WORKLOADS:
        dt = 1 if w_.dtype == "bf16" else 0
        nchw = lambda n, c, hh, ww: (c * hh * ww, hh * ww, ww, 1)
        nhwc = lambda n, c, hh, ww: (hh * ww * c, 1, ww * c, c)
        xs = (nchw if w_.x_layout == "NCHW" else nhwc)(w_.N, w_.C, w_.H, w_.W)
        ys = (nchw if w_.y_layout == "NCHW" else nhwc)(w_.N, w_.K, w_.P, w_.Q)
        x, w, c, y = _descs(w_.N, w_.C, w_.H, w_.W, w_.K, w_.R, w_.S, (w_.pad_h, w_.pad_w), (w_.u, w_.v),
                            w_.mode, dt, xs=xs, ys=ys)
        assert ig.get_output_dim(c, x, w) == (w_.N, w_.K, w_.P, w_.Q)
        assert ig.get_workspace_size(h, x, w, c, y) == 0
        plan = ig.get_plan(h, x, w, c, y)
        name = ig.kernel_names()[plan.kernelId]
        assert name.startswith(w_.dtype)
        tiles = -(-w_.K // plan.tileM) * -(-(w_.N * w_.P * w_.Q) // plan.tileN)
        per_xcd = -(-tiles // 8)
        if plan.gatherMode not in (4, 5):   # persistent workgroups: at most what 32 compute units per XCD hold
            # (two by LDS and registers; three or, for tiles up to 64 x 128, four for the kernels with steps of 16)
            by_regs = (4 if plan.tileM * plan.tileN <= 64 * 128 else 3) if plan.tileK == 16 else (
                4 if plan.gatherMode == 2 and plan.tileM * plan.tileN <= 64 * 64 and plan.tileK == 32 else 2)
            per_xcd = min(per_xcd, 32 * max(1, min(by_regs, 160 * 1024 // plan.ldsBytes)))
        assert plan.gridX == 8 * per_xcd
        assert plan.kSteps in (-(-(w_.C * w_.R * w_.S) // plan.tileK), w_.R * w_.S * -(-w_.C // plan.tileK))
        assert plan.ldsBytes <= 160 * 1024
        assert plan.swapOperands == (1 if w_.y_layout == "NHWC" else 0)
        if w_ is wl.WORKLOADS[1]:
            # 363 reduction indices, unpadded, 96 output channels: tap offsets from the LDS table, 23 steps
            # of 16 (three workgroups per compute unit), the step that rounds 23 up is not multiplied
            assert (plan.gatherMode, plan.kSteps, plan.tileM, plan.tileK) == (13, 23, 96, 16)


def test_optional_forward_workspace_is_only_asked_for_where_cutting_the_reduction_pays():
    """The mandatory workspace query reports zero for every problem; the optional one a whole
    number of copies of y for a problem with few tiles and a long reduction, zero otherwise."""
    h = ig.Handle()
    small = _descs(N=2, C=128, H=17, W=17, K=128, R=7, S=7, pad=(0, 0))
    assert ig.get_workspace_size(h, *small) == 0
    ws = ig.get_optional_workspace_size(h, *small)
    ybytes = 2 * 128 * 11 * 11 * 4
    assert ws >= 2 * ybytes and ws % ybytes == 0
    for w_ in wl.WORKLOADS[1:4]:     # the fp32 workloads fill the chip: nothing to gain
        nchw = lambda n, c, hh, ww: (c * hh * ww, hh * ww, ww, 1)
        d = _descs(w_.N, w_.C, w_.H, w_.W, w_.K, w_.R, w_.S, (w_.pad_h, w_.pad_w), (w_.u, w_.v), w_.mode, 0,
                   xs=nchw(w_.N, w_.C, w_.H, w_.W), ys=nchw(w_.N, w_.K, w_.P, w_.Q))
        assert ig.get_optional_workspace_size(h, *d) == 0
    # a float problem in tap-major order with plenty of tiles: room for the filter with the channel index innermost
    # (more than 63 taps; with fewer a padded float layer runs in filter order with a mask of the taps outside, and asks for nothing)
    big = _descs(N=64, C=64, H=20, W=20, K=70, R=9, S=9, pad=(4, 4))
    assert ig.get_plan(h, *big).gatherMode == 1
    assert ig.get_optional_workspace_size(h, *big) == 70 * 64 * 81 * 4 and ig.get_workspace_size(h, *big) == 0
    masked = _descs(N=64, C=64, H=20, W=20, K=70, R=5, S=5, pad=(2, 2))
    assert ig.get_plan(h, *masked).gatherMode == 14 and ig.get_optional_workspace_size(h, *masked) == 0
    # a short reduction is never cut; neither is an output with gaps between its elements
    assert ig.get_optional_workspace_size(h, *_descs(N=2, C=3, H=17, W=17, K=16, R=3, S=3, pad=(0, 0))) == 0
    # few channels and a zero border: room for x with the border written out
    assert ig.get_optional_workspace_size(h, *_descs(N=2, C=3, H=17, W=17, K=16, R=3, S=3)) == 2 * 3 * 19 * 19 * 4
    gaps = _descs(N=2, C=128, H=17, W=17, K=128, R=7, S=7, pad=(0, 0), ys=(128 * 11 * 12, 11 * 12, 12, 1))
    assert ig.get_optional_workspace_size(h, *gaps) == 0


def test_bf16_channel_vector_modes_are_offered_only_where_they_apply():
    """bf16, nine taps, channels contiguous and in sixteens: 16-byte channel vectors, read from
    a staged patch of the zero-extended image while every tile's pixel range fits it (512
    pixels), else gathered tap by tap; any other layout falls back to the element-wise kernels."""
    h = ig.Handle()
    nhwc = lambda c, hh, ww: (hh * ww * c, 1, ww * c, c)

    def mode(N, C, H, W, K, R=3, S=3, pad=(1, 1), stride=(1, 1), xs=None):
        x, w, c, y = _descs(N, C, H, W, K, R, S, pad, stride, 1, 1, xs=xs or nhwc(C, H, W))
        return ig.get_plan(h, x, w, c, y)

    p5 = mode(32, 512, 14, 14, 512)
    # (200 tiles for 256 compute units: the kernel with two groups of multipliers, steps of 32 channels, 12 wavefronts)
    assert p5.gatherMode == 5 and p5.kSteps == 512 // 32 and p5.tileK == 288 and p5.threads == 768 and p5.gridX == 200
    p5 = mode(256, 512, 14, 14, 512)
    assert p5.gatherMode == 5 and p5.kSteps == 512 // 16 and p5.tileK == 144 and (p5.tileM, p5.tileN) == (128, 256)
    assert mode(2, 32, 10, 12, 8, 1, 9, (0, 4)).gatherMode == 5          # nine taps in a row
    # a 128-column tile of a 300-pixel-wide image spans 3 rows of 302 pixels: too long for the patch
    assert mode(1, 32, 20, 300, 8).gatherMode == 4
    # its pixel range grows with the stride
    assert mode(2, 32, 40, 40, 8, stride=(4, 4)).gatherMode == 4
    assert mode(2, 24, 14, 14, 8).gatherMode in (0, 1)                    # channels not in sixteens
    assert mode(2, 32, 14, 14, 8, 5, 5, (2, 2)).gatherMode in (0, 1)      # not nine taps
    assert mode(2, 32, 14, 14, 8, xs=(32 * 196, 196, 14, 1)).gatherMode in (0, 1)   # NCHW
    assert mode(2, 32, 14, 14, 8, xs=(14 * 14 * 32 + 4, 1, 14 * 32, 32)).gatherMode in (0, 1)  # image pitch not 16-byte


def _fwd_status(x, w, c, y, xp=256, wp=256, yp=256, handle=None, alpha=True, beta=True):
    """Call igcConvolutionForward with fake (never dereferenced) pointers: only legal
    for argument sets that validation rejects before any GPU call."""
    L = ig.lib()
    h = handle or ig.Handle()
    a, b = ctypes.c_float(1), ctypes.c_float(0)
    return L.igcConvolutionForward(h.ptr, ctypes.byref(a) if alpha else None, x.ptr if x else None, xp,
                                   w.ptr if w else None, wp, c.ptr if c else None, None, 0,
                                   ctypes.byref(b) if beta else None, y.ptr if y else None, yp)


def test_forward_rejects_bad_arguments_before_any_gpu_call():
    x, w, c, y = _descs()
    assert _fwd_status(None, w, c, y) == ig.IGC_STATUS_BAD_PARAM
    assert _fwd_status(x, w, c, y, xp=None) == ig.IGC_STATUS_BAD_PARAM
    assert _fwd_status(x, w, c, y, yp=None) == ig.IGC_STATUS_BAD_PARAM
    assert _fwd_status(x, w, c, y, alpha=False) == ig.IGC_STATUS_BAD_PARAM
    assert _fwd_status(x, w, c, y, beta=False) == ig.IGC_STATUS_BAD_PARAM
    assert _fwd_status(x, w, c, y, xp=258 + 1) == ig.IGC_STATUS_BAD_PARAM        # misaligned x
    # unset descriptor
    assert _fwd_status(ig.TensorDescriptor(), w, c, y) == ig.IGC_STATUS_NOT_INITIALIZED
    # channel mismatch
    w2 = ig.FilterDescriptor().set(0, 4, 5, 3, 3)
    assert _fwd_status(x, w2, c, y) == ig.IGC_STATUS_BAD_PARAM
    # wrong y dims
    ybad = ig.TensorDescriptor().set(0, 2, 4, 8, 7, (4 * 8 * 7, 56, 7, 1))
    assert _fwd_status(x, w, c, ybad) == ig.IGC_STATUS_BAD_PARAM
    # aliasing y strides
    yal = ig.TensorDescriptor().set(0, 2, 4, 8, 8, (256, 64, 8, 0))
    assert _fwd_status(x, w, c, yal) == ig.IGC_STATUS_BAD_PARAM
    yal2 = ig.TensorDescriptor().set(0, 2, 4, 8, 8, (256, 60, 8, 1))            # planes overlap
    assert _fwd_status(x, w, c, yal2) == ig.IGC_STATUS_BAD_PARAM
    # data types
    xb = ig.TensorDescriptor().set(1, 2, 3, 8, 8, (192, 64, 8, 1))
    assert _fwd_status(xb, w, c, y) == ig.IGC_STATUS_NOT_SUPPORTED                # bf16 x, f32 w
    yb = ig.TensorDescriptor().set(1, 2, 4, 8, 8, (256, 64, 8, 1))
    assert _fwd_status(x, w, c, yb) == ig.IGC_STATUS_NOT_SUPPORTED                # bf16 y
    # offsets reaching 2^31 bytes
    xbig = ig.TensorDescriptor().set(0, 2, 3, 8, 8, (1 << 29, 64, 8, 1))
    assert _fwd_status(xbig, w, c, y) == ig.IGC_STATUS_NOT_SUPPORTED
    # kernel override of the wrong data type
    h = ig.Handle()
    h.set_kernel_override(len(ig.kernel_names()) - 1)       # a kernel of another data type
    assert _fwd_status(x, w, c, y, handle=h) == ig.IGC_STATUS_NOT_SUPPORTED


def test_backward_passes_validate_before_any_gpu_call():
    """Backward data / backward filter: workspace queries and every rejection path run
    without a GPU (fake device pointers; a rejected call launches nothing)."""
    h = ig.Handle()
    x, w, c, y = _descs(N=2, C=3, H=9, W=8, K=4, R=3, S=3, pad=(1, 1), stride=(2, 1))
    # float, a stride above 1 and few channels (u*v*C <= 128 output maps): room for the filter of the one forward
    # pass that serves all phases (6 maps x K x 2 x 3 taps, rounded up to 256 bytes) and for its result
    # (N x 6 maps x (P + 1) x (Q + 2)); unit strides or many channels: none
    assert ig.get_backward_data_workspace_size(h, w, y, c, x) == 768 + 2 * 6 * 6 * 10 * 4
    x1, w1, c1, y1 = _descs(N=2, C=3, H=9, W=8, K=4, R=3, S=3, pad=(1, 1), stride=(1, 1))
    assert ig.get_backward_data_workspace_size(h, w1, y1, c1, x1) == 0
    # many channels: one launch per phase.  bfloat16 phases run in tap-major order: room for the filter with the
    # reduction index innermost; float phases run in filter order under a mask of the taps outside: none
    x2, w2, c2, y2 = _descs(N=2, C=40, H=9, W=8, K=4, R=3, S=3, pad=(1, 1), stride=(2, 2))
    assert ig.get_backward_data_workspace_size(h, w2, y2, c2, x2) == 0
    _, w2b, _, y2b = _descs(N=2, C=40, H=9, W=8, K=4, R=3, S=3, pad=(1, 1), stride=(2, 2), dt=ig.IGC_DATA_BFLOAT16,
                            ydt=ig.IGC_DATA_BFLOAT16)
    assert ig.get_backward_data_workspace_size(h, w2b, y2b, c2, x2) == 4 * 40 * 9 * 2       # (dx is float)
    # bf16, unit stride, nine taps, K in sixteens, dy with unit channel stride: room for the
    # filter with k and c exchanged; any of these conditions missing: none
    def bd_ws(K=32, stride=(1, 1), dt=ig.IGC_DATA_BFLOAT16, nhwc=True, R=3, S=3, pad=(1, 1)):
        xb, wb, cb, yb = _descs(N=2, C=5, H=9, W=8, K=K, R=R, S=S, pad=pad, stride=stride, dt=dt)
        n, k, p_, q = yb.get()[1]
        yb = ig.TensorDescriptor().set(dt, n, k, p_, q, (p_ * q * k, 1, q * k, k) if nhwc else (k * p_ * q, p_ * q, q, 1))
        dxb = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, *xb.get()[1], xb.get()[2])
        return ig.get_backward_data_workspace_size(h, wb, yb, cb, dxb)
    assert bd_ws() == 32 * 5 * 9 * 2
    assert bd_ws(pad=(0, 2)) == 32 * 5 * 9 * 2
    assert bd_ws(R=1, S=9, pad=(0, 4)) == 32 * 5 * 9 * 2
    # (not that route; the general route asks for nothing, or - launches in tap-major order - for the filter's size again)
    assert bd_ws(K=24) in (0, 24 * 5 * 9 * 2) and bd_ws(stride=(1, 2)) in (0, 32 * 5 * 9 * 2)
    # (float: nothing, or - should the planner run it in tap-major order - the filter's size in floats)
    assert bd_ws(dt=ig.IGC_DATA_FLOAT) in (0, 32 * 5 * 9 * 4)
    assert bd_ws(nhwc=False) in (0, 32 * 5 * 9 * 2) and bd_ws(R=5, S=5, pad=(2, 2)) in (0, 32 * 5 * 25 * 2)
    K, C, R, S = 4, 3, 3, 3
    ws = ig.get_backward_filter_workspace_size(h, x, y, c, w)
    assert ws % (K * C * R * S * 4) == 0
    L = ig.lib()
    one = ctypes.c_float(1.0)
    fake = ctypes.c_void_p(256)

    def bd(wd=w, dyd=y, cd=c, dxd=x, wp=fake, dyp=fake, dxp=fake):
        return L.igcConvolutionBackwardData(h.ptr, ctypes.byref(one), wd.ptr, wp, dyd.ptr, dyp, cd.ptr, None, 0,
                                            ctypes.byref(one), dxd.ptr, dxp)

    def bf(xd=x, dyd=y, cd=c, dwd=w, xp=fake, dyp=fake, dwp=fake, wsp=None):
        return L.igcConvolutionBackwardFilter(h.ptr, ctypes.byref(one), xd.ptr, xp, dyd.ptr, dyp, cd.ptr, wsp, 0,
                                              ctypes.byref(one), dwd.ptr, dwp)

    assert bd(dxp=None) == ig.IGC_STATUS_BAD_PARAM and bf(dwp=None) == ig.IGC_STATUS_BAD_PARAM
    assert bd(dyp=ctypes.c_void_p(258)) == ig.IGC_STATUS_BAD_PARAM          # misaligned float pointer
    assert bf(wsp=ctypes.c_void_p(258)) == ig.IGC_STATUS_BAD_PARAM
    # dy whose size is not eq. 1 of dx's
    _, _, _, ybad = _descs(N=2, C=3, H=9, W=8, K=4, R=3, S=3, pad=(1, 1), stride=(2, 1), ydims=(2, 4, 5, 9))
    assert bd(dyd=ybad) == ig.IGC_STATUS_BAD_PARAM and bf(dyd=ybad) == ig.IGC_STATUS_BAD_PARAM
    # channel counts that do not match the filter
    xbad = ig.TensorDescriptor().set(0, 2, 5, 9, 8, (5 * 72, 72, 8, 1))
    assert bd(dxd=xbad) == ig.IGC_STATUS_BAD_PARAM and bf(xd=xbad) == ig.IGC_STATUS_BAD_PARAM
    # dx with aliasing strides
    xalias = ig.TensorDescriptor().set(0, 2, 3, 9, 8, (0, 72, 8, 1))
    assert bd(dxd=xalias) == ig.IGC_STATUS_BAD_PARAM
    # data types: dx / dw are float; the inputs agree with each other
    xb16 = ig.TensorDescriptor().set(1, 2, 3, 9, 8, (216, 72, 8, 1))
    assert bd(dxd=xb16) == ig.IGC_STATUS_NOT_SUPPORTED
    assert bf(xd=xb16) == ig.IGC_STATUS_NOT_SUPPORTED                       # x bf16 with dy float
    wb16 = ig.FilterDescriptor().set(1, 4, 3, 3, 3)
    assert bf(dwd=wb16) == ig.IGC_STATUS_NOT_SUPPORTED and bd(wd=wb16) == ig.IGC_STATUS_NOT_SUPPORTED
    # descriptors never set
    assert bd(dxd=ig.TensorDescriptor()) == ig.IGC_STATUS_NOT_INITIALIZED
    assert bf(dwd=ig.FilterDescriptor()) == ig.IGC_STATUS_NOT_INITIALIZED
    # backward filter: the window coordinates must fit 14 bits
    xl, wl_, cl, yl = _descs(N=1, C=1, H=16000, W=8, K=1, R=3, S=3, pad=(300, 1))
    assert L.igcConvolutionBackwardFilter(h.ptr, ctypes.byref(one), xl.ptr, fake, yl.ptr, fake, cl.ptr, None, 0,
                                          ctypes.byref(one), wl_.ptr, fake) == ig.IGC_STATUS_NOT_SUPPORTED


def test_other_functions_validate_before_any_gpu_call():
    """Activations, tensor addition, softmax, pooling: descriptor handling and every rejection
    path without a GPU."""
    h = ig.Handle()
    L = ig.lib()
    one = ctypes.c_float(1.0)
    fake = ctypes.c_void_p(256)
    t = lambda n, c, hh, ww, dt=0, st=None: ig.TensorDescriptor().set(dt, n, c, hh, ww, st or (c * hh * ww, hh * ww, ww, 1))
    x, y = t(2, 3, 8, 8), t(2, 3, 8, 8)
    act = lambda xd=x, yd=y, mode=1, xp=fake, yp=fake: L.igcActivationForward(h.ptr, mode, ctypes.byref(one), xd.ptr, xp,
                                                                             ctypes.byref(one), yd.ptr, yp)
    assert act(mode=7) == ig.IGC_STATUS_BAD_PARAM and act(yp=None) == ig.IGC_STATUS_BAD_PARAM
    assert act(yd=t(2, 3, 8, 9)) == ig.IGC_STATUS_BAD_PARAM                     # dimensions differ
    assert act(yd=t(2, 3, 8, 8, st=(0, 64, 8, 1))) == ig.IGC_STATUS_BAD_PARAM   # aliasing output
    assert act(xd=t(2, 3, 8, 8, dt=1)) == ig.IGC_STATUS_NOT_SUPPORTED           # bf16
    assert act(xd=ig.TensorDescriptor()) == ig.IGC_STATUS_NOT_INITIALIZED
    assert act(xp=ctypes.c_void_p(258)) == ig.IGC_STATUS_BAD_PARAM
    add = lambda bd: L.igcAddTensor(h.ptr, ctypes.byref(one), bd.ptr, fake, ctypes.byref(one), y.ptr, fake)
    assert add(t(1, 4, 1, 1)) == ig.IGC_STATUS_BAD_PARAM                        # 4 is neither 1 nor C
    sm = lambda mode: L.igcSoftmaxForward(h.ptr, mode, ctypes.byref(one), x.ptr, fake, ctypes.byref(one), y.ptr, None)
    assert sm(1) == ig.IGC_STATUS_BAD_PARAM
    assert L.igcSoftmaxForward(h.ptr, 5, ctypes.byref(one), x.ptr, fake, ctypes.byref(one), y.ptr, fake) == ig.IGC_STATUS_BAD_PARAM
    # pooling descriptor: round trip, output size, rejections
    pool = ig.PoolingDescriptor().set(ig.IGC_POOLING_AVERAGE, 3, 2, 1, 0, 2, 3)
    assert pool.get() == (ig.IGC_POOLING_AVERAGE, 3, 2, 1, 0, 2, 3)
    assert ig.get_pooling_output_dim(pool, t(2, 3, 9, 11)) == (2, 3, (9 + 2 - 3) // 2 + 1, (11 - 2) // 3 + 1)
    for bad in [(0, 0, 2, 0, 0, 1, 1), (0, 2, 2, 2, 0, 1, 1), (0, 2, 2, 0, 0, 0, 1), (9, 2, 2, 0, 0, 1, 1), (0, 2, 2, -1, 0, 1, 1)]:
        with pytest.raises(ig.IgcError):
            ig.PoolingDescriptor().set(*bad)
    with pytest.raises(ig.IgcError):
        ig.get_pooling_output_dim(ig.PoolingDescriptor().set(0, 5, 5, 0, 0, 1, 1), t(1, 1, 4, 4))    # window larger than the image
    with pytest.raises(ig.IgcError):
        ig.get_pooling_output_dim(ig.PoolingDescriptor(), x)                                         # never set
    xp = t(2, 3, 9, 11)
    pf = lambda yd: L.igcPoolingForward(h.ptr, pool.ptr, ctypes.byref(one), xp.ptr, fake, ctypes.byref(one), yd.ptr, fake)
    assert pf(t(2, 3, 5, 5)) == ig.IGC_STATUS_BAD_PARAM                          # y is not (2,3,5,4)
    tt = lambda xd=x, yd=y, p=fake: L.igcTransformTensor(h.ptr, ctypes.byref(one), xd.ptr, p, ctypes.byref(one), yd.ptr, fake)
    assert tt(yd=t(2, 3, 8, 9)) == ig.IGC_STATUS_BAD_PARAM and tt(p=None) == ig.IGC_STATUS_BAD_PARAM
    assert tt(yd=t(2, 3, 8, 8, st=(0, 64, 8, 1))) == ig.IGC_STATUS_BAD_PARAM and tt(xd=t(2, 3, 8, 8, dt=1)) == ig.IGC_STATUS_NOT_SUPPORTED
    # backward forms: dimensions of every tensor are checked, outputs must not alias
    smb = lambda yd=x, dyd=x, dxd=y, mode=1, p=fake: L.igcSoftmaxBackward(h.ptr, mode, ctypes.byref(one), yd.ptr, fake, dyd.ptr, p,
                                                                          ctypes.byref(one), dxd.ptr, fake)
    assert smb(mode=2) == ig.IGC_STATUS_BAD_PARAM and smb(p=None) == ig.IGC_STATUS_BAD_PARAM
    assert smb(dyd=t(2, 3, 8, 9)) == ig.IGC_STATUS_BAD_PARAM and smb(yd=t(2, 4, 8, 8)) == ig.IGC_STATUS_BAD_PARAM
    assert smb(dxd=t(2, 3, 8, 8, st=(192, 64, 8, 0))) == ig.IGC_STATUS_BAD_PARAM
    assert smb(dyd=t(2, 3, 8, 8, dt=1)) == ig.IGC_STATUS_NOT_SUPPORTED
    pb = lambda dyd=t(2, 3, 5, 4), xd=xp, dxd=t(2, 3, 9, 11), pd=pool: L.igcPoolingBackward(
        h.ptr, pd.ptr, ctypes.byref(one), dyd.ptr, fake, xd.ptr, fake, ctypes.byref(one), dxd.ptr, fake)
    assert pb(dyd=t(2, 3, 5, 5)) == ig.IGC_STATUS_BAD_PARAM and pb(dxd=t(2, 3, 9, 12)) == ig.IGC_STATUS_BAD_PARAM
    assert pb(pd=ig.PoolingDescriptor()) == ig.IGC_STATUS_NOT_INITIALIZED
    assert pb(dxd=t(2, 3, 9, 11, st=(0, 99, 11, 1))) == ig.IGC_STATUS_BAD_PARAM


def test_backward_bias_is_validated_and_planned_before_any_gpu_call():
    """The bias gradient: the workspace it asks for (one double per range and feature map, none for small tensors) and
    every rejection path, without a GPU."""
    h = ig.Handle()
    L = ig.lib()
    one = ctypes.c_float(1.0)
    fake = ctypes.c_void_p(256)
    t = lambda n, c, hh, ww, dt=0, st=None: ig.TensorDescriptor().set(dt, n, c, hh, ww, st or (c * hh * ww, hh * ww, ww, 1))
    dy, db = t(128, 64, 56, 56), t(1, 64, 1, 1)
    big = ig.get_backward_bias_workspace_size(h, dy, db)
    assert big > 0 and big % (64 * 8) == 0 and big <= 1024 * 64 * 8          # whole ranges of 64 doubles, at most 1024 of them
    assert ig.get_backward_bias_workspace_size(h, t(2, 3, 5, 7), t(1, 3, 1, 1)) == 0
    nhwc = t(128, 64, 56, 56, st=(56 * 56 * 64, 1, 56 * 64, 64))
    assert ig.get_backward_bias_workspace_size(h, nhwc, db) > 0
    ig.set_compute_units(h, 64)                                               # fewer compute units, fewer ranges
    assert 0 < ig.get_backward_bias_workspace_size(h, dy, db) < big
    call = lambda dyd=dy, dbd=db, dyp=fake, dbp=fake: L.igcConvolutionBackwardBias(
        h.ptr, ctypes.byref(one), dyd.ptr, dyp, None, 0, ctypes.byref(one), dbd.ptr, dbp)
    assert call(dyp=None) == ig.IGC_STATUS_BAD_PARAM and call(dbp=None) == ig.IGC_STATUS_BAD_PARAM
    assert call(dbd=t(1, 63, 1, 1)) == ig.IGC_STATUS_BAD_PARAM               # feature maps differ
    assert call(dbd=t(2, 64, 1, 1)) == ig.IGC_STATUS_BAD_PARAM               # not (1,C,1,1)
    assert call(dbd=t(1, 64, 1, 1, st=(0, 0, 1, 1))) == ig.IGC_STATUS_BAD_PARAM     # feature maps would share an element
    assert call(dbd=t(1, 64, 1, 1, dt=1)) == ig.IGC_STATUS_NOT_SUPPORTED     # a bfloat16 result
    assert call(dbd=t(1, 64, 1, 1, dt=2)) == ig.IGC_STATUS_NOT_SUPPORTED     # float gradients, double result
    assert call(dyd=ig.TensorDescriptor()) == ig.IGC_STATUS_NOT_INITIALIZED
    assert call(dyp=ctypes.c_void_p(258)) == ig.IGC_STATUS_BAD_PARAM         # misaligned
    with pytest.raises(ig.IgcError):
        ig.get_backward_bias_workspace_size(h, dy, t(1, 65, 1, 1))


def test_setters_reject_bad_values():
    L = ig.lib()
    t = ig.TensorDescriptor()
    assert L.igcSetTensor4dDescriptor(t.ptr, 0, 0, 1, 1, 1, 1, 1, 1, 1) == ig.IGC_STATUS_BAD_PARAM
    assert L.igcSetTensor4dDescriptor(t.ptr, 0, 1, 1, 1, 1, -1, 1, 1, 1) == ig.IGC_STATUS_BAD_PARAM
    assert L.igcSetTensor4dDescriptor(t.ptr, 7, 1, 1, 1, 1, 1, 1, 1, 1) == ig.IGC_STATUS_BAD_PARAM
    assert L.igcSetTensor4dDescriptor(None, 0, 1, 1, 1, 1, 1, 1, 1, 1) == ig.IGC_STATUS_BAD_PARAM
    f = ig.FilterDescriptor()
    assert L.igcSetFilter4dDescriptor(f.ptr, 0, 1, 1, 0, 1) == ig.IGC_STATUS_BAD_PARAM
    c = ig.ConvolutionDescriptor()
    assert L.igcSetConvolution2dDescriptor(c.ptr, -1, 0, 1, 1, 0) == ig.IGC_STATUS_BAD_PARAM
    assert L.igcSetConvolution2dDescriptor(c.ptr, 0, 0, 0, 1, 0) == ig.IGC_STATUS_BAD_PARAM
    assert L.igcSetConvolution2dDescriptor(c.ptr, 0, 0, 1, 1, 2) == ig.IGC_STATUS_BAD_PARAM
    # out-params untouched on failure
    n = ctypes.c_int(-5)
    assert L.igcGetFilter4dDescriptor(f.ptr, ctypes.byref(n), ctypes.byref(n), ctypes.byref(n), ctypes.byref(n),
                                      ctypes.byref(n)) == ig.IGC_STATUS_NOT_INITIALIZED
    assert n.value == -5
    assert L.igcCreate(None) == ig.IGC_STATUS_BAD_PARAM
    assert L.igcDestroy(None) == ig.IGC_STATUS_BAD_PARAM


def test_stream_roundtrip():
    h = ig.Handle()
    assert h.get_stream() == 0
    h.set_stream(0x1234)
    assert h.get_stream() == 0x1234


def test_magic_division_exhaustive_small_and_sampled_large():
    """Division by launch-time constants as multiply + shift (Section 3.1): brute force
    against integer division for the divisors the workloads produce and for edge cases."""
    divisors = {1, 2, 3, 5, 7, 9, 11, 13, 14, 55, 56, 121, 169, 196, 3025, 3136, 1 << 10, (1 << 10) + 1,
                (1 << 16) - 1, 1 << 16, (1 << 20) + 7, (1 << 30) - 1, 1 << 30, (1 << 31) - 1}
    rng = np.random.default_rng(3)
    divisors |= {int(v) for v in rng.integers(1, 1 << 31, size=40)}
    edge = np.array([0, 1, 2, (1 << 31) - 1, (1 << 31) - 2, 1 << 30], dtype=np.uint64)
    for d in sorted(divisors):
        mul, shift = ig.magic_divisor(d)
        n = np.concatenate([np.arange(0, 70000, dtype=np.uint64),
                            rng.integers(0, 1 << 31, size=20000).astype(np.uint64), edge,
                            np.arange(1, 300, dtype=np.uint64) * np.uint64(d) % np.uint64(1 << 31),
                            (np.arange(1, 300, dtype=np.uint64) * np.uint64(d) - np.uint64(1)) % np.uint64(1 << 31)])
        q = (((n * np.uint64(mul)) >> np.uint64(32)) + n) >> np.uint64(shift)
        assert np.array_equal(q, n // np.uint64(d)), d
        # the library's own evaluator agrees with the formula
        for v in (0, 1, d - 1, d, d + 1, (1 << 31) - 1):
            assert ig.magic_divide(v, mul, shift) == v // d
    with pytest.raises(ig.IgcError):
        ig.magic_divisor(0)
    with pytest.raises(ig.IgcError):
        ig.magic_divisor(1 << 31)


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    import paper_1410_0759_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        b.lib()


def test_double_precision_is_planned_and_mixed_types_are_rejected():
    h = ig.Handle()
    D, F = ig.IGC_DATA_DOUBLE, ig.IGC_DATA_FLOAT
    x, w, c, y = _descs(N=2, C=5, H=9, W=8, K=70, dt=D, ydt=D)
    plan = ig.get_plan(h, x, w, c, y)
    # (nine taps: filter order under a tap mask, the pipelined kernels; persistent workgroups, here one per tile)
    assert plan.tileM in (64, 128) and (plan.tileN, plan.tileK, plan.gatherMode) == (64, 16, 14)
    assert ig.kernel_names()[plan.kernelId].startswith("f64")
    tiles = ((70 + plan.tileM - 1) // plan.tileM) * ((2 * 9 * 8 + plan.tileN - 1) // plan.tileN)
    assert plan.gridX >= tiles and plan.gridX % 8 == 0
    # more than 63 taps: the generic gather, one workgroup per tile
    x8, w8, c8, y8 = _descs(N=2, C=5, H=9, W=8, K=70, R=8, S=8, pad=(4, 4), dt=D, ydt=D)
    plan = ig.get_plan(h, x8, w8, c8, y8)
    assert (plan.tileM, plan.tileN, plan.tileK, plan.gatherMode) == (64, 64, 16, 0)
    tiles = ((70 + 63) // 64) * ((2 * 10 * 9 + 63) // 64)
    assert plan.gridX >= tiles and plan.gridX % 8 == 0
    assert ig.get_workspace_size(h, x, w, c, y) == 0 and ig.get_optional_workspace_size(h, x, w, c, y) == 0
    assert _fwd_status(x, w, c, _descs(N=2, C=5, H=9, W=8, K=70, dt=D, ydt=F)[3]) == ig.IGC_STATUS_NOT_SUPPORTED
    xf = _descs(N=2, C=5, H=9, W=8, K=70)[0]
    assert _fwd_status(xf, w, c, y) == ig.IGC_STATUS_NOT_SUPPORTED
    # backward passes: the output's type follows the inputs'
    assert ig.get_backward_data_workspace_size(h, w, y, c, x) == 0
    assert ig.get_backward_filter_workspace_size(h, x, y, c, w) % (70 * 5 * 9 * 8) == 0
    with pytest.raises(ig.IgcError):
        ig.get_backward_data_workspace_size(h, w, y, c, xf)
    wf = ig.FilterDescriptor().set(F, 70, 5, 3, 3)
    with pytest.raises(ig.IgcError):
        ig.get_backward_filter_workspace_size(h, x, y, c, wf)


def test_backward_filter_workspace_fits_the_no_alloc_scratch_array():
    """igcConvolutionBackwardFilterNoAlloc serves a problem when the workspace its ordinary form asks for fits the
    library's scratch array.  The ranges of a cut reduction are chosen so that all (tile, range) workgroups are
    resident at once - at most 512 tiles of at most 64 KB; in double precision at most 2048 workgroups of 32 KB -, so the
    sizes stay within the array; checked here over
    layer shapes small and large, all three data types."""
    h = ig.Handle()
    worst = 0
    for dt in (ig.IGC_DATA_FLOAT, ig.IGC_DATA_BFLOAT16, ig.IGC_DATA_DOUBLE):
        for (N, C, H, W, K, R, pad, u) in [(64, 3, 227, 227, 96, 11, 0, 4), (128, 64, 56, 56, 64, 3, 1, 1), (128, 384, 13, 13, 256, 3, 1, 1),
                                           (32, 512, 14, 14, 512, 3, 1, 1), (256, 512, 14, 14, 512, 3, 1, 1), (64, 128, 48, 48, 128, 1, 0, 1),
                                           (64, 256, 28, 28, 512, 3, 1, 1), (128, 96, 27, 27, 256, 5, 2, 1), (1, 1, 5, 5, 1, 3, 0, 1),
                                           (512, 130, 30, 30, 130, 3, 1, 1), (128, 1024, 7, 7, 1024, 1, 0, 1)]:
            x = ig.TensorDescriptor().set(dt, N, C, H, W, (C * H * W, 1, W * C, C) if dt == ig.IGC_DATA_BFLOAT16 else (C * H * W, H * W, W, 1))
            P = (H + 2 * pad - R) // u + 1
            dy = ig.TensorDescriptor().set(dt, N, K, P, P, (K * P * P, 1, P * K, K) if dt == ig.IGC_DATA_BFLOAT16 else (K * P * P, P * P, P, 1))
            dw = ig.FilterDescriptor().set(ig.IGC_DATA_DOUBLE if dt == ig.IGC_DATA_DOUBLE else ig.IGC_DATA_FLOAT, K, C, R, R)
            conv = ig.ConvolutionDescriptor().set(pad, pad, u, u, 1)
            worst = max(worst, ig.get_backward_filter_workspace_size(h, x, dy, conv, dw))
    assert 0 < worst <= ig.NOALLOC_SCRATCH_BYTES, worst


def _random_layer(rng):
    """A random layer the library accepts: small sizes, every kind of stride, border and layout."""
    N, C, K = int(rng.integers(1, 5)), int(rng.integers(1, 40)), int(rng.integers(1, 140))
    R, S = int(rng.integers(1, 8)), int(rng.integers(1, 8))
    pad = (int(rng.integers(0, R)), int(rng.integers(0, S)))
    stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    H = int(rng.integers(max(1, R - 2 * pad[0]), 30))
    W = int(rng.integers(max(1, S - 2 * pad[1]), 30))
    return N, C, H, W, K, R, S, pad, stride


def test_address_reach_stays_inside_the_buffer_extents():
    """For every accepted problem the largest offset the kernels' address arithmetic forms for an existing element
    - evaluated by the library in 64 bits from the launch parameters of the kernel it would run - lies inside the
    extent its buffer descriptor is given, and below 2^31: forward and backward data (all stride phases), the three
    data types, both layouts, the workloads at full size."""
    h = ig.Handle()
    rng = np.random.default_rng(14100759)
    dts = (ig.IGC_DATA_FLOAT, ig.IGC_DATA_BFLOAT16, ig.IGC_DATA_DOUBLE)
    cases = [_random_layer(rng) for _ in range(400)]
    cases += [(w_.N, w_.C, w_.H, w_.W, w_.K, w_.R, w_.S, (w_.pad_h, w_.pad_w), (w_.u, w_.v)) for w_ in wl.WORKLOADS]
    seen_modes = set()
    for i, (N, C, H, W, K, R, S, pad, stride) in enumerate(cases):
        dt = dts[i % 3]
        ydt = ig.IGC_DATA_DOUBLE if dt == ig.IGC_DATA_DOUBLE else ig.IGC_DATA_FLOAT
        nhwc = (i // 3) % 2 == 1
        xs = (H * W * C, 1, W * C, C) if nhwc else None
        x, w, c, y = _descs(N, C, H, W, K, R, S, pad, stride, i % 2, dt, xs=xs, ydt=ydt)
        n, k, p, q = y.get()[1]
        if nhwc:
            y = ig.TensorDescriptor().set(ydt, n, k, p, q, (p * q * k, 1, q * k, k))
        seen_modes.add(ig.get_plan(h, x, w, c, y).gatherMode)
        reach, extent = ig.get_forward_address_reach(h, x, w, c, y)
        es = {ig.IGC_DATA_FLOAT: 4, ig.IGC_DATA_BFLOAT16: 2, ig.IGC_DATA_DOUBLE: 8}[dt]
        assert extent[1] == K * C * R * S * es and reach[1] == extent[1]          # the packed filter is read to its end
        assert reach[2] == extent[2] == n * k * p * q * (8 if ydt == ig.IGC_DATA_DOUBLE else 4)
        assert 0 < reach[0] <= extent[0] == N * C * H * W * es
        assert all(e < 2 ** 31 for e in extent)
        # backward data: dy and dx exchange the roles; dx has the input's type rule (float for bfloat16 inputs)
        dyd = ig.TensorDescriptor().set(dt, n, k, p, q, (p * q * k, 1, q * k, k) if nhwc else (k * p * q, p * q, q, 1))
        dxd = ig.TensorDescriptor().set(ydt, N, C, H, W, xs or (C * H * W, H * W, W, 1))
        reach, extent = ig.get_backward_data_address_reach(h, w, dyd, c, dxd)
        assert 0 < reach[0] <= extent[0] and 0 < reach[1] <= extent[1] and 0 < reach[2] <= extent[2], (cases[i], reach, extent)
        # every element of dx belongs to some phase: the last one is reached
        assert reach[2] == extent[2]
    assert {0, 3, 14} <= seen_modes    # (generic, nine-tap table and masked plans were among them)


def test_plans_follow_the_compute_unit_count_of_the_handle():
    """The handle carries the device's compute-unit count (256 without a device); persistent grids and the choice
    between tile shapes follow it."""
    h = ig.Handle()
    assert ig.get_compute_units(h) == 256      # no GPU here: MI355X's count stands in
    w_ = wl.by_index(3)
    d = _descs(w_.N, w_.C, w_.H, w_.W, w_.K, w_.R, w_.S, (w_.pad_h, w_.pad_w), (w_.u, w_.v), w_.mode, 0)
    p256 = ig.get_plan(h, *d)
    ig.set_compute_units(h, 304)
    assert ig.get_compute_units(h) == 304
    p304 = ig.get_plan(h, *d)
    ig.set_compute_units(h, 64)
    p64 = ig.get_plan(h, *d)
    # cfg 3 has thousands of tiles: the persistent grid is the number of workgroups the chip holds at once
    per_cu = p256.gridX // 256
    assert per_cu in (1, 2, 3, 4) and p256.gridX == 256 * per_cu
    assert p304.gridX == 304 * (p304.gridX // 304) and p64.gridX == 64 * (p64.gridX // 64)
    for bad in (0, 7, 5000):
        with pytest.raises(ig.IgcError):
            ig.set_compute_units(h, bad)
