"""GPU parity of the double-precision path (forward, backward data, backward filter) against
the CPU oracle.  The oracle takes float32-valued inputs and works in double; a double input
is built as hi + 2^-30 * lo with hi, lo float32-valued, and because all three passes are
bilinear in their two inputs the expected result is the oracle's own results combined:
f(a, b) = f(a_hi, b_hi) + e (f(a_lo, b_hi) + f(a_hi, b_lo)) + e^2 f(a_lo, b_lo), e = 2^-30.
A path that rounded its inputs or its sums to float would miss by 1e-9 .. 1e-7; the bar is
max|gpu - oracle| / max|oracle| <= 1e-12."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import workloads as wl
from oracle import conv_oracle as oc

E = 2.0 ** -30


def _gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def _pair(seed, shape, layout="NCHW"):
    rng = np.random.default_rng(seed)
    hi = wl.with_layout(rng.uniform(-1, 1, size=shape).astype(np.float32), layout)
    lo = wl.with_layout(rng.uniform(-1, 1, size=shape).astype(np.float32), layout)
    full = wl.with_layout(np.empty(shape, dtype=np.float64), layout)
    full[...] = hi.astype(np.float64) + E * lo.astype(np.float64)
    return hi, lo, full


def _bilinear(f, a, b):
    return f(a[0], b[0]) + E * (f(a[1], b[0]) + f(a[0], b[1])) + E * E * f(a[1], b[1])


# N, C, H, W, K, R, S, pad, stride
PROBLEMS = [
    (2, 5, 9, 11, 7, 3, 3, (1, 1), (1, 1)),
    (3, 40, 14, 13, 150, 3, 3, (1, 1), (1, 1)),       # several tiles, ragged in every direction
    (2, 3, 23, 21, 70, 5, 5, (2, 2), (2, 2)),         # four stride phases in backward data
    (1, 6, 30, 17, 20, 7, 1, (3, 0), (3, 1)),
    (2, 4, 12, 12, 9, 1, 1, (0, 0), (2, 2)),          # phases that meet no tap
    (1, 3, 35, 35, 96, 11, 11, (0, 0), (4, 4)),       # first-layer shape
    (2, 2, 8, 8, 4, 4, 4, (3, 3), (1, 1)),            # "full" padding
    (1, 1, 1, 1, 1, 1, 1, (0, 0), (1, 1)),
]
IDS = [str(i) for i in range(len(PROBLEMS))]


def _close(got, want):
    gu = _gpu()
    assert got.shape == want.shape and np.all(np.isfinite(got))
    err = gu.rel_err(got, want)
    assert err <= gu.BOUND["f64"], "rel err %.3g" % err


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
@pytest.mark.parametrize("prob", PROBLEMS, ids=IDS)
def test_forward_f64(prob, mode):
    gu = _gpu()
    N, C, H, W, K, R, S, pad, stride = prob
    for layout in ("NCHW", "NHWC"):
        x, w = _pair(1, (N, C, H, W), layout), _pair(2, (K, C, R, S))
        print("f64 forward", prob, mode, layout, flush=True)
        want = _bilinear(lambda a, b: oc.conv_forward(a, b, pad=pad, stride=stride, mode=mode), x, w)
        got, plan = gu.run(x[2], w[2], pad, stride, mode, dtype="f64", y_layout=layout)
        _close(got, want)
        assert plan.tileM == plan.tileN and plan.tileM in (64, 128) and plan.tileK == 16
    y0 = np.random.default_rng(3).uniform(-1, 1, size=want.shape)
    got, _ = gu.run(x[2], w[2], pad, stride, mode, alpha=0.5, beta=-1.5, y0=y0, dtype="f64", y_layout="NHWC")
    _close(got, 0.5 * want - 1.5 * y0)


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
@pytest.mark.parametrize("prob", PROBLEMS, ids=IDS)
def test_backward_data_f64(prob, mode):
    gu = _gpu()
    N, C, H, W, K, R, S, pad, stride = prob
    P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
    for layout in ("NCHW", "NHWC"):
        dy, w = _pair(4, (N, K, P, Q), layout), _pair(5, (K, C, R, S))
        print("f64 backward data", prob, mode, layout, flush=True)
        want = _bilinear(lambda a, b: oc.conv_backward_data(a, b, (H, W), pad=pad, stride=stride, mode=mode), dy, w)
        _close(gu.run_backward_data(dy[2], w[2], (H, W), pad, stride, mode, dtype="f64", dx_layout=layout), want)
    old = np.random.default_rng(6).uniform(-1, 1, size=want.shape)
    got = gu.run_backward_data(dy[2], w[2], (H, W), pad, stride, mode, 2.0, 0.75, old, "f64", "NCHW")
    _close(got, 2.0 * want + 0.75 * old)


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
@pytest.mark.parametrize("prob", PROBLEMS, ids=IDS)
def test_backward_filter_f64(prob, mode):
    gu = _gpu()
    N, C, H, W, K, R, S, pad, stride = prob
    P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
    for layout in ("NCHW", "NHWC"):
        x, dy = _pair(7, (N, C, H, W), layout), _pair(8, (N, K, P, Q), layout)
        print("f64 backward filter", prob, mode, layout, flush=True)
        want = _bilinear(lambda a, b: oc.conv_backward_filter(a, b, (R, S), pad=pad, stride=stride, mode=mode), x, dy)
        for workspace in ("full", "none"):
            got, asked = gu.run_backward_filter(x[2], dy[2], (R, S), pad, stride, mode, dtype="f64", workspace=workspace)
            assert asked % (K * C * R * S * 8) == 0
            _close(got, want)
    old = np.random.default_rng(9).uniform(-1, 1, size=want.shape)
    got, _ = gu.run_backward_filter(x[2], dy[2], (R, S), pad, stride, mode, -0.5, 2.0, old, "f64")
    _close(got, -0.5 * want + 2.0 * old)


def test_f64_at_a_layer_size():
    """The mid-layer workload's shape on 4 images (several hundred tiles, reduction 576): all
    three passes, and the transpose identities between them with every side from the library."""
    gu = _gpu()
    N, C, H, W, K, R, S, pad, stride = 4, 64, 56, 56, 64, 3, 3, (1, 1), (1, 1)
    x, w, dy = _pair(10, (N, C, H, W)), _pair(11, (K, C, R, S)), _pair(12, (N, K, H, W))
    y, _ = gu.run(x[2], w[2], pad, stride, 1, dtype="f64")
    _close(y, _bilinear(lambda a, b: oc.conv_forward(a, b, pad=pad, stride=stride, mode=1), x, w))
    dx = gu.run_backward_data(dy[2], w[2], (H, W), pad, stride, 1, dtype="f64")
    dw, asked = gu.run_backward_filter(x[2], dy[2], (R, S), pad, stride, 1, dtype="f64")
    assert asked > 0
    lhs = float(np.sum(y * dy[2]))
    scale = float(np.sqrt(np.sum(y * y) * np.sum(dy[2] ** 2)))
    assert abs(lhs - float(np.sum(dx * x[2]))) <= 1e-12 * scale
    assert abs(lhs - float(np.sum(dw * w[2]))) <= 1e-12 * scale


@pytest.mark.parametrize("name", ["f64 64x64x16 generic"])
def test_forward_f64_with_each_tile(name):
    gu = _gpu()
    import paper_1410_0759_amd as ig
    N, C, H, W, K, R, S, pad, stride = 3, 40, 14, 13, 150, 3, 3, (1, 1), (2, 1)
    x, w = _pair(21, (N, C, H, W)), _pair(22, (K, C, R, S))
    want = _bilinear(lambda a, b: oc.conv_forward(a, b, pad=pad, stride=stride, mode=0), x, w)
    got, plan = gu.run(x[2], w[2], pad, stride, 0, dtype="f64", kernel=ig.kernel_names().index(name))
    assert ig.kernel_names()[plan.kernelId] == name
    _close(got, want)


def test_f64_rejections():
    gu = _gpu()
    import paper_1410_0759_amd as ig
    x, w = _pair(1, (1, 2, 5, 5)), _pair(2, (3, 2, 3, 3))
    g = gu.GpuConv(x[2], w[2], (0, 0), (1, 1), 1, dtype="f64")
    with pytest.raises(ig.IgcError):      # the fused epilogue exists in single precision only
        g.launch_fused(1.0, 0.0, np.zeros(3, np.float32), ig.IGC_ACTIVATION_RELU)
