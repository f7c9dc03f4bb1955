"""GPU parity of the double-precision forms of the library's other functions (activations,
tensor addition and transformation, softmax, pooling; forward and backward) against the CPU
oracle on full-precision double inputs.  Bar: max|gpu - oracle| / max|oracle| <= 1e-13 (a path
that rounded an input or a result to float would miss by ~1e-8)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import workloads as wl
from oracle import pointwise_oracle as po

TOL = 1e-13
SHAPES = [(2, 3, 5, 7), (1, 1, 1, 1), (3, 16, 12, 12), (2, 5, 9, 64), (4, 130, 3, 3), (1, 2, 1, 1000)]


def _gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def rnd(seed, *shape, lo=-3.0, hi=3.0):
    return np.random.default_rng(seed).uniform(lo, hi, size=shape)       # float64, all 53 bits in use


def close(got, want, tol=TOL):
    gu = _gpu()
    assert got.shape == want.shape and np.all(np.isfinite(got))
    err = gu.rel_err(got, want)
    assert err <= tol, err


@pytest.mark.parametrize("mode", [0, 1, 2], ids=["sigmoid", "relu", "tanh"])
def test_activations_f64(mode):
    gu = _gpu()
    for shape in SHAPES:
        x, dy, old = rnd(1, *shape), rnd(2, *shape), rnd(3, *shape)
        print("f64 activation", mode, shape, flush=True)
        close(gu.run_activation_forward(mode, x), po.activation_forward(mode, x))
        close(gu.run_activation_forward(mode, wl.with_layout(x, "NHWC"), 0.5, -1.5, old, "NCHW"), po.activation_forward(mode, x, 0.5, -1.5, old))
        y = po.activation_forward(mode, x)
        close(gu.run_activation_backward(mode, y, dy, x), po.activation_backward(mode, y, dy, x))
        close(gu.run_activation_backward(mode, wl.with_layout(y, "NHWC"), dy, wl.with_layout(x, "NHWC"), 2.0, 0.5, old, "NHWC"),
              po.activation_backward(mode, y, dy, x, 2.0, 0.5, old))
    x = np.array([-700.0, -30.0, -1e-9, 0.0, 1e-9, 30.0, 700.0, 20.0]).reshape(1, 2, 2, 2)
    close(gu.run_activation_forward(mode, x), po.activation_forward(mode, x))


def test_add_and_transform_f64():
    gu = _gpu()
    for shape in SHAPES + [(3, 70, 9, 11), (2, 64, 56, 56)]:
        N, C, H, W = shape
        x, old = rnd(4, *shape), rnd(5, *shape)
        for bshape in [(1, C, 1, 1), shape, (N, 1, 1, W)]:
            b = rnd(6, *bshape)
            close(gu.run_add_tensor(b, shape, 2.0, 1.0, old, "NHWC"), po.add_tensor(b, shape, 2.0, 1.0, old))
        for src in ("NCHW", "NHWC"):
            for dst in ("NCHW", "NHWC"):
                assert np.array_equal(gu.run_transform_tensor(wl.with_layout(x, src), layout=dst), x)      # a copy is exact
        close(gu.run_transform_tensor(wl.with_layout(x, "NHWC"), -0.5, 2.0, old, "NCHW"), po.add_tensor(x, shape, -0.5, 2.0, old))


@pytest.mark.parametrize("mode", [0, 1], ids=["instance", "channel"])
def test_softmax_f64(mode):
    gu = _gpu()
    for shape in SHAPES + [(64, 1000, 1, 1), (2, 21, 33, 17)]:
        x, dy, old = rnd(7, *shape, lo=-10, hi=10), rnd(8, *shape), rnd(9, *shape)
        print("f64 softmax", mode, shape, flush=True)
        y = po.softmax_forward(mode, x)
        close(gu.run_softmax_forward(mode, x), y)
        close(gu.run_softmax_forward(mode, wl.with_layout(x, "NHWC"), 0.5, 2.0, old, "NHWC"), po.softmax_forward(mode, x, 0.5, 2.0, old))
        close(gu.run_softmax_backward(mode, y, dy), po.softmax_backward(mode, y, dy))
        close(gu.run_softmax_backward(mode, wl.with_layout(y, "NHWC"), dy, 0.5, 2.0, old, "NHWC"), po.softmax_backward(mode, y, dy, 0.5, 2.0, old))
    x = rnd(10, 2, 7, 3, 3) + 3000.0
    close(gu.run_softmax_forward(mode, x), po.softmax_forward(mode, x))


@pytest.mark.parametrize("mode", [0, 1], ids=["max", "average"])
def test_pooling_f64(mode):
    gu = _gpu()
    cases = [((2, 3, 9, 11), (2, 2), (0, 0), (2, 2)), ((2, 3, 9, 11), (3, 3), (1, 1), (2, 2)), ((1, 5, 13, 13), (3, 2), (1, 0), (1, 3)),
             ((3, 5, 55, 55), (3, 3), (0, 0), (2, 2)), ((2, 4, 8, 8), (5, 5), (2, 2), (4, 4)), ((1, 1, 1, 1), (1, 1), (0, 0), (1, 1)),
             ((2, 2, 130, 40), (2, 2), (1, 1), (2, 2)), ((1, 2, 9, 700), (3, 3), (1, 1), (1, 1)), ((1, 1, 4, 3000), (3, 3), (1, 1), (1, 1))]
    for shape, win, pad, st in cases:
        x = rnd(11, *shape) - 5.0
        P, Q = po.pooling_output_dim(shape[2], win[0], pad[0], st[0]), po.pooling_output_dim(shape[3], win[1], pad[1], st[1])
        dy, old = rnd(12, shape[0], shape[1], P, Q), rnd(13, *shape)
        print("f64 pooling", mode, shape, win, pad, st, flush=True)
        want = po.pooling_forward(mode, x, win, pad, st)
        close(gu.run_pooling_forward(mode, x, win, pad, st), want)
        close(gu.run_pooling_forward(mode, wl.with_layout(x, "NHWC"), win, pad, st, layout="NHWC"), want)
        wantb = po.pooling_backward(mode, x, dy, win, pad, st)
        close(gu.run_pooling_backward(mode, x, dy, win, pad, st), wantb)
        close(gu.run_pooling_backward(mode, wl.with_layout(x, "NHWC"), wl.with_layout(dy, "NHWC"), win, pad, st, layout="NHWC"), wantb)
        close(gu.run_pooling_backward(mode, x, dy, win, pad, st, 0.5, -1.0, old), po.pooling_backward(mode, x, dy, win, pad, st, 0.5, -1.0, old))


def test_mixed_types_are_rejected():
    gu = _gpu()
    import paper_1410_0759_amd as ig
    import torch
    x = torch.zeros(2 * 3 * 4 * 5, dtype=torch.float64, device="cuda")
    d64 = ig.TensorDescriptor().set(ig.IGC_DATA_DOUBLE, 2, 3, 4, 5, (60, 20, 5, 1))
    d32 = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, 2, 3, 4, 5, (60, 20, 5, 1))
    h = ig.Handle()
    assert ig.activation_forward(h, 1, 1.0, d32, x.data_ptr(), 0.0, d64, x.data_ptr()) == ig.IGC_STATUS_NOT_SUPPORTED
    assert ig.activation_forward(h, 1, 1.0, d64, x.data_ptr(), 0.0, d32, x.data_ptr()) == ig.IGC_STATUS_NOT_SUPPORTED
    assert ig.transform_tensor(h, 1.0, d64, x.data_ptr(), 0.0, d32, x.data_ptr()) == ig.IGC_STATUS_NOT_SUPPORTED


def test_backward_bias_in_double_precision():
    """The bias gradient with double tensors: double sums, double result, double alpha and beta."""
    gu = _gpu()
    for i, shape in enumerate([(2, 3, 5, 7), (5, 70, 9, 11), (8, 64, 28, 28), (3, 130, 17, 5)]):
        dy = np.random.default_rng(500 + i).uniform(-1, 1, size=shape)
        old = np.random.default_rng(520 + i).uniform(-1, 1, size=shape[1])
        for layout in ("NCHW", "NHWC"):
            dyl = wl.with_layout(dy, layout)
            want = po.bias_backward(dy)
            for ws in ("full", "none"):
                got = gu.run_backward_bias(dyl, workspace=ws)
                assert gu.rel_err(got, want) <= gu.BOUND["f64"]
            got = gu.run_backward_bias(dyl, -0.5, 2.0, old, db_stride=2)
            assert gu.rel_err(got, po.bias_backward(dy, -0.5, 2.0, old)) <= gu.BOUND["f64"]
    # values a float could not hold
    d = np.ones((1, 2, 1, 2)); d[0, 1, 0, 1] = 2.0 ** -40
    assert gu.run_backward_bias(d)[1] == 1.0 + 2.0 ** -40
