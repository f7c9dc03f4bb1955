"""GPU parity of the library's other functions (activations, tensor addition, softmax,
pooling) against the CPU oracle, element by element.  Bar: max|gpu - oracle| / max|oracle|
<= 2e-5 (fp32), the same as for the convolutions."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import workloads as wl
from oracle import pointwise_oracle as po

TOL = 2e-5


def _gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def rnd(seed, *shape, lo=-4.0, hi=4.0):
    return np.random.default_rng(seed).uniform(lo, hi, size=shape).astype(np.float32)


def close(got, want):
    gu = _gpu()
    assert got.shape == want.shape and np.all(np.isfinite(got))
    err = gu.rel_err(got, want)
    assert err <= TOL, err


SHAPES = [(2, 3, 5, 7), (1, 1, 1, 1), (3, 16, 12, 12), (2, 5, 9, 64), (4, 130, 3, 3), (1, 2, 1, 1000)]


@pytest.mark.parametrize("mode", [0, 1, 2], ids=["sigmoid", "relu", "tanh"])
@pytest.mark.parametrize("shape", SHAPES, ids=[str(i) for i in range(len(SHAPES))])
def test_activation_forward(shape, mode):
    gu = _gpu()
    x = rnd(1, *shape)
    close(gu.run_activation_forward(mode, x), po.activation_forward(mode, x))
    old = rnd(2, *shape)
    close(gu.run_activation_forward(mode, wl.with_layout(x, "NHWC"), 0.5, -1.5, old, "NHWC"),
          po.activation_forward(mode, x, 0.5, -1.5, old))
    # input and output in different layouts; a pitched (sliced) input
    close(gu.run_activation_forward(mode, wl.with_layout(x, "NHWC"), layout="NCHW"), po.activation_forward(mode, x))
    wide = rnd(3, shape[0], shape[1], shape[2], shape[3] + 3)
    close(gu.run_activation_forward(mode, wide[..., 1:-2]), po.activation_forward(mode, np.ascontiguousarray(wide[..., 1:-2])))


def test_activation_extremes_and_in_place():
    gu = _gpu()
    import torch
    import paper_1410_0759_amd as ig
    x = np.array([-200.0, -30.0, -1e-3, 0.0, 1e-3, 30.0, 200.0, 88.0], dtype=np.float32).reshape(1, 2, 2, 2)
    for mode in (0, 1, 2):
        close(gu.run_activation_forward(mode, x), po.activation_forward(mode, x))
    # in place: x and y are the same buffer with the same descriptor
    x = rnd(4, 2, 8, 6, 10)
    t = torch.from_numpy(x).cuda()
    d = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, *x.shape, (480, 60, 10, 1))
    h = ig.Handle()
    ig.check(ig.activation_forward(h, ig.IGC_ACTIVATION_TANH, 1.0, d, t.data_ptr(), 0.0, d, t.data_ptr()), "in place")
    torch.cuda.synchronize()
    close(t.cpu().numpy().astype(np.float64), po.activation_forward(po.TANH, x))


@pytest.mark.parametrize("mode", [0, 1, 2], ids=["sigmoid", "relu", "tanh"])
def test_activation_backward(mode):
    gu = _gpu()
    for shape in SHAPES:
        x, dy = rnd(5, *shape), rnd(6, *shape)
        y = po.activation_forward(mode, x).astype(np.float32)
        close(gu.run_activation_backward(mode, y, dy, x), po.activation_backward(mode, y, dy, x))
        old = rnd(7, *shape)
        close(gu.run_activation_backward(mode, wl.with_layout(y, "NHWC"), dy, wl.with_layout(x, "NHWC"), 2.0, 0.5, old, "NHWC"),
              po.activation_backward(mode, y, dy, x, 2.0, 0.5, old))


def test_add_tensor_broadcasting():
    gu = _gpu()
    for shape in SHAPES:
        N, C, H, W = shape
        old = rnd(8, *shape)
        for bshape in [(1, C, 1, 1), shape, (N, 1, 1, W), (1, 1, 1, 1), (1, C, H, 1)]:
            b = rnd(9, *bshape)
            for layout in ("NCHW", "NHWC"):
                close(gu.run_add_tensor(b, shape, 2.0, 1.0, old, layout), po.add_tensor(b, shape, 2.0, 1.0, old))
        close(gu.run_add_tensor(rnd(10, 1, C, 1, 1), shape), po.add_tensor(rnd(10, 1, C, 1, 1), shape))


@pytest.mark.parametrize("mode", [0, 1], ids=["instance", "channel"])
def test_softmax_forward(mode):
    gu = _gpu()
    for shape in SHAPES + [(64, 1000, 1, 1), (2, 21, 33, 17)]:
        x = rnd(11, *shape, lo=-10, hi=10)
        want = po.softmax_forward(mode, x)
        close(gu.run_softmax_forward(mode, x), want)
        close(gu.run_softmax_forward(mode, wl.with_layout(x, "NHWC"), layout="NHWC"), want)
        old = rnd(12, *shape)
        close(gu.run_softmax_forward(mode, x, 0.5, 2.0, old, "NHWC"), po.softmax_forward(mode, x, 0.5, 2.0, old))
    # stability: huge values, a dominant element
    x = (rnd(13, 2, 7, 3, 3) + np.float32(3000.0)).astype(np.float32)
    close(gu.run_softmax_forward(mode, x), po.softmax_forward(mode, x))
    x = rnd(14, 2, 7, 3, 3)
    x[:, 2] += 500.0
    close(gu.run_softmax_forward(mode, x), po.softmax_forward(mode, x))


@pytest.mark.parametrize("mode", [0, 1], ids=["max", "average"])
def test_pooling_forward(mode):
    gu = _gpu()
    cases = [((2, 3, 9, 11), (2, 2), (0, 0), (2, 2)), ((2, 3, 9, 11), (3, 3), (1, 1), (2, 2)),
             ((1, 5, 13, 13), (3, 2), (1, 0), (1, 3)), ((3, 96, 27, 27), (3, 3), (0, 0), (2, 2)),
             ((2, 4, 7, 7), (7, 7), (0, 0), (1, 1)), ((2, 4, 8, 8), (5, 5), (2, 2), (4, 4)), ((1, 1, 1, 1), (1, 1), (0, 0), (1, 1)),
             ((3, 5, 55, 55), (3, 3), (0, 0), (2, 2)), ((2, 3, 37, 20), (3, 3), (1, 1), (1, 1)), ((2, 3, 11, 9), (2, 2), (0, 0), (3, 3)),
             ((2, 2, 130, 40), (2, 2), (1, 1), (2, 2)),      # more output rows than one workgroup takes
             ((1, 2, 9, 700), (3, 3), (1, 1), (1, 1)),       # wide rows: fewer rows per workgroup
             ((1, 1, 4, 6000), (3, 3), (1, 1), (1, 1))]      # too wide for the row-strip kernel
    for shape, win, pad, st in cases:
        print("pooling forward", mode, shape, win, pad, st, flush=True)
        x = rnd(15, *shape) - np.float32(5.0)     # all negative: a zero border must never win the maximum
        want = po.pooling_forward(mode, x, win, pad, st)
        close(gu.run_pooling_forward(mode, x, win, pad, st), want)
        close(gu.run_pooling_forward(mode, wl.with_layout(x, "NHWC"), win, pad, st, layout="NHWC"), want)
        old = rnd(16, *want.shape)
        close(gu.run_pooling_forward(mode, x, win, pad, st, 0.5, -1.0, old), po.pooling_forward(mode, x, win, pad, st, 0.5, -1.0, old))


@pytest.mark.parametrize("mode", [0, 1], ids=["instance", "channel"])
def test_softmax_backward(mode):
    gu = _gpu()
    for shape in SHAPES + [(64, 1000, 1, 1), (2, 21, 33, 17)]:
        y = po.softmax_forward(mode, rnd(31, *shape, lo=-4, hi=4)).astype(np.float32)
        dy = rnd(32, *shape)
        print("softmax backward", mode, shape, flush=True)
        want = po.softmax_backward(mode, y, dy)
        close(gu.run_softmax_backward(mode, y, dy), want)
        close(gu.run_softmax_backward(mode, wl.with_layout(y, "NHWC"), dy, layout="NHWC"), want)
        close(gu.run_softmax_backward(mode, y, wl.with_layout(dy, "NHWC")), want)
        old = rnd(33, *shape)
        close(gu.run_softmax_backward(mode, y, dy, 0.5, 2.0, old, "NHWC"), po.softmax_backward(mode, y, dy, 0.5, 2.0, old))


@pytest.mark.parametrize("mode", [0, 1], ids=["max", "average"])
def test_pooling_backward(mode):
    gu = _gpu()
    cases = [((2, 3, 9, 11), (2, 2), (0, 0), (2, 2)), ((2, 3, 9, 11), (3, 3), (1, 1), (2, 2)),
             ((1, 5, 13, 13), (3, 2), (1, 0), (1, 3)), ((3, 96, 27, 27), (3, 3), (0, 0), (2, 2)),
             ((2, 4, 7, 7), (7, 7), (0, 0), (1, 1)), ((2, 4, 8, 8), (5, 5), (2, 2), (4, 4)), ((1, 1, 1, 1), (1, 1), (0, 0), (1, 1)),
             ((2, 3, 10, 12), (3, 3), (0, 0), (1, 1)), ((2, 3, 11, 9), (2, 2), (0, 0), (3, 3)), ((1, 2, 6, 30), (1, 5), (0, 2), (1, 2)),
             ((3, 5, 55, 55), (3, 3), (0, 0), (2, 2)), ((2, 3, 37, 20), (3, 3), (1, 1), (1, 1)),
             ((1, 2, 9, 700), (3, 3), (1, 1), (1, 1)),       # wide rows: fewer rows per workgroup
             ((1, 1, 4, 2000), (3, 3), (1, 1), (1, 1)),      # too wide for the row-strip kernel
             # stride 2 both ways (a thread per 2 x 2 cell of inputs): several strips of rows, a last row and
             # column no window reaches, zero borders
             ((2, 2, 130, 40), (3, 3), (1, 1), (2, 2)), ((2, 2, 130, 40), (2, 2), (1, 1), (2, 2)),
             ((2, 3, 10, 12), (3, 3), (0, 0), (2, 2)), ((1, 2, 70, 255), (3, 3), (2, 2), (2, 2)), ((1, 2, 66, 256), (2, 2), (0, 0), (2, 2))]
    for shape, win, pad, st in cases:
        x = rnd(35, *shape) - np.float32(5.0)
        P, Q = po.pooling_output_dim(shape[2], win[0], pad[0], st[0]), po.pooling_output_dim(shape[3], win[1], pad[1], st[1])
        dy = rnd(36, shape[0], shape[1], P, Q)
        print("pooling backward", mode, shape, win, pad, st, flush=True)
        want = po.pooling_backward(mode, x, dy, win, pad, st)
        close(gu.run_pooling_backward(mode, x, dy, win, pad, st), want)
        close(gu.run_pooling_backward(mode, wl.with_layout(x, "NHWC"), wl.with_layout(dy, "NHWC"), win, pad, st, layout="NHWC"), want)
        old = rnd(37, *shape)
        close(gu.run_pooling_backward(mode, x, dy, win, pad, st, 0.5, -1.0, old), po.pooling_backward(mode, x, dy, win, pad, st, 0.5, -1.0, old))
    # equal maxima: data on a coarse grid (many ties inside every window); the first in scan order takes the gradient
    x = np.round(rnd(38, 2, 3, 12, 14)).astype(np.float32)
    for win, pad, st in [((3, 3), (1, 1), (2, 2)), ((2, 2), (0, 0), (1, 1)), ((4, 3), (2, 1), (2, 1))]:
        P, Q = po.pooling_output_dim(12, win[0], pad[0], st[0]), po.pooling_output_dim(14, win[1], pad[1], st[1])
        dy = rnd(39, 2, 3, P, Q)
        close(gu.run_pooling_backward(mode, x, dy, win, pad, st), po.pooling_backward(mode, x, dy, win, pad, st))


def test_transform_tensor_changes_layout():
    gu = _gpu()
    for shape in SHAPES + [(3, 70, 9, 11), (2, 64, 56, 56), (1, 200, 1, 33), (5, 17, 64, 1), (2, 16, 4, 4), (2, 130, 3, 67)]:
        x = rnd(41, *shape)
        want = x.astype(np.float64)
        old = rnd(42, *shape)
        for src in ("NCHW", "NHWC"):
            for dst in ("NCHW", "NHWC"):
                print("transform", shape, src, dst, flush=True)
                xs = wl.with_layout(x, src)
                assert np.array_equal(gu.run_transform_tensor(xs, layout=dst), want)        # a copy is exact
                close(gu.run_transform_tensor(xs, -0.5, 2.0, old, dst), po.add_tensor(x, shape, -0.5, 2.0, old))
    # a pitched destination (rows padded to 80 elements) and a channel slice as the source
    x = rnd(43, 2, 24, 9, 70)
    y_strides = (24 * 9 * 80, 9 * 80, 80, 1)
    assert np.array_equal(gu.run_transform_tensor(wl.with_layout(x, "NHWC"), y_strides=y_strides), x.astype(np.float64))
    part = wl.with_layout(x, "NHWC")[:, 4:20]
    assert np.array_equal(gu.run_transform_tensor(part, layout="NCHW"), x[:, 4:20].astype(np.float64))
    # other orders of the dimensions: w-major source into NCHW, h-major destination
    xt = np.ascontiguousarray(x.transpose(3, 0, 1, 2)).transpose(1, 2, 3, 0)        # memory order W,N,C,H
    assert np.array_equal(gu.run_transform_tensor(xt, layout="NCHW"), x.astype(np.float64))
    assert np.array_equal(gu.run_transform_tensor(x, y_strides=(24 * 70 * 9, 70 * 9, 1, 9)), x.astype(np.float64))


def test_matrix_rate_probe():
    """The measurement aid of the bench: the register-only MFMA loop returns a plausible rate for every data type, with
    uniform and with pseudo-random operands (the same instruction stream, other values: never faster), and refuses bad
    arguments."""
    import torch
    import paper_1410_0759_amd as ig
    _gpu()
    h = ig.Handle()
    h.set_stream(torch.cuda.current_stream().cuda_stream)
    cus, khz = ig.get_device_properties(h)
    assert cus >= 8 and khz > 100000
    for name, dt, peak in (("f32", ig.IGC_DATA_FLOAT, 157.3), ("bf16", ig.IGC_DATA_BFLOAT16, 2516.6), ("f64", ig.IGC_DATA_DOUBLE, 78.6)):
        ig.measure_matrix_rate_operands(h, dt, 20, 0)   # (clocks)
        uniform = ig.measure_matrix_rate_operands(h, dt, 40, 0)
        same = ig.measure_matrix_rate(h, dt, 40)
        random = ig.measure_matrix_rate_operands(h, dt, 40, 1)
        print("matrix rate", name, uniform, same, random, flush=True)
        assert 0.3 * peak < random <= 1.05 * uniform and uniform < 1.1 * peak
        assert abs(same - uniform) < 0.1 * uniform
    for bad in ((ig.IGC_DATA_FLOAT, 0, 0), (ig.IGC_DATA_FLOAT, 5000, 1), (ig.IGC_DATA_FLOAT, 10, 2), (17, 10, 0)):
        with pytest.raises(ig.IgcError):
            ig.measure_matrix_rate_operands(h, *bad)


def test_backward_bias():
    """db[c] = alpha * sum of dy over images and pixels + beta * db: every layout and input type, with the workspace the
    library asks for, with none and with too little (then one range), a pitched db, repeatable bit for bit."""
    gu = _gpu()
    shapes = SHAPES + [(5, 70, 9, 11), (16, 64, 28, 28), (3, 200, 17, 5), (64, 3, 40, 41), (2, 1, 300, 300)]
    for i, shape in enumerate(shapes):
        dy = rnd(300 + i, *shape, lo=-1.0, hi=1.0)
        want = po.bias_backward(dy)
        old = rnd(320 + i, shape[1]).astype(np.float64)
        for layout in ("NCHW", "NHWC"):
            dyl = wl.with_layout(dy, layout)
            print("backward bias", shape, layout, flush=True)
            asked = []
            got = gu.run_backward_bias(dyl, asked=asked)
            close(got, want)
            assert np.array_equal(got, gu.run_backward_bias(dyl))                          # the same bits again
            close(gu.run_backward_bias(dyl, workspace="none"), want)
            close(gu.run_backward_bias(dyl, workspace=max(asked[0] - 8, 0)), want)         # too little: not used
            close(gu.run_backward_bias(dyl, -0.5, 2.0, old, db_stride=3), po.bias_backward(dy, -0.5, 2.0, old))
            # bfloat16 gradients (the oracle consumes the rounded values)
            dyb = wl.round_to_bf16(dy)
            close(gu.run_backward_bias(wl.with_layout(dyb, layout), dtype="bf16"), po.bias_backward(dyb))
    # a pitched, sliced gradient: every second feature map of a larger tensor
    big = rnd(340, 4, 24, 9, 20, lo=-1.0, hi=1.0)
    part = big[:, 3:19:2, :, 2:17]
    close(gu.run_backward_bias(part), po.bias_backward(np.ascontiguousarray(part)))
    # a single large element in a sea of zeros lands in its own feature map
    z = np.zeros((3, 130, 7, 9), dtype=np.float32)
    z[2, 129, 6, 8] = 7.0
    got = gu.run_backward_bias(wl.with_layout(z, "NHWC"))
    assert got[129] == 7.0 and np.count_nonzero(got) == 1
