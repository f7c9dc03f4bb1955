"""GPU parity of the backward passes: the HIP library (through its C ABI) against the CPU
oracle's backward forms, element by element on the same seeded inputs.  Bar as for the
forward pass: max|gpu - oracle| / max|oracle| <= 2e-5 (fp32), <= 1e-2 (bf16 inputs)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import workloads as wl
from oracle import conv_oracle as oc


def _gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def _rnd(seed, shape, dtype):
    a = np.random.default_rng(seed).uniform(-1, 1, size=shape).astype(np.float32)
    return wl.round_to_bf16(a) if dtype == "bf16" else a


# N, C, H, W, K, R, S, pad, stride
BWD_PROBLEMS = [
    (2, 5, 9, 11, 7, 3, 3, (1, 1), (1, 1)),
    (3, 40, 14, 13, 150, 3, 3, (1, 1), (1, 1)),       # several tiles, ragged channel chunks
    (2, 3, 23, 21, 70, 5, 5, (2, 2), (2, 2)),         # four phases
    (1, 6, 30, 17, 20, 7, 1, (3, 0), (3, 1)),         # a phase with fewer taps
    (2, 4, 12, 12, 9, 1, 1, (0, 0), (2, 2)),          # 1x1, stride 2: three phases meet no tap
    (1, 3, 35, 35, 96, 11, 11, (0, 0), (4, 4)),       # first-layer shape, 16 phases
    (2, 7, 12, 40, 33, 1, 7, (0, 3), (1, 3)),
    (2, 2, 8, 8, 4, 4, 4, (3, 3), (1, 1)),            # "full" padding
    (2, 8, 10, 11, 5, 3, 3, (0, 0), (3, 3)),          # stride leaves rows and columns unread
    (2, 24, 12, 13, 64, 3, 3, (1, 1), (1, 1)),        # nine taps, K in fours: nine-tap table with strided filter reads
    (3, 70, 9, 9, 132, 3, 3, (0, 2), (1, 1)),         # the same with several row tiles and an odd step count
    (1, 8, 20, 21, 16, 9, 9, (4, 4), (3, 3)),         # 9x9 with stride 3: every phase has nine taps
    (2, 6, 11, 10, 12, 1, 9, (0, 4), (1, 1)),         # nine taps in a row
]


def _check_bd(prob, dtype, mode, alpha=1.0, beta=0.0, dx_layout="NCHW", dy_layout="NCHW", seed=0, workspace="full",
              asked=None):
    gu = _gpu()
    N, C, H, W, K, R, S, pad, stride = prob
    P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
    dy = wl.with_layout(_rnd(seed + 1, (N, K, P, Q), dtype), dy_layout)
    w = _rnd(seed + 2, (K, C, R, S), dtype)
    dx_old = _rnd(seed + 3, (N, C, H, W), "f32") if beta != 0.0 else None
    print("backward data", prob, dtype, mode, alpha, beta, dx_layout, dy_layout, flush=True)
    got = gu.run_backward_data(dy, w, (H, W), pad, stride, mode, alpha, beta, dx_old, dtype, dx_layout, workspace, asked)
    want = oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride, mode=mode, alpha=alpha, beta=beta, dx_old=dx_old)
    assert got.shape == want.shape
    assert np.all(np.isfinite(got)), "non-finite output (NaN prefill leaked or garbage)"
    err = gu.rel_err(got, want)
    assert err <= gu.BOUND[dtype], "rel err %.3g > %.3g" % (err, gu.BOUND[dtype])
    return err


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("prob", BWD_PROBLEMS, ids=[str(i) for i in range(len(BWD_PROBLEMS))])
def test_backward_data_sweep(prob, dtype, mode):
    _check_bd(prob, dtype, mode, seed=10 * BWD_PROBLEMS.index(prob))


@pytest.mark.parametrize("dx_layout,dy_layout", [("NHWC", "NHWC"), ("NHWC", "NCHW"), ("NCHW", "NHWC")])
def test_backward_data_layouts(dx_layout, dy_layout):
    _check_bd(BWD_PROBLEMS[1], "f32", 1, dx_layout=dx_layout, dy_layout=dy_layout)
    _check_bd(BWD_PROBLEMS[2], "bf16", 0, dx_layout=dx_layout, dy_layout=dy_layout)


def test_backward_data_accumulates():
    """out = alpha * raw + beta * old; rows the forward pass never reads keep beta * old."""
    for prob in (BWD_PROBLEMS[1], BWD_PROBLEMS[4], BWD_PROBLEMS[8]):
        _check_bd(prob, "f32", 1, alpha=0.5, beta=-1.5)
        _check_bd(prob, "f32", 0, alpha=2.0, beta=1.0, dx_layout="NHWC")


# float, a stride above 1 and few channels: with the workspace it asks for the library runs all phases as one
# forward pass over dy (u*v*C output maps) and moves the result to dx; without, one launch per phase.
# N, C, H, W, K, R, S, pad, stride
BWD_PACKED_PHASES = [
    (2, 3, 35, 33, 8, 11, 11, (0, 0), (4, 4)),      # the first-layer shape: 16 phases, 3x3 taps each
    (2, 3, 37, 34, 8, 11, 11, (0, 0), (4, 4)),      # rows and columns no window reaches
    (2, 3, 19, 18, 5, 3, 3, (1, 1), (2, 1)),        # one axis strided
    (1, 4, 20, 21, 6, 5, 4, (2, 1), (3, 2)),        # unequal everything, padded
    (2, 8, 17, 16, 7, 2, 2, (0, 0), (2, 2)),        # windows that do not overlap
    (1, 2, 13, 14, 4, 2, 2, (0, 0), (3, 3)),        # stride above the filter size: phases without taps
    (1, 3, 23, 22, 4, 7, 7, (6, 6), (2, 2)),        # "full" padding
    (3, 32, 12, 12, 9, 3, 3, (1, 1), (2, 2)),       # 128 maps: the most the route takes
]


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
def test_backward_data_strided_few_channels_both_routes(mode):
    for i, prob in enumerate(BWD_PACKED_PHASES):
        asked = []
        _check_bd(prob, "f32", mode, seed=40 + i, asked=asked)
        assert asked[0] > 0, "this problem should ask for the workspace of the one-pass route"
        _check_bd(prob, "f32", mode, seed=40 + i, workspace="none")
        _check_bd(prob, "f32", mode, seed=40 + i, workspace=asked[0] - 4)      # too small: the general route
    _check_bd(BWD_PACKED_PHASES[1], "f32", mode, alpha=0.5, beta=-1.5, dx_layout="NHWC", dy_layout="NHWC")
    _check_bd(BWD_PACKED_PHASES[3], "f32", mode, alpha=2.0, beta=1.0)
    # many channels: the per-phase launches fill their tiles; they read the filter through its strides in the
    # reduction's own order (one decode per thread and step) and ask for nothing
    asked = []
    _check_bd((2, 40, 12, 12, 9, 3, 3, (1, 1), (2, 2)), "f32", mode, asked=asked)
    assert asked[0] == 0


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
def test_backward_data_tap_major_with_filter_workspace(mode):
    """bfloat16 phases in tap-major order (filters other than nine taps, or strided nine-tap ones whose phases have
    fewer taps; float problems read the filter through its strides in filter order instead): with a workspace of
    the filter's size the filter is rewritten as wt[c][t][k] and read through those strides.  Same sums in the
    same order: the same bits as without the workspace."""
    gu = _gpu()
    for i, prob in enumerate([(3, 40, 14, 13, 70, 5, 5, (2, 2), (1, 1)), (2, 150, 9, 11, 33, 7, 3, (3, 1), (1, 1)),
                              (2, 64, 15, 15, 48, 5, 5, (2, 2), (3, 3)), (2, 40, 12, 12, 9, 3, 3, (1, 1), (2, 2))]):
        N, C, H, W, K, R, S, pad, stride = prob
        P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
        dy, w = _rnd(61 + i, (N, K, P, Q), "bf16"), _rnd(71 + i, (K, C, R, S), "bf16")
        want = oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride, mode=mode)
        asked = []
        print("backward data, filter workspace", prob, mode, flush=True)
        got = gu.run_backward_data(dy, w, (H, W), pad, stride, mode, dtype="bf16", asked=asked)
        assert asked[0] == K * C * R * S * 2
        assert gu.rel_err(got, want) <= gu.BOUND["bf16"]
        assert np.array_equal(got, gu.run_backward_data(dy, w, (H, W), pad, stride, mode, dtype="bf16", workspace="none"))
        assert np.array_equal(got, gu.run_backward_data(dy, w, (H, W), pad, stride, mode, dtype="bf16", workspace=asked[0] - 4))


# bf16, unit stride, nine taps, dy with contiguous channels (K a multiple of 16): the library asks
# for room for the filter with k and c exchanged and runs the forward pass's channel-vector
# kernels over dy.  N, C, H, W, K, R, S, pad, stride
BWD_AS_FORWARD = [
    (2, 16, 9, 11, 16, 3, 3, (1, 1), (1, 1)),
    (3, 40, 14, 13, 144, 3, 3, (1, 1), (1, 1)),      # C not a multiple of the exchange block, several row tiles
    (2, 5, 12, 10, 32, 3, 3, (0, 0), (1, 1)),        # pad 0 becomes "full" padding of dy
    (2, 24, 8, 9, 48, 3, 3, (2, 2), (1, 1)),         # "full" padding becomes pad 0
    (2, 7, 6, 20, 32, 1, 9, (0, 3), (1, 1)),         # nine taps in a row
    (1, 130, 28, 28, 64, 3, 3, (1, 0), (1, 1)),      # unequal pads, 130 rows
    (2, 40, 9, 11, 48, 1, 1, (0, 0), (1, 1)),        # 1x1: the filter transposed, then a plain product
    (3, 7, 14, 13, 136, 1, 1, (0, 0), (1, 1)),
]


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
@pytest.mark.parametrize("prob", BWD_AS_FORWARD, ids=[str(i) for i in range(len(BWD_AS_FORWARD))])
def test_backward_data_bf16_channel_vectors(prob, mode):
    N, C, H, W, K, R, S, pad, stride = prob
    for dx_layout in ("NHWC", "NCHW"):
        asked = []
        _check_bd(prob, "bf16", mode, dx_layout=dx_layout, dy_layout="NHWC", seed=7, asked=asked)
        assert asked == [K * C * R * S * 2]
    # the same problem without the workspace (general route), and with one that is too small
    _check_bd(prob, "bf16", mode, dx_layout="NHWC", dy_layout="NHWC", seed=7, workspace="none")
    _check_bd(prob, "bf16", mode, dx_layout="NHWC", dy_layout="NHWC", seed=7, workspace=K * C * R * S * 2 - 2)
    _check_bd(prob, "bf16", mode, alpha=-0.5, beta=2.0, dx_layout="NHWC", dy_layout="NHWC", seed=8)
    # shapes that do not qualify ask for nothing
    asked = []
    _check_bd(prob, "bf16", mode, dy_layout="NCHW", seed=7, asked=asked)
    _check_bd(prob, "f32", mode, dy_layout="NHWC", seed=7, asked=asked)
    # (nothing, or the filter's size should the general route's launches run in tap-major order)
    assert asked[0] in (0, K * C * R * S * 2) and asked[1] in (0, K * C * R * S * 4)


def test_backward_data_is_the_transpose_of_forward_on_the_gpu():
    """<forward(x,w), dy> == <x, backward_data(dy,w)> with both sides from the library."""
    gu = _gpu()
    N, C, H, W, K, R, S, pad, stride = BWD_PROBLEMS[2]
    x, w = _rnd(1, (N, C, H, W), "f32"), _rnd(2, (K, C, R, S), "f32")
    y, _ = gu.run(x, w, pad, stride, 1)
    dy = _rnd(3, y.shape, "f32")
    dx = gu.run_backward_data(dy, w, (H, W), pad, stride, 1)
    lhs, rhs = float(np.sum(y * dy)), float(np.sum(dx * x))
    assert abs(lhs - rhs) <= 1e-4 * max(1.0, abs(lhs))


# ------------------------------------------------------------------ backward filter
def _check_bf(prob, dtype, mode, alpha=1.0, beta=0.0, x_layout="NCHW", dy_layout="NCHW", workspace="full", seed=0):
    gu = _gpu()
    N, C, H, W, K, R, S, pad, stride = prob
    P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
    x = wl.with_layout(_rnd(seed + 1, (N, C, H, W), dtype), x_layout)
    dy = wl.with_layout(_rnd(seed + 2, (N, K, P, Q), dtype), dy_layout)
    dw_old = _rnd(seed + 3, (K, C, R, S), "f32") if beta != 0.0 else None
    print("backward filter", prob, dtype, mode, alpha, beta, x_layout, dy_layout, workspace, flush=True)
    got, asked = gu.run_backward_filter(x, dy, (R, S), pad, stride, mode, alpha, beta, dw_old, dtype, workspace)
    want = oc.conv_backward_filter(x, dy, (R, S), pad=pad, stride=stride, mode=mode, alpha=alpha, beta=beta, dw_old=dw_old)
    assert got.shape == want.shape
    assert np.all(np.isfinite(got)), "non-finite output (NaN prefill or workspace leaked)"
    err = gu.rel_err(got, want)
    assert err <= gu.BOUND[dtype], "rel err %.3g > %.3g" % (err, gu.BOUND[dtype])
    return got, asked


BF_PROBLEMS = BWD_PROBLEMS + [
    (16, 24, 28, 28, 40, 3, 3, (1, 1), (1, 1)),       # long reduction: cut into many ranges
    (8, 3, 57, 57, 96, 11, 11, (0, 0), (4, 4)),       # many columns, few channels
]


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("prob", BF_PROBLEMS, ids=[str(i) for i in range(len(BF_PROBLEMS))])
def test_backward_filter_sweep(prob, dtype, mode):
    _check_bf(prob, dtype, mode, seed=10 * BF_PROBLEMS.index(prob))


@pytest.mark.parametrize("x_layout,dy_layout", [("NHWC", "NHWC"), ("NHWC", "NCHW"), ("NCHW", "NHWC")])
def test_backward_filter_layouts(x_layout, dy_layout):
    _check_bf(BF_PROBLEMS[1], "f32", 1, x_layout=x_layout, dy_layout=dy_layout)
    _check_bf(BF_PROBLEMS[2], "bf16", 0, x_layout=x_layout, dy_layout=dy_layout)


def test_backward_filter_workspace_sizes_and_accumulate():
    """Any workspace size works (none: one range straight into dw; partial: fewer ranges), the
    results agree to rounding, and alpha/beta apply once whatever the number of ranges."""
    prob = BF_PROBLEMS[-2]
    full, asked = _check_bf(prob, "f32", 1, alpha=0.5, beta=-1.5)
    K, C, R, S = prob[4], prob[1], prob[5], prob[6]
    part = K * C * R * S * 4
    assert asked >= 2 * part and asked % part == 0, "this problem should be cut into several ranges"
    for ws in ("none", part, 3 * part + 8, asked + 4096):
        got, _ = _check_bf(prob, "f32", 1, alpha=0.5, beta=-1.5, workspace=ws)
        assert np.max(np.abs(got - full)) <= 1e-4 * np.max(np.abs(full))
    again, _ = _check_bf(prob, "f32", 1, alpha=0.5, beta=-1.5)
    assert np.array_equal(again, full), "same call, same bits"


# bf16 with contiguous channels in x and dy, C >= 24, C and K multiples of 8: the channel-vector
# kernels (operand tiles transposed in registers).  N, C, H, W, K, R, S, pad, stride
BF_VECTOR_PROBLEMS = [
    (2, 24, 12, 13, 64, 3, 3, (1, 1), (1, 1)),
    (3, 40, 14, 13, 152, 3, 3, (1, 1), (1, 1)),       # ragged row and column tiles
    (1, 136, 7, 9, 8, 3, 3, (1, 1), (1, 1)),          # 63 pixels: a single, partial step; K below a vector row tile
    (2, 32, 9, 9, 72, 1, 1, (0, 0), (1, 1)),          # 1x1
    (2, 24, 15, 17, 40, 5, 5, (2, 2), (2, 2)),        # stride 2, 25 taps
    (2, 64, 10, 12, 200, 3, 2, (0, 1), (1, 2)),       # unequal filter, pads and strides
    (5, 48, 20, 20, 96, 3, 3, (2, 2), (1, 1)),        # "full" padding, 2420 pixels: several ranges
    (1, 24, 6, 70, 16, 1, 7, (0, 3), (1, 3)),
]


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
@pytest.mark.parametrize("prob", BF_VECTOR_PROBLEMS, ids=[str(i) for i in range(len(BF_VECTOR_PROBLEMS))])
def test_backward_filter_bf16_channel_vectors(prob, mode):
    kw = dict(x_layout="NHWC", dy_layout="NHWC", seed=5)
    first, asked = _check_bf(prob, "bf16", mode, **kw)
    again, _ = _check_bf(prob, "bf16", mode, **kw)
    assert np.array_equal(first, again)            # ordered sum of the ranges: repeatable bit by bit
    _check_bf(prob, "bf16", mode, workspace="none", **kw)
    assert asked > 0                                # (these kernels use a workspace even for a single range)
    for part in (asked // 2, asked - 4, 64):        # room for fewer ranges, down to none (results written straight to dw)
        _check_bf(prob, "bf16", mode, workspace=part, **kw)
    _check_bf(prob, "bf16", mode, alpha=0.5, beta=-2.0, **kw)
    _check_bf(prob, "bf16", mode, alpha=0.5, beta=-2.0, workspace="none", **kw)
    # one operand without contiguous channels: the element-wise kernels take over
    _check_bf(prob, "bf16", mode, x_layout="NHWC", dy_layout="NCHW", seed=5)


def test_backward_filter_is_the_transpose_of_forward_on_the_gpu():
    gu = _gpu()
    N, C, H, W, K, R, S, pad, stride = BWD_PROBLEMS[2]
    x, w = _rnd(1, (N, C, H, W), "f32"), _rnd(2, (K, C, R, S), "f32")
    y, _ = gu.run(x, w, pad, stride, 0)
    dy = _rnd(3, y.shape, "f32")
    dw, _ = gu.run_backward_filter(x, dy, (R, S), pad, stride, 0)
    lhs, rhs = float(np.sum(y * dy)), float(np.sum(dw * w))
    assert abs(lhs - rhs) <= 1e-4 * max(1.0, abs(lhs))


# ------------------------------------------------------------------ the workloads' own sizes
@pytest.mark.parametrize("index", [2, 3, 4, 5])
def test_backward_at_workload_size(index):
    """Backward data and backward filter at the size of workloads 2-5, in the launch
    configuration the bench times; compared with the oracle on the first images (backward
    data: those images of dx, all elements; backward filter: the pass run on those images)
    and, at full size, through the transpose identity <dy, forward(x,w)> = <dx, x> = <dw, w>
    with the forward result from the library."""
    gu = _gpu()
    w_ = wl.by_index(index)
    x, w, _ = wl.make_inputs(w_)
    pad, stride = (w_.pad_h, w_.pad_w), (w_.u, w_.v)
    dy = np.random.default_rng(77 + index).uniform(-1, 1, size=(w_.N, w_.K, w_.P, w_.Q)).astype(np.float32)
    if w_.dtype == "bf16":
        dy = wl.round_to_bf16(dy)
    dy = wl.with_layout(dy, w_.y_layout)
    n = 4
    print("backward at workload size", w_.name, flush=True)
    dx = gu.run_backward_data(dy, w, (w_.H, w_.W), pad, stride, w_.mode, dtype=w_.dtype, dx_layout=w_.x_layout)
    want = oc.conv_backward_data(dy[:n], w, (w_.H, w_.W), pad=pad, stride=stride, mode=w_.mode)
    assert gu.rel_err(dx[:n], want) <= gu.BOUND[w_.dtype]
    if index == 2:
        # the strided first layer has two routes: all stride phases as one pass (with the workspace,
        # above) and one launch per phase (without); both against the oracle, and against each other
        dx_phases = gu.run_backward_data(dy, w, (w_.H, w_.W), pad, stride, w_.mode, dtype=w_.dtype, dx_layout=w_.x_layout,
                                         workspace="none")
        assert gu.rel_err(dx_phases[:n], want) <= gu.BOUND[w_.dtype]
        assert gu.rel_err(dx_phases, dx) <= gu.BOUND[w_.dtype]
    dw_n, _ = gu.run_backward_filter(x[:n], dy[:n], (w_.R, w_.S), pad, stride, w_.mode, dtype=w_.dtype)
    want = oc.conv_backward_filter(x[:n], dy[:n], (w_.R, w_.S), pad=pad, stride=stride, mode=w_.mode)
    assert gu.rel_err(dw_n, want) <= gu.BOUND[w_.dtype]
    dw, asked = gu.run_backward_filter(x, dy, (w_.R, w_.S), pad, stride, w_.mode, dtype=w_.dtype)
    assert asked > 0
    y, _ = gu.run(x, w, pad, stride, w_.mode, dtype=w_.dtype, y_layout=w_.y_layout)
    lhs = float(np.sum(y * dy.astype(np.float64)))
    scale = float(np.sqrt(np.sum(y * y) * np.sum(dy.astype(np.float64) ** 2)))
    tol = 1e-5 if w_.dtype == "f32" else 1e-3
    assert abs(lhs - float(np.sum(dx * x.astype(np.float64)))) <= tol * scale
    assert abs(lhs - float(np.sum(dw * w.astype(np.float64)))) <= tol * scale


# ------------------------------------------------------------------ seeded random problems, all three passes
def _random_problem(rng):
    R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    if rng.random() < 0.3:
        R, S = 3, 3
    u, v = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    pad = (int(rng.integers(0, R)), int(rng.integers(0, S)))
    H, W = int(rng.integers(R, R + 14)), int(rng.integers(S, S + 14))
    N, C, K = int(rng.integers(1, 4)), int(rng.choice([1, 3, 4, 16, 24, 33, 64])), int(rng.choice([1, 5, 8, 32, 70, 130]))
    return N, C, H, W, K, R, S, pad, (u, v)


@pytest.mark.parametrize("chunk", range(4))
def test_random_problems_forward_and_both_backward_passes(chunk):
    """40 seeded random problems (filter 1..5, stride 1..3, any pad below the filter size, odd
    channel counts, both layouts, both modes, both data types): every pass against its oracle."""
    gu = _gpu()
    rng = np.random.default_rng(4242 + chunk)
    for i in range(10):
        N, C, H, W, K, R, S, pad, stride = prob = _random_problem(rng)
        r_ = rng.random()
        dtype = "bf16" if r_ < 0.35 else ("f64" if r_ < 0.5 else "f32")
        mode = int(rng.integers(0, 2))
        xl, yl = ("NHWC" if rng.random() < 0.5 else "NCHW"), ("NHWC" if rng.random() < 0.5 else "NCHW")
        P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
        x = wl.with_layout(_rnd(100 * chunk + i, (N, C, H, W), dtype), xl)
        w = _rnd(100 * chunk + i + 50, (K, C, R, S), dtype)
        dy = wl.with_layout(_rnd(100 * chunk + i + 70, (N, K, P, Q), dtype), yl)
        print("random problem", prob, dtype, mode, xl, yl, flush=True)
        # (double precision: float32-valued data held as doubles - the oracle takes float32 values and works in double)
        gx, gw, gdy = (x, w, dy) if dtype != "f64" else (x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64))
        y, _ = gu.run(gx, gw, pad, stride, mode, dtype=dtype, y_layout=yl)
        assert gu.rel_err(y, oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode)) <= gu.BOUND[dtype]
        dx = gu.run_backward_data(gdy, gw, (H, W), pad, stride, mode, dtype=dtype, dx_layout=xl)
        want = oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride, mode=mode)
        assert np.max(np.abs(dx - want)) <= gu.BOUND[dtype] * max(np.max(np.abs(want)), 1e-30)
        dw, _ = gu.run_backward_filter(gx, gdy, (R, S), pad, stride, mode, dtype=dtype)
        assert gu.rel_err(dw, oc.conv_backward_filter(x, dy, (R, S), pad=pad, stride=stride, mode=mode)) <= gu.BOUND[dtype]


# ------------------------------------------------------------------ extents just below the 2^31-byte limit
def test_all_passes_with_a_tensor_of_almost_two_gibibytes():
    """x (and dx) of 1 x 8 x 8191 x 8191 floats = 2 146 959 392 bytes, 524 256 bytes below the
    limit of the 32-bit byte offsets: the last rows of the last channel sit at the highest
    offsets the library can form.  3x3, stride 2, no padding.  The oracle checks the top and the
    bottom strip of every result (a strip of the image is a problem of its own)."""
    gu = _gpu()
    N, C, H, W, K, R, S, stride = 1, 8, 8191, 8191, 4, 3, 3, (2, 2)
    P, Q = oc.output_dim(H, R, 2, 0), oc.output_dim(W, S, 2, 0)
    rng = np.random.default_rng(2031)
    x = rng.random(size=(N, C, H, W), dtype=np.float32) - np.float32(0.5)
    w = _rnd(1, (K, C, R, S), "f32")
    rows = 65                       # image rows in a strip: 32 output rows
    prow = (rows - R) // 2 + 1
    print("forward near the offset limit", flush=True)
    y, _ = gu.run(x, w, (0, 0), stride, 1)
    assert y.shape == (N, K, P, Q)
    for strip, out in ((slice(0, rows), slice(0, prow)), (slice(H - rows, H), slice(P - prow, P))):
        want = oc.conv_forward(np.ascontiguousarray(x[:, :, strip]), w, stride=stride, mode=1)
        assert gu.rel_err(y[:, :, out], want) <= gu.BOUND["f32"]
    del y
    print("backward filter near the offset limit", flush=True)
    # dy zero except in the top and bottom strips: dw is then the sum of the two strips' own results
    dy = np.zeros((N, K, P, Q), dtype=np.float32)
    dy[:, :, :prow] = rng.random(size=(N, K, prow, Q), dtype=np.float32) - np.float32(0.5)
    dy[:, :, P - prow:] = rng.random(size=(N, K, prow, Q), dtype=np.float32) - np.float32(0.5)
    dw, _ = gu.run_backward_filter(x, dy, (R, S), (0, 0), stride, 1)
    want = (oc.conv_backward_filter(np.ascontiguousarray(x[:, :, :rows]), np.ascontiguousarray(dy[:, :, :prow]), (R, S), stride=stride, mode=1)
            + oc.conv_backward_filter(np.ascontiguousarray(x[:, :, H - rows:]), np.ascontiguousarray(dy[:, :, P - prow:]), (R, S), stride=stride, mode=1))
    assert gu.rel_err(dw, want) <= gu.BOUND["f32"]
    del x
    print("backward data near the offset limit", flush=True)
    dx = gu.run_backward_data(dy, w, (H, W), (0, 0), stride, 1)
    assert dx.shape == (N, C, H, W)
    top = oc.conv_backward_data(np.ascontiguousarray(dy[:, :, :prow]), w, (rows, W), stride=stride, mode=1)
    bottom = oc.conv_backward_data(np.ascontiguousarray(dy[:, :, P - prow:]), w, (rows, W), stride=stride, mode=1)
    assert gu.rel_err(dx[:, :, :rows], top) <= gu.BOUND["f32"]
    assert gu.rel_err(dx[:, :, H - rows:], bottom) <= gu.BOUND["f32"]
    assert not np.any(dx[:, :, rows:H - rows])      # rows that only zero gradients reach


def test_bf16_channel_vector_routes_fall_back_on_pointers_off_the_16_byte_grid():
    """The channel-vector kernels read 16-byte vectors; tensors that start 2 bytes off that grid
    (or a workspace that does) must take the element-wise routes and give the same results."""
    gu = _gpu()
    import torch
    import paper_1410_0759_amd as ig
    N, C, H, W, K, R, S = 2, 32, 9, 10, 48, 3, 3
    x = wl.with_layout(_rnd(1, (N, C, H, W), "bf16"), "NHWC")
    dy = wl.with_layout(_rnd(2, (N, K, H, W), "bf16"), "NHWC")
    w = _rnd(3, (K, C, R, S), "bf16")
    want_dw = oc.conv_backward_filter(x, dy, (R, S), pad=(1, 1), mode=1)
    want_dx = oc.conv_backward_data(dy, w, (H, W), pad=(1, 1), mode=1)

    def shifted(a):      # device copy of a's memory span, starting one element after a 256-byte boundary
        flat = np.ascontiguousarray(np.lib.stride_tricks.as_strided(a, shape=(gu.extent(a.shape, gu.elem_strides(a)),), strides=(a.itemsize,)))
        buf = torch.zeros(flat.size + 8, dtype=torch.bfloat16, device="cuda")
        buf[1:1 + flat.size].copy_(torch.from_numpy(flat).to(torch.bfloat16))
        assert buf.data_ptr() % 16 == 0
        return buf, buf.data_ptr() + 2

    BF = ig.IGC_DATA_BFLOAT16
    xd = ig.TensorDescriptor().set(BF, N, C, H, W, gu.elem_strides(x))
    dyd = ig.TensorDescriptor().set(BF, N, K, H, W, gu.elem_strides(dy))
    wd = ig.FilterDescriptor().set(BF, K, C, R, S)
    dwd = ig.FilterDescriptor().set(ig.IGC_DATA_FLOAT, K, C, R, S)
    dxd = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, N, C, H, W, (C * H * W, H * W, W, 1))
    conv = ig.ConvolutionDescriptor().set(1, 1, 1, 1, ig.IGC_CROSS_CORRELATION)
    h = ig.Handle()
    h.set_stream(torch.cuda.current_stream().cuda_stream)
    xb, xp = shifted(x)
    dyb, dyp = shifted(dy)
    wb, wp = shifted(w)
    ws_bytes = ig.get_backward_filter_workspace_size(h, xd, dyd, conv, dwd)
    ws = torch.empty(ws_bytes // 4 + 4, device="cuda")
    dw = torch.full((K, C, R, S), float("nan"), device="cuda")
    ig.check(ig.convolution_backward_filter(h, 1.0, xd, xp, dyd, dyp, conv, 0.0, dwd, dw.data_ptr(), ws.data_ptr(), ws_bytes), "wgrad")
    torch.cuda.synchronize()
    assert gu.rel_err(dw.cpu().numpy().astype(np.float64), want_dw) <= gu.BOUND["bf16"]
    ws2_bytes = ig.get_backward_data_workspace_size(h, wd, dyd, conv, dxd)
    assert ws2_bytes == K * C * 9 * 2
    ws2 = torch.empty(ws2_bytes // 4 + 4, device="cuda")
    for dy_ptr, ws_ptr in ((dyp, ws2.data_ptr()), (dyp, ws2.data_ptr() + 4)):   # dy off the grid; the workspace off it too
        dx = torch.full((N, C, H, W), float("nan"), device="cuda")
        ig.check(ig.convolution_backward_data(h, 1.0, wd, wp, dyd, dy_ptr, conv, 0.0, dxd, dx.data_ptr(), ws_ptr, ws2_bytes), "dgrad")
        torch.cuda.synchronize()
        assert gu.rel_err(dx.cpu().numpy().astype(np.float64), want_dx) <= gu.BOUND["bf16"]


def _random_layers(count, seed):
    """Seeded random layers: sizes, taps, borders (up to "full" and beyond the filter), strides, both modes, both data
    types, packed and channel-fastest tensors, with and without a workspace."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        dtype = ("f32", "bf16")[int(rng.integers(0, 2))]
        R, S = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        u, v = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        pad = (int(rng.integers(0, R + 1)), int(rng.integers(0, S + 1)))
        H, W = int(rng.integers(1, 25)), int(rng.integers(1, 25))
        if H + 2 * pad[0] < R or W + 2 * pad[1] < S:
            continue
        N, K = int(rng.integers(1, 7)), int(rng.integers(1, 91))
        C = int(rng.integers(1, 81))
        if rng.integers(0, 3) == 0:
            C = 16 * int(rng.integers(1, 6))     # whole channel vectors: the bf16 channel-vector kernels become eligible
        layout = ("NCHW", "NHWC")[int(rng.integers(0, 2))]
        alpha, beta = (1.0, 0.5, -2.0)[int(rng.integers(0, 3))], (0.0, 0.0, 1.0, -1.5)[int(rng.integers(0, 4))]
        out.append(((N, C, H, W, K, R, S, pad, (u, v)), dtype, int(rng.integers(0, 2)), layout,
                    ("full", "none")[int(rng.integers(0, 2))], alpha, beta))
    return out


def test_random_layers_all_three_passes():
    """150 seeded random layers, each through the forward pass, backward data and backward filter with the kernels
    the library picks, against the oracle (alpha and beta included)."""
    gu = _gpu()
    for i, (prob, dtype, mode, layout, workspace, alpha, beta) in enumerate(_random_layers(150, 2024)):
        N, C, H, W, K, R, S, pad, stride = prob
        print("random layer", i, prob, dtype, mode, layout, workspace, alpha, beta, flush=True)
        x = wl.with_layout(_rnd(7000 + i, (N, C, H, W), dtype), layout)
        w = _rnd(7100 + i, (K, C, R, S), dtype)
        P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
        y0 = _rnd(7150 + i, (N, K, P, Q), "f32") if beta != 0.0 else None
        want = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode, alpha=alpha, beta=beta, y_old=y0)
        got, _ = gu.run(x, w, pad, stride, mode, alpha, beta, y0, dtype, layout)
        assert np.all(np.isfinite(got)) and gu.rel_err(got, want) <= gu.BOUND[dtype]
        _check_bd(prob, dtype, mode, alpha, beta, dx_layout=layout, dy_layout=layout, seed=7200 + 3 * i, workspace=workspace)
        _check_bf(prob, dtype, mode, alpha, beta, x_layout=layout, dy_layout=layout, seed=7400 + 3 * i, workspace=workspace)
