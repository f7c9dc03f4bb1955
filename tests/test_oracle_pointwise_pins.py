"""Pins for the CPU oracle of the library's other functions (Section 2.2): activations,
softmax, pooling, tensor addition with broadcasting.  Closed forms, hand-worked values,
invariants and independent library routines - never the oracle against itself."""
import numpy as np
import pytest

from oracle import pointwise_oracle as po


def rnd(seed, *shape, lo=-3.0, hi=3.0):
    return np.random.default_rng(seed).uniform(lo, hi, size=shape).astype(np.float32)


def nhwc(a):
    return np.ascontiguousarray(a.transpose(0, 2, 3, 1)).transpose(0, 3, 1, 2)


# ---------------------------------------------------------------- activations
def test_activation_known_values():
    x = np.array([0.0, 1.0, -1.0, np.log(3.0), -50.0, 50.0], dtype=np.float32).reshape(1, 1, 2, 3)
    xd = x.astype(np.float64)
    s = po.activation_forward(po.SIGMOID, x)
    assert s[0, 0, 0, 0] == 0.5
    assert abs(s[0, 0, 1, 0] - 0.75) < 1e-7            # sigmoid(ln 3) = 3/4 (x is ln 3 rounded to fp32)
    assert np.allclose(s + po.activation_forward(po.SIGMOID, -x), 1.0, rtol=0, atol=1e-15)   # s(x) + s(-x) = 1
    assert 0.0 < s[0, 0, 1, 1] < 1e-20 and s[0, 0, 1, 2] == 1.0    # sigmoid(-50) ~ 2e-22, sigmoid(50) rounds to 1
    r = po.activation_forward(po.RELU, x)
    assert np.array_equal(r, np.maximum(xd, 0.0))
    t = po.activation_forward(po.TANH, x)
    assert t[0, 0, 0, 0] == 0.0 and np.allclose(t, -po.activation_forward(po.TANH, -x), rtol=0, atol=0)
    assert abs(t[0, 0, 1, 0] - 0.8) < 1e-7             # tanh(ln 3) = (9-1)/(9+1)
    assert np.allclose(t, 2.0 * po.activation_forward(po.SIGMOID, (2 * x).astype(np.float32)) - 1.0, atol=1e-12)


def test_activation_against_numpy_and_scipy():
    from scipy.special import expit
    x = rnd(1, 2, 3, 4, 5)
    assert np.allclose(po.activation_forward(po.SIGMOID, x), expit(x.astype(np.float64)), rtol=1e-14, atol=0)
    assert np.allclose(po.activation_forward(po.TANH, x), np.tanh(x.astype(np.float64)), rtol=1e-14, atol=0)


def test_activation_backward_is_the_derivative():
    """Central differences of the forward function (in fp64 via the closed forms)."""
    x = rnd(2, 1, 2, 3, 4)
    dy = rnd(3, 1, 2, 3, 4)
    xd = x.astype(np.float64)
    f = {po.SIGMOID: lambda v: 1 / (1 + np.exp(-v)), po.RELU: lambda v: np.maximum(v, 0), po.TANH: np.tanh}
    for mode in (po.SIGMOID, po.RELU, po.TANH):
        y = f[mode](xd).astype(np.float32)
        dx = po.activation_backward(mode, y, dy, x)
        eps = 1e-6
        num = (f[mode](xd + eps) - f[mode](xd - eps)) / (2 * eps) * dy
        tol = 1e-6 if mode != po.RELU else 1e-9       # y was rounded to fp32 for sigmoid/tanh
        assert np.allclose(dx, num, rtol=0, atol=tol), mode
    # the rectifier's derivative is taken from x, not from y: x <= 0 gives exactly 0
    dx = po.activation_backward(po.RELU, np.zeros_like(x), dy, x)
    assert np.array_equal(dx != 0, (x > 0) & (dy != 0))


def test_alpha_beta_and_layouts():
    x = rnd(4, 2, 3, 4, 5)
    old = rnd(5, 2, 3, 4, 5)
    raw = po.activation_forward(po.TANH, x)
    assert np.allclose(po.activation_forward(po.TANH, x, alpha=0.5, beta=-2.0, y_old=old), 0.5 * raw - 2.0 * old, atol=1e-15)
    assert np.array_equal(po.activation_forward(po.TANH, nhwc(x), layout="NHWC"), raw)
    with pytest.raises(ValueError):
        po.activation_forward(po.TANH, x, beta=1.0)


# ---------------------------------------------------------------- tensor addition
def test_add_tensor_broadcasts_size_one_dimensions():
    shape = (2, 3, 4, 5)
    old = rnd(6, *shape)
    bias = rnd(7, 1, 3, 1, 1)
    got = po.add_tensor(bias, shape, alpha=2.0, beta=1.0, y_old=old)
    assert np.array_equal(got, 2.0 * bias.astype(np.float64) + old.astype(np.float64))      # numpy broadcasting
    full = rnd(8, *shape)
    assert np.array_equal(po.add_tensor(full, shape), full.astype(np.float64))
    row = rnd(9, 2, 1, 1, 5)
    assert np.array_equal(po.add_tensor(row, shape, beta=-1.0, y_old=old), row.astype(np.float64) - old)
    with pytest.raises(ValueError):
        po.add_tensor(rnd(10, 1, 2, 1, 1), shape)     # 2 is neither 1 nor C


def test_bias_gradient_hand_values_and_the_transpose_of_the_broadcast():
    """db[c] = sum of dy over images and pixels.  Hand case on the integers 0..15 as a (2,2,2,2) tensor: feature map 0
    holds 0..3 and 8..11 (sum 44), feature map 1 holds 4..7 and 12..15 (sum 76); all ones count the N*H*W pixels; the
    function is the transpose of add_tensor's broadcast of a (1,C,1,1) bias (<broadcast(b), dy> = <b, db>), with
    add_tensor pinned on its own above; numpy's sum over the axes; any layout; the accumulate form."""
    dy = np.arange(16, dtype=np.float32).reshape(2, 2, 2, 2)
    assert np.array_equal(po.bias_backward(dy), [44.0, 76.0])
    assert np.array_equal(po.bias_backward(np.ones((3, 5, 4, 7), dtype=np.float32)), np.full(5, 3 * 4 * 7.0))
    dy = rnd(61, 3, 5, 4, 7)
    b = rnd(62, 1, 5, 1, 1)
    lhs = float(np.sum(po.add_tensor(b, dy.shape) * dy.astype(np.float64)))
    rhs = float(np.dot(b.astype(np.float64).reshape(-1), po.bias_backward(dy)))
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), 1.0)
    want = dy.astype(np.float64).sum(axis=(0, 2, 3))
    assert np.allclose(po.bias_backward(dy), want, rtol=1e-14, atol=1e-13)
    assert np.array_equal(po.bias_backward(nhwc(dy)), po.bias_backward(dy))          # strides, not layout, address dy
    old = rnd(63, 5).astype(np.float64)
    assert np.allclose(po.bias_backward(dy, alpha=-0.5, beta=2.0, db_old=old), -0.5 * want + 2.0 * old, rtol=1e-14, atol=1e-13)
    with pytest.raises(ValueError):
        po.bias_backward(dy, beta=1.0)
    # a single large element in a sea of small ones lands in its own feature map only
    z = np.zeros((2, 3, 4, 4), dtype=np.float32)
    z[1, 2, 3, 0] = 7.0
    assert np.array_equal(po.bias_backward(z), [0.0, 0.0, 7.0])
    # double inputs are not truncated to float on the way
    d = np.full((1, 1, 1, 2), 1.0, dtype=np.float64)
    d[0, 0, 0, 1] = 2.0 ** -40
    assert po.bias_backward(d)[0] == 1.0 + 2.0 ** -40


# ---------------------------------------------------------------- softmax
def test_softmax_hand_values_and_stability():
    # exp(0) : exp(ln 2) : exp(ln 3) = 1 : 2 : 3 -> 1/6, 2/6, 3/6 over the channels
    x = np.log(np.array([1.0, 2.0, 3.0])).astype(np.float32).reshape(1, 3, 1, 1)
    y = po.softmax_forward(po.SOFTMAX_CHANNEL, x)
    assert np.allclose(y.ravel(), [1 / 6, 2 / 6, 3 / 6], rtol=0, atol=1e-7)
    # shifting a group by a constant changes nothing; huge inputs neither overflow nor give NaN
    big = (x + np.float32(1000.0)).astype(np.float32)
    yb = po.softmax_forward(po.SOFTMAX_CHANNEL, big)
    assert np.all(np.isfinite(yb)) and np.allclose(yb.ravel(), [1 / 6, 2 / 6, 3 / 6], rtol=0, atol=1e-4)
    # one dominant element: exactly 1 and (underflowed) 0
    d = np.array([0.0, 2000.0, -2000.0], dtype=np.float32).reshape(1, 3, 1, 1)
    assert np.array_equal(po.softmax_forward(po.SOFTMAX_CHANNEL, d).ravel(), [0.0, 1.0, 0.0])


def test_softmax_modes_group_sums_and_scipy():
    from scipy.special import softmax
    x = rnd(11, 3, 5, 4, 6, lo=-8, hi=8)
    xd = x.astype(np.float64)
    ch = po.softmax_forward(po.SOFTMAX_CHANNEL, x)
    assert np.allclose(ch.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert np.allclose(ch, softmax(xd, axis=1), rtol=1e-13, atol=0)
    inst = po.softmax_forward(po.SOFTMAX_INSTANCE, x)
    assert np.allclose(inst.reshape(3, -1).sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert np.allclose(inst, softmax(xd.reshape(3, -1), axis=1).reshape(x.shape), rtol=1e-13, atol=0)
    assert not np.allclose(ch, inst)
    # with H = W = 1 the two modes coincide
    v = rnd(12, 2, 7, 1, 1)
    assert np.array_equal(po.softmax_forward(po.SOFTMAX_CHANNEL, v), po.softmax_forward(po.SOFTMAX_INSTANCE, v))
    assert np.array_equal(po.softmax_forward(po.SOFTMAX_CHANNEL, nhwc(x), layout="NHWC"), ch)


# ---------------------------------------------------------------- pooling
def test_pooling_hand_cases():
    x = np.arange(1, 17, dtype=np.float32).reshape(1, 1, 4, 4)      # rows 1..4, 5..8, 9..12, 13..16
    # 2x2 windows, stride 2: maxima are the bottom-right corners, averages the window means
    assert np.array_equal(po.pooling_forward(po.POOL_MAX, x, (2, 2), stride=(2, 2)).ravel(), [6, 8, 14, 16])
    assert np.array_equal(po.pooling_forward(po.POOL_AVERAGE, x, (2, 2), stride=(2, 2)).ravel(), [3.5, 5.5, 11.5, 13.5])
    # 3x3, pad 1, stride 3 -> P = Q = floor((4+2-3)/3)+1 = 2; window (0,0) covers rows -1..1, cols -1..1:
    # in-image elements 1,2,5,6 -> max 6, mean 3.5; window (1,1) covers rows 2..4, cols 2..4: 11,12,15,16 -> 16, 13.5
    mx = po.pooling_forward(po.POOL_MAX, x, (3, 3), pad=(1, 1), stride=(3, 3))
    av = po.pooling_forward(po.POOL_AVERAGE, x, (3, 3), pad=(1, 1), stride=(3, 3))
    assert mx.shape == (1, 1, 2, 2) and mx[0, 0, 0, 0] == 6 and mx[0, 0, 1, 1] == 16
    assert av[0, 0, 0, 0] == 3.5 and av[0, 0, 1, 1] == 13.5
    # window (0,1): rows -1..1, cols 2..4 -> 3,4,7,8
    assert mx[0, 0, 0, 1] == 8 and av[0, 0, 0, 1] == 5.5
    # negative data: the zero border must not win the maximum
    assert po.pooling_forward(po.POOL_MAX, -x, (3, 3), pad=(1, 1), stride=(3, 3))[0, 0, 0, 0] == -1


def test_pooling_against_torch_and_identities():
    torch = pytest.importorskip("torch")
    x = rnd(13, 2, 3, 9, 11)
    xt = torch.tensor(x, dtype=torch.float64)
    for win, pad, st in [((2, 2), (0, 0), (2, 2)), ((3, 3), (1, 1), (2, 2)), ((3, 2), (1, 0), (1, 3)), ((5, 5), (2, 2), (4, 4))]:
        mx = po.pooling_forward(po.POOL_MAX, x, win, pad, st)
        av = po.pooling_forward(po.POOL_AVERAGE, x, win, pad, st)
        assert np.array_equal(mx, torch.nn.functional.max_pool2d(xt, win, st, pad).numpy())
        want = torch.nn.functional.avg_pool2d(xt, win, st, pad, count_include_pad=False).numpy()
        assert np.allclose(av, want, rtol=0, atol=1e-14)
    # a 1x1 window with stride 1 is the identity; a window covering the image is the global max / mean
    assert np.array_equal(po.pooling_forward(po.POOL_MAX, x, (1, 1)), x.astype(np.float64))
    g = po.pooling_forward(po.POOL_AVERAGE, x, (9, 11))
    assert g.shape == (2, 3, 1, 1) and np.allclose(g[..., 0, 0], x.astype(np.float64).mean(axis=(2, 3)), atol=1e-14)
    assert np.array_equal(po.pooling_forward(po.POOL_MAX, nhwc(x), (3, 3), (1, 1), (2, 2), layout="NHWC"),
                          po.pooling_forward(po.POOL_MAX, x, (3, 3), (1, 1), (2, 2)))
    with pytest.raises(ValueError):
        po.pooling_forward(po.POOL_MAX, x, (2, 2), pad=(2, 0))      # pad >= window


# ---------------------------------------------------------------- backward forms of softmax and pooling
def test_softmax_backward_closed_forms():
    # two elements, x = (0, ln 3): y = (1/4, 3/4).  dy = (1, 0): dot = 1/4,
    # dx = (1/4 * (1 - 1/4), 3/4 * (0 - 1/4)) = (3/16, -3/16)
    y = np.array([0.25, 0.75], dtype=np.float32).reshape(1, 2, 1, 1)
    dy = np.array([1.0, 0.0], dtype=np.float32).reshape(1, 2, 1, 1)
    for mode in (po.SOFTMAX_CHANNEL, po.SOFTMAX_INSTANCE):
        assert np.array_equal(po.softmax_backward(mode, y, dy).ravel(), [3 / 16, -3 / 16])
    # the same two numbers along w: one group per image, but single-element groups per location
    yw, dyw = y.reshape(1, 1, 1, 2), dy.reshape(1, 1, 1, 2)
    assert np.array_equal(po.softmax_backward(po.SOFTMAX_INSTANCE, yw, dyw).ravel(), [3 / 16, -3 / 16])
    assert np.array_equal(po.softmax_backward(po.SOFTMAX_CHANNEL, yw, dyw).ravel(), [0.25 * (1 - 0.25), 0.0])
    # a uniform y = 1/n: dx_i = (dy_i - mean(dy)) / n; a constant dy: dx = 0 (y sums to one)
    n = 8
    yu = np.full((2, n, 1, 1), 1.0 / n, dtype=np.float32)
    d = rnd(3, 2, n, 1, 1)
    want = (d.astype(np.float64) - d.astype(np.float64).mean(axis=1, keepdims=True)) / n
    assert np.allclose(po.softmax_backward(po.SOFTMAX_CHANNEL, yu, d), want, rtol=0, atol=1e-15)
    ys = po.softmax_forward(po.SOFTMAX_CHANNEL, rnd(4, 2, 5, 3, 4)).astype(np.float32)
    assert np.max(np.abs(po.softmax_backward(po.SOFTMAX_CHANNEL, ys, np.full_like(ys, 2.5)))) < 1e-6
    # alpha, beta and layouts
    old = rnd(5, 2, 5, 3, 4).astype(np.float64)
    dd = rnd(6, 2, 5, 3, 4)
    raw = po.softmax_backward(po.SOFTMAX_CHANNEL, ys, dd)
    assert np.allclose(po.softmax_backward(po.SOFTMAX_CHANNEL, nhwc(ys), dd, alpha=2.0, beta=-0.5, dx_old=old, layout="NHWC"),
                       2.0 * raw - 0.5 * old, rtol=0, atol=1e-15)


@pytest.mark.parametrize("mode", [po.SOFTMAX_INSTANCE, po.SOFTMAX_CHANNEL])
def test_softmax_backward_is_the_transposed_jacobian_of_forward(mode):
    """Central differences of the (separately pinned) forward function, element by element:
    dx_i = sum_j dy_j * d y_j / d x_i.  Inputs on a 1/64 grid and a step of 1/512 are exact in
    fp32, so the only error is the O(step^2) truncation."""
    rng = np.random.default_rng(11)
    x = (rng.integers(-128, 128, size=(2, 3, 2, 2)) / 64.0).astype(np.float32)
    dy = rnd(12, 2, 3, 2, 2)
    y = po.softmax_forward(mode, x)
    got = po.softmax_backward(mode, y.astype(np.float32), dy)
    eps = 1.0 / 512
    want = np.zeros(x.shape)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        dydx = (po.softmax_forward(mode, xp) - po.softmax_forward(mode, xm)) / (2 * eps)
        want[idx] = np.sum(dydx * dy.astype(np.float64))
    assert np.max(np.abs(got - want)) < 5e-6


def test_pooling_backward_hand_cases():
    x = np.arange(1, 17, dtype=np.float32).reshape(1, 1, 4, 4)
    dy = np.array([[1.0, 2.0], [3.0, 4.0]], dtype=np.float32).reshape(1, 1, 2, 2)
    # 2x2 windows, stride 2: each window's maximum is its bottom-right corner
    mx = po.pooling_backward(po.POOL_MAX, x, dy, (2, 2), stride=(2, 2))[0, 0]
    assert np.array_equal(mx, [[0, 0, 0, 0], [0, 1, 0, 2], [0, 0, 0, 0], [0, 3, 0, 4]])
    av = po.pooling_backward(po.POOL_AVERAGE, x, dy, (2, 2), stride=(2, 2))[0, 0]
    assert np.array_equal(av, np.kron(dy[0, 0], np.ones((2, 2))) / 4)
    # 3x3, pad 1, stride 3 on 4x4: windows (0,0): rows/cols {0,1} (4 elements), (0,1): rows {0,1}, cols {2,3},
    # (1,0): rows {2,3}, cols {0,1}, (1,1): rows/cols {2,3}; maxima at (1,1), (1,3), (3,1), (3,3)
    mx = po.pooling_backward(po.POOL_MAX, x, dy, (3, 3), pad=(1, 1), stride=(3, 3))[0, 0]
    assert np.array_equal(mx, [[0, 0, 0, 0], [0, 1, 0, 2], [0, 0, 0, 0], [0, 3, 0, 4]])
    av = po.pooling_backward(po.POOL_AVERAGE, x, dy, (3, 3), pad=(1, 1), stride=(3, 3))[0, 0]
    assert np.array_equal(av, np.kron(dy[0, 0], np.ones((2, 2))) / 4)
    # overlapping windows (3 wide, stride 1, one row): x = (1, 5, 2, 4): windows {1,5,2} and {5,2,4} both
    # pick the 5; averages: element 0 gets a/3, elements 1,2 get (a+b)/3, element 3 gets b/3
    x1 = np.array([1, 5, 2, 4], dtype=np.float32).reshape(1, 1, 1, 4)
    d1 = np.array([3.0, 6.0], dtype=np.float32).reshape(1, 1, 1, 2)
    assert np.array_equal(po.pooling_backward(po.POOL_MAX, x1, d1, (1, 3)).ravel(), [0, 9, 0, 0])
    assert np.array_equal(po.pooling_backward(po.POOL_AVERAGE, x1, d1, (1, 3)).ravel(), [1, 3, 3, 2])
    # equal maxima: the first in scan order receives the gradient (all-equal data: the top-left in-image element)
    c = np.full((1, 1, 4, 4), 7.0, dtype=np.float32)
    mx = po.pooling_backward(po.POOL_MAX, c, dy, (3, 3), pad=(1, 1), stride=(3, 3))[0, 0]
    assert np.array_equal(mx, [[1, 0, 2, 0], [0, 0, 0, 0], [3, 0, 4, 0], [0, 0, 0, 0]])
    # all-negative data next to the zero border: the border never takes the gradient
    mx = po.pooling_backward(po.POOL_MAX, -x, dy, (3, 3), pad=(1, 1), stride=(3, 3))[0, 0]
    assert np.array_equal(mx, [[1, 0, 2, 0], [0, 0, 0, 0], [3, 0, 4, 0], [0, 0, 0, 0]])


def test_pooling_backward_against_torch_autograd_and_the_transpose_identity():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(21)
    # distinct values (a permutation), so that every maximum is unique
    x = (rng.permutation(2 * 3 * 9 * 11).reshape(2, 3, 9, 11) / 16.0 - 10.0).astype(np.float32)
    for win, pad, st in [((2, 2), (0, 0), (2, 2)), ((3, 3), (1, 1), (2, 2)), ((3, 2), (1, 0), (1, 3)), ((5, 5), (2, 2), (4, 4)),
                         ((3, 3), (0, 0), (1, 1)), ((2, 2), (0, 0), (3, 3))]:
        P, Q = po.pooling_output_dim(9, win[0], pad[0], st[0]), po.pooling_output_dim(11, win[1], pad[1], st[1])
        dy = rnd(22, 2, 3, P, Q)
        for mode in (po.POOL_MAX, po.POOL_AVERAGE):
            xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
            if mode == po.POOL_MAX:
                yt = torch.nn.functional.max_pool2d(xt, win, st, pad)
            else:
                yt = torch.nn.functional.avg_pool2d(xt, win, st, pad, count_include_pad=False)
            yt.backward(torch.tensor(dy, dtype=torch.float64))
            got = po.pooling_backward(mode, x, dy, win, pad, st)
            assert np.allclose(got, xt.grad.numpy(), rtol=0, atol=1e-14), (win, pad, st, mode)
            # every window hands out exactly its gradient
            assert abs(got.sum() - dy.astype(np.float64).sum()) < 1e-10
        # average pooling is linear: <forward(x), dy> = <x, backward(dy)>
        lhs = np.sum(po.pooling_forward(po.POOL_AVERAGE, x, win, pad, st) * dy)
        rhs = np.sum(po.pooling_backward(po.POOL_AVERAGE, x, dy, win, pad, st) * x)
        assert abs(lhs - rhs) < 1e-9
    # elements no window reaches (stride 3, 2x2 windows) get beta * old only
    old = rnd(23, 2, 3, 9, 11).astype(np.float64)
    dy = rnd(24, 2, 3, 3, 4)
    got = po.pooling_backward(po.POOL_MAX, nhwc(x), dy, (2, 2), stride=(3, 3), alpha=2.0, beta=0.5, dx_old=old, layout="NHWC")
    assert np.array_equal(got[:, :, 2::3, :], 0.5 * old[:, :, 2::3, :])
    assert np.allclose(got, 2.0 * po.pooling_backward(po.POOL_MAX, x, dy, (2, 2), stride=(3, 3)) + 0.5 * old, atol=1e-15)


# ---------------------------------------------------------------- double-precision inputs
def test_double_inputs_share_the_arithmetic_and_are_not_truncated():
    """The functions for double inputs are the same bodies compiled for another element type: on
    float32-representable data both forms agree bit for bit, and on data that needs all 53 bits
    they follow scipy / numpy / torch in double (a truncation to float would miss by ~1e-8)."""
    torch = pytest.importorskip("torch")
    from scipy.special import expit, softmax
    x32 = rnd(51, 2, 5, 6, 7)
    d32 = rnd(52, 2, 5, 6, 7)
    x64, d64 = x32.astype(np.float64), d32.astype(np.float64)
    for mode in (po.SIGMOID, po.RELU, po.TANH):
        assert np.array_equal(po.activation_forward(mode, x64), po.activation_forward(mode, x32))
        y32 = po.activation_forward(mode, x32).astype(np.float32)
        assert np.array_equal(po.activation_backward(mode, y32.astype(np.float64), d64, x64), po.activation_backward(mode, y32, d32, x32))
    for mode in (po.SOFTMAX_INSTANCE, po.SOFTMAX_CHANNEL):
        assert np.array_equal(po.softmax_forward(mode, x64), po.softmax_forward(mode, x32))
        y32 = po.softmax_forward(mode, x32).astype(np.float32)
        assert np.array_equal(po.softmax_backward(mode, y32.astype(np.float64), d64), po.softmax_backward(mode, y32, d32))
    for mode in (po.POOL_MAX, po.POOL_AVERAGE):
        assert np.array_equal(po.pooling_forward(mode, x64, (3, 3), (1, 1), (2, 2)), po.pooling_forward(mode, x32, (3, 3), (1, 1), (2, 2)))
        g32 = rnd(53, 2, 5, 3, 4)
        assert np.array_equal(po.pooling_backward(mode, x64, g32.astype(np.float64), (3, 3), (1, 1), (2, 2)),
                              po.pooling_backward(mode, x32, g32, (3, 3), (1, 1), (2, 2)))
    assert np.array_equal(po.add_tensor(x64[:, :, :1, :1], x32.shape, 2.0), po.add_tensor(x32[:, :, :1, :1], x32.shape, 2.0))
    # full-precision data
    x = np.random.default_rng(54).uniform(-3, 3, size=(2, 5, 6, 7))
    assert np.max(np.abs(x - x.astype(np.float32))) > 1e-8
    assert np.allclose(po.activation_forward(po.SIGMOID, x), expit(x), rtol=1e-15, atol=0)
    assert np.allclose(po.activation_forward(po.TANH, x), np.tanh(x), rtol=1e-15, atol=1e-16)
    assert np.array_equal(po.activation_forward(po.RELU, x), np.maximum(x, 0.0))
    assert np.allclose(po.softmax_forward(po.SOFTMAX_CHANNEL, x), softmax(x, axis=1), rtol=1e-14, atol=0)
    xt = torch.tensor(x)
    assert np.array_equal(po.pooling_forward(po.POOL_MAX, x, (3, 3), (1, 1), (2, 2)), torch.nn.functional.max_pool2d(xt, 3, 2, 1).numpy())
    assert np.allclose(po.pooling_forward(po.POOL_AVERAGE, x, (2, 2), stride=(2, 2)), torch.nn.functional.avg_pool2d(xt, 2, 2).numpy(), rtol=1e-15)
    assert np.array_equal(po.add_tensor(x, x.shape), x)
    with pytest.raises(AssertionError):
        po.activation_backward(po.TANH, x, x.astype(np.float32), x)      # one element type per call
