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
