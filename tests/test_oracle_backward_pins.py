"""Pins for the backward forms of the CPU oracle (derivatives of the forward form of
Section 2.1.1 with respect to the input and to the filters).

They are pinned to things other than themselves: hand-worked cases, the transpose
identity against the (separately pinned) forward oracle, finite differences of the
forward oracle, the 1x1 case as two matrix products, and PyTorch's CPU autograd in
fp64 as an independent library.  A wrong sign or index, r and s swapped, the mode
ignored, pad or stride on one axis only, or a transposed (k,c) fails several of them.
"""
import json
import os

import numpy as np
import pytest

from oracle import conv_oracle as oc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
CONV, XCORR = oc.CONVOLUTION, oc.CROSS_CORRELATION

with open(os.path.join(GOLDEN, "hand_cases_backward.json")) as fh:
    HAND = json.load(fh)["cases"]


def rnd(seed, *shape):
    return np.random.default_rng(seed).uniform(-1, 1, size=shape).astype(np.float32)


PROBLEMS = [
    # N, C, H, W, K, R, S, pad, stride
    (2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1)),
    (1, 2, 9, 8, 3, 3, 2, (0, 1), (2, 1)),
    (2, 2, 10, 11, 2, 5, 3, (2, 0), (3, 2)),    # stride leaves input rows unused
    (1, 4, 5, 5, 5, 1, 1, (0, 0), (1, 1)),
    (1, 1, 6, 9, 2, 2, 4, (1, 3), (2, 3)),      # "full"-like padding, even filter sizes
    (3, 2, 4, 4, 2, 4, 4, (3, 3), (1, 1)),
]


@pytest.mark.parametrize("case", HAND, ids=[c["name"] for c in HAND])
def test_hand_computed_cases(case):
    x = np.array(case["x"], dtype=np.float32)
    w = np.array(case["w"], dtype=np.float32)
    dy = np.array(case["dy"], dtype=np.float32)
    pad, stride, mode = tuple(case["pad"]), tuple(case["stride"]), case["mode"]
    dx = oc.conv_backward_data(dy, w, x.shape[2:], pad=pad, stride=stride, mode=mode)
    dw = oc.conv_backward_filter(x, dy, w.shape[2:], pad=pad, stride=stride, mode=mode)
    assert np.array_equal(dx, np.array(case["dx"], dtype=np.float64))
    assert np.array_equal(dw, np.array(case["dw"], dtype=np.float64))


@pytest.mark.parametrize("mode", [CONV, XCORR])
@pytest.mark.parametrize("prob", PROBLEMS, ids=[str(i) for i in range(len(PROBLEMS))])
def test_transpose_identity_against_forward(prob, mode):
    """<conv(x,w), dy> = <x, backward_data(dy,w)> = <w, backward_filter(x,dy)>: the forward
    map is linear in x and in w, and the backward forms are its transposes."""
    N, C, H, W, K, R, S, pad, stride = prob
    x, w = rnd(1, N, C, H, W), rnd(2, K, C, R, S)
    y = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode)
    dy = rnd(3, *y.shape)
    lhs = float(np.sum(y * dy))
    dx = oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride, mode=mode)
    dw = oc.conv_backward_filter(x, dy, (R, S), pad=pad, stride=stride, mode=mode)
    assert dx.shape == x.shape and dw.shape == w.shape
    assert abs(lhs - float(np.sum(dx * x))) <= 1e-10 * max(1.0, abs(lhs))
    assert abs(lhs - float(np.sum(dw * w))) <= 1e-10 * max(1.0, abs(lhs))


@pytest.mark.parametrize("mode", [CONV, XCORR])
def test_every_element_by_unit_perturbation(mode):
    """Element by element: dx[e] is the change of <conv(x,w), dy> when x[e] grows by one
    (the map is linear, so the difference is exact up to rounding), likewise dw."""
    N, C, H, W, K, R, S, pad, stride = 1, 2, 5, 4, 2, 3, 2, (1, 0), (2, 1)
    x, w = rnd(4, N, C, H, W), rnd(5, K, C, R, S)
    y0 = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode)
    dy = rnd(6, *y0.shape)
    base = float(np.sum(y0 * dy))
    dx = oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride, mode=mode)
    dw = oc.conv_backward_filter(x, dy, (R, S), pad=pad, stride=stride, mode=mode)
    for idx in np.ndindex(*x.shape):
        xp = x.copy()
        xp[idx] += 1.0
        d = float(np.sum(oc.conv_forward(xp, w, pad=pad, stride=stride, mode=mode) * dy)) - base
        assert abs(d - dx[idx]) < 1e-5, (idx, d, dx[idx])
    for idx in np.ndindex(*w.shape):
        wp = w.copy()
        wp[idx] += 1.0
        d = float(np.sum(oc.conv_forward(x, wp, pad=pad, stride=stride, mode=mode) * dy)) - base
        assert abs(d - dw[idx]) < 1e-5, (idx, d, dw[idx])


def test_1x1_is_two_matrix_products():
    """R=S=1, u=v=1, pad 0: y_n = W @ x_n, so dx_n = W^T @ dy_n and dW = sum_n dy_n @ x_n^T."""
    N, C, H, W, K = 3, 5, 4, 6, 7
    x, w, dy = rnd(7, N, C, H, W), rnd(8, K, C, 1, 1), rnd(9, N, K, H, W)
    Wm = w.reshape(K, C).astype(np.float64)
    dx = oc.conv_backward_data(dy, w, (H, W))
    dw = oc.conv_backward_filter(x, dy, (1, 1))
    want_dw = np.zeros((K, C))
    for n in range(N):
        dyn = dy[n].reshape(K, H * W).astype(np.float64)
        assert np.allclose(dx[n].reshape(C, H * W), Wm.T @ dyn, rtol=0, atol=1e-12)
        want_dw += dyn @ x[n].reshape(C, H * W).astype(np.float64).T
    assert np.allclose(dw.reshape(K, C), want_dw, rtol=0, atol=1e-12)


def test_unused_input_rows_get_no_gradient():
    """(H + 2 pad - R) not divisible by u: the last input rows are never read by the
    forward loop (eq. 1 rounds the output size), so their derivative is zero."""
    x_shape = (1, 1, 8, 8)   # R=3, u=3, pad 0: P = 2, rows 0..5 used, rows 6, 7 unused
    w, dy = rnd(10, 1, 1, 3, 3), rnd(11, 1, 1, 2, 2)
    dx = oc.conv_backward_data(dy, w, x_shape[2:], stride=(3, 3))
    assert np.all(dx[..., 6:, :] == 0) and np.all(dx[..., :, 6:] == 0) and np.any(dx[..., :6, :6] != 0)


def test_alpha_beta_accumulate_mode():
    """Raw or accumulated results (Section 2.1.1, last paragraph): out = alpha*raw + beta*old;
    beta = 0 never reads the old buffer."""
    N, C, H, W, K, R, S, pad, stride = PROBLEMS[1]
    x, w = rnd(12, N, C, H, W), rnd(13, K, C, R, S)
    P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
    dy = rnd(14, N, K, P, Q)
    dx_raw = oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride)
    dw_raw = oc.conv_backward_filter(x, dy, (R, S), pad=pad, stride=stride)
    dx_old, dw_old = rnd(15, N, C, H, W), rnd(16, K, C, R, S)
    dx = oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride, alpha=0.5, beta=-2.0, dx_old=dx_old)
    dw = oc.conv_backward_filter(x, dy, (R, S), pad=pad, stride=stride, alpha=0.5, beta=-2.0, dw_old=dw_old)
    assert np.allclose(dx, 0.5 * dx_raw - 2.0 * dx_old, rtol=0, atol=1e-13)
    assert np.allclose(dw, 0.5 * dw_raw - 2.0 * dw_old, rtol=0, atol=1e-13)
    with pytest.raises(ValueError):
        oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride, beta=1.0)


def test_layout_invariance():
    """NCHW or NHWC memory order of dy, x and dx (Section 2.1.1: arbitrary strides) gives the
    same logical tensors."""
    N, C, H, W, K, R, S, pad, stride = PROBLEMS[0]
    x, w = rnd(17, N, C, H, W), rnd(18, K, C, R, S)
    dy = rnd(19, N, K, H, W)
    nhwc = lambda a: np.ascontiguousarray(a.transpose(0, 2, 3, 1)).transpose(0, 3, 1, 2)
    dx = oc.conv_backward_data(dy, w, (H, W), pad=pad)
    assert np.array_equal(dx, oc.conv_backward_data(nhwc(dy), w, (H, W), pad=pad, dx_layout="NHWC"))
    dw = oc.conv_backward_filter(x, dy, (R, S), pad=pad)
    assert np.array_equal(dw, oc.conv_backward_filter(nhwc(x), nhwc(dy), (R, S), pad=pad))


@pytest.mark.parametrize("mode", [CONV, XCORR])
def test_against_torch_cpu_autograd_fp64(mode):
    """Independent library (not authoritative): torch's conv2d is a cross-correlation, so
    eq. 2's form is obtained by turning the filter by 180 degrees on the way in and out."""
    torch = pytest.importorskip("torch")
    for N, C, H, W, K, R, S, pad, stride in PROBLEMS:
        x, w = rnd(20, N, C, H, W), rnd(21, K, C, R, S)
        P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
        dy = rnd(22, N, K, P, Q)
        xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
        wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
        weff = wt.flip(2, 3) if mode == CONV else wt
        y = torch.nn.functional.conv2d(xt, weff, stride=stride, padding=pad)
        y.backward(torch.tensor(dy, dtype=torch.float64))
        dx = oc.conv_backward_data(dy, w, (H, W), pad=pad, stride=stride, mode=mode)
        dw = oc.conv_backward_filter(x, dy, (R, S), pad=pad, stride=stride, mode=mode)
        assert np.allclose(dx, xt.grad.numpy(), rtol=0, atol=1e-12)
        assert np.allclose(dw, wt.grad.numpy(), rtol=0, atol=1e-12)


def test_rejects_bad_problems():
    w, dy = rnd(23, 2, 2, 3, 3), rnd(24, 1, 2, 4, 4)
    with pytest.raises(ValueError):
        oc.conv_backward_data(dy, w, (7, 6))            # (7,6) does not give 4x4 outputs
    with pytest.raises(ValueError):
        oc.conv_backward_filter(rnd(25, 1, 2, 7, 6), dy, (3, 3))
