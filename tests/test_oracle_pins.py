"""Pins for the CPU oracle: it is checked against what the paper and the mathematics
fix, never against itself or against the HIP path.

Each test names the passage it comes from.  A plausible mistake in the oracle (a
dropped term, a wrong sign in eq. 2, swapped r/s, a transposed stride, pad applied
on one side only, u and v swapped) fails at least one of these.
"""
import json
import os

import numpy as np
import pytest

from oracle import conv_oracle as oc
from oracle import lowering as low
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
CONV, XCORR = oc.CONVOLUTION, oc.CROSS_CORRELATION


def rnd(seed, *shape):
    return np.random.default_rng(seed).uniform(-1, 1, size=shape).astype(np.float32)


# ---------------------------------------------------------------- hand-worked cases
with open(os.path.join(GOLDEN, "hand_cases.json")) as fh:
    HAND = json.load(fh)["cases"]


@pytest.mark.parametrize("case", HAND, ids=[c["name"] for c in HAND])
def test_hand_computed_cases(case):
    """eq. 1-3 worked by hand (tests/golden/hand_cases.json)."""
    x = np.array(case["x"], dtype=np.float32)
    w = np.array(case["w"], dtype=np.float32)
    want = np.array(case["y"], dtype=np.float64)
    got = oc.conv_forward(x, w, pad=tuple(case["pad"]), stride=tuple(case["stride"]), mode=case["mode"])
    assert got.shape == want.shape
    assert np.array_equal(got, want)
    # the lowering derivation must agree with the same hand values
    got2, _, _ = low.conv_forward_lowered(x, w, tuple(case["pad"]), tuple(case["stride"]), case["mode"])
    assert np.array_equal(got2, want)


# ---------------------------------------------------------------- eq. 1
def test_output_dim_closed_form():
    """eq. 1's ceiling equals floor((H + 2 pad - R)/u) + 1 whenever H + 2 pad - R >= 0."""
    rng = np.random.default_rng(1)
    for _ in range(5000):
        H, R, u, pad = (int(rng.integers(1, 300)), int(rng.integers(1, 13)),
                        int(rng.integers(1, 6)), int(rng.integers(0, 7)))
        if H + 2 * pad - R < 0:
            assert oc.output_dim(H, R, u, pad) <= 0
            continue
        assert oc.output_dim(H, R, u, pad) == (H + 2 * pad - R) // u + 1


def test_output_dim_matlab_modes():
    """Section 2.1.1: valid (pad 0), same (pad floor(R/2), odd R), full (pad R-1)."""
    for H in (5, 13, 32, 227):
        for R in (1, 3, 5, 11):
            if R > H:
                continue
            assert oc.output_dim(H, R, 1, 0) == H - R + 1
            assert oc.output_dim(H, R, 1, R // 2) == H
            assert oc.output_dim(H, R, 1, R - 1) == H + R - 1


def test_workload_output_dims():
    """P, Q stored with the workloads equal eq. 1."""
    for w_ in wl.WORKLOADS + wl.TABLE2_LAYERS:
        assert oc.output_dim(w_.H, w_.R, w_.u, w_.pad_h) == w_.P
        assert oc.output_dim(w_.W, w_.S, w_.v, w_.pad_w) == w_.Q


# ---------------------------------------------------------------- special cases with a textbook form
def test_1x1_is_a_gemm():
    """R = S = 1, unit stride, no padding: O_m = F_m (K x C) . D (C x N*H*W)."""
    x, w = rnd(2, 3, 5, 6, 7), rnd(3, 4, 5, 1, 1)
    for mode in (CONV, XCORR):
        y = oc.conv_forward(x, w, mode=mode)
        Wm = w.reshape(4, 5).astype(np.float64)
        Xm = x.astype(np.float64).transpose(1, 0, 2, 3).reshape(5, -1)
        want = (Wm @ Xm).reshape(4, 3, 6, 7).transpose(1, 0, 2, 3)
        np.testing.assert_allclose(y, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("mode", [CONV, XCORR])
def test_centred_delta_reproduces_channel(mode):
    """Odd R,S, pad floor(R/2): a filter that is 1 at the centre of channel c0
    copies that channel (eq. 2 maps the centre tap to (p,q) in both modes)."""
    x = rnd(4, 2, 3, 8, 9)
    w = np.zeros((3, 3, 3, 5), dtype=np.float32)
    for k, c0 in enumerate((2, 0, 1)):
        w[k, c0, 1, 2] = 1.0
    y = oc.conv_forward(x, w, pad=(1, 2), mode=mode)
    for k, c0 in enumerate((2, 0, 1)):
        assert np.array_equal(y[:, k], x[:, c0].astype(np.float64))


def test_offcentre_delta_shift_direction_distinguishes_modes():
    """A tap at (r,s) = (0,0) of a 3x3 filter, pad 1: cross-correlation reads
    x[p-1,q-1]; eq. 2 reads x[p+1,q+1]."""
    x = rnd(5, 1, 1, 6, 7)
    w = np.zeros((1, 1, 3, 3), dtype=np.float32)
    w[0, 0, 0, 0] = 1.0
    xd = x.astype(np.float64)[0, 0]
    yx = oc.conv_forward(x, w, pad=(1, 1), mode=XCORR)[0, 0]
    yc = oc.conv_forward(x, w, pad=(1, 1), mode=CONV)[0, 0]
    want_x = np.zeros_like(xd)
    want_x[1:, 1:] = xd[:-1, :-1]
    want_c = np.zeros_like(xd)
    want_c[:-1, :-1] = xd[1:, 1:]
    assert np.array_equal(yx, want_x)
    assert np.array_equal(yc, want_c)


def test_conv_equals_xcorr_with_flipped_filter():
    x, w = rnd(6, 2, 3, 9, 8), rnd(7, 4, 3, 3, 2)
    a = oc.conv_forward(x, w, pad=(2, 1), stride=(2, 1), mode=CONV)
    b = oc.conv_forward(x, w[:, :, ::-1, ::-1].copy(), pad=(2, 1), stride=(2, 1), mode=XCORR)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


@pytest.mark.parametrize("mode", [CONV, XCORR])
def test_linearity(mode):
    """eq. 3 is linear in D and in F."""
    x1, x2 = rnd(8, 2, 3, 7, 7), rnd(9, 2, 3, 7, 7)
    w1, w2 = rnd(10, 3, 3, 3, 3), rnd(11, 3, 3, 3, 3)
    a, b = 2.0, -0.5
    f = lambda x, w: oc.conv_forward(x, w, pad=(1, 1), stride=(1, 2), mode=mode)
    # the oracle takes fp32 inputs, so the combined input is rounded once to fp32:
    # that rounding (<= 2^-24 * 2.5 per element, 27 taps of |w| <= 1) bounds the gap
    xs32 = (a * x1.astype(np.float64) + b * x2.astype(np.float64)).astype(np.float32)
    lhs = f(xs32, w1)
    rhs = a * f(x1, w1) + b * f(x2, w1)
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=5e-6)
    # exact version: scale by powers of two only
    np.testing.assert_allclose(f(4.0 * x1, w1), 4.0 * f(x1, w1), rtol=0, atol=0)
    # additivity with disjoint supports is exact: x1 masked to even columns, x2 to odd
    m = np.zeros_like(x1)
    m[..., ::2] = 1
    xa, xb = x1 * m, x1 * (1 - m)
    np.testing.assert_allclose(f(xa, w1) + f(xb, w1), f(x1, w1), rtol=0, atol=1e-13)
    wa, wb = w1.copy(), w1.copy()
    wa[:, :, :, 1:] = 0
    wb[:, :, :, :1] = 0
    np.testing.assert_allclose(f(x1, wa) + f(x1, wb), f(x1, w1), rtol=0, atol=1e-13)
    np.testing.assert_allclose(f(x1, 0.25 * w2), 0.25 * f(x1, w2), rtol=0, atol=0)


@pytest.mark.parametrize("mode", [CONV, XCORR])
def test_padding_identity(mode):
    """D0 is D extended by zeros: pad (a,b) == pad 0 on an explicitly padded copy."""
    x, w = rnd(12, 2, 2, 6, 5), rnd(13, 3, 2, 3, 2)
    a, b = 2, 1
    xp = np.zeros((2, 2, 6 + 2 * a, 5 + 2 * b), dtype=np.float32)
    xp[:, :, a:a + 6, b:b + 5] = x
    y1 = oc.conv_forward(x, w, pad=(a, b), stride=(1, 2), mode=mode)
    y2 = oc.conv_forward(xp, w, pad=(0, 0), stride=(1, 2), mode=mode)
    assert np.array_equal(y1, y2)


@pytest.mark.parametrize("mode", [CONV, XCORR])
def test_stride_identity(mode):
    """Strides compute a subset of the unit-stride outputs: y_uv == y_11[::u, ::v].
    (Section 2.1.1; for eq. 2 this needs the same R-1-r offset in both, which holds
    when the strided grid starts at output 0.)"""
    x, w = rnd(14, 1, 2, 11, 12), rnd(15, 2, 2, 3, 4)
    full = oc.conv_forward(x, w, pad=(1, 2), mode=mode)
    for u, v in ((2, 1), (1, 3), (3, 2)):
        sub = oc.conv_forward(x, w, pad=(1, 2), stride=(u, v), mode=mode)
        assert np.array_equal(sub, full[:, :, ::u, ::v])


# ---------------------------------------------------------------- lowering (Section 3, Fig. 1)
def test_fig1_lowering_shapes_and_agreement():
    with open(os.path.join(GOLDEN, "fig1_shapes.json")) as fh:
        g = json.load(fh)
    pr = g["problem"]
    x = np.arange(1, 1 + pr["C"] * 9, dtype=np.float32).reshape(1, pr["C"], 3, 3)
    w = rnd(16, pr["K"], pr["C"], pr["R"], pr["S"])
    y, Fm, Dm = low.conv_forward_lowered(x, w, mode=XCORR)
    assert list(Fm.shape) == g["F_m_shape"]
    assert list(Dm.shape) == g["D_m_shape"]
    assert list(y.reshape(pr["K"], -1).shape) == g["O_m_shape"]
    # every input element is distinct here, so duplication can be counted
    _, counts = np.unique(Dm, return_counts=True)
    assert counts.max() == g["max_duplication"]       # "up to RS = 4 times"
    np.testing.assert_allclose(oc.conv_forward(x, w, mode=XCORR), y, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_lowering_cross_oracle_random(seed):
    rng = np.random.default_rng(100 + seed)
    N, C, K = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
    R, S = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    H, W = int(rng.integers(R, R + 6)), int(rng.integers(S, S + 6))
    pad = (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
    stride = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
    x, w = rnd(200 + seed, N, C, H, W), rnd(300 + seed, K, C, R, S)
    for mode in (CONV, XCORR):
        y2, _, _ = low.conv_forward_lowered(x, w, pad, stride, mode)
        y1 = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode)
        np.testing.assert_allclose(y1, y2, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- alpha / beta
def test_alpha_beta_and_write_only_y():
    x, w = rnd(17, 2, 3, 6, 6), rnd(18, 4, 3, 3, 3)
    y0 = rnd(19, 2, 4, 6, 6)
    base = oc.conv_forward(x, w, pad=(1, 1))
    got = oc.conv_forward(x, w, pad=(1, 1), alpha=0.75, beta=-2.0, y_old=y0)
    np.testing.assert_allclose(got, 0.75 * base - 2.0 * y0.astype(np.float64), rtol=0, atol=1e-14)
    acc = oc.conv_forward(x, w, pad=(1, 1), alpha=1.0, beta=1.0, y_old=y0)
    np.testing.assert_allclose(acc, base + y0, rtol=0, atol=1e-14)
    # beta == 0: y_old is never read, NaN in it cannot leak
    nan = np.full_like(y0, np.nan)
    assert np.array_equal(oc.conv_forward(x, w, pad=(1, 1), beta=0.0, y_old=nan), base)
    # alpha == 0 still writes beta * y_old
    z = oc.conv_forward(x, w, pad=(1, 1), alpha=0.0, beta=3.0, y_old=y0)
    assert np.array_equal(z, 3.0 * y0.astype(np.float64))


# ---------------------------------------------------------------- strides / layouts
def test_layout_invariance():
    """Section 2.1.1: user-defined strides; interleaved (NHWC) vs separate (NCHW)
    feature maps, padded pitch, channel-slice views give the same logical tensor."""
    x, w = rnd(20, 2, 4, 6, 5), rnd(21, 3, 4, 3, 3)
    ref = oc.conv_forward(x, w, pad=(1, 0), stride=(1, 2))
    x_nhwc = wl.with_layout(x, "NHWC")
    assert x_nhwc.strides != x.strides
    assert np.array_equal(oc.conv_forward(x_nhwc, w, pad=(1, 0), stride=(1, 2)), ref)
    assert np.array_equal(oc.conv_forward(x, w, pad=(1, 0), stride=(1, 2), y_layout="NHWC"), ref)
    pitched = np.full((2, 4, 6, 9), 7.0, dtype=np.float32)
    pitched[..., :5] = x
    assert np.array_equal(oc.conv_forward(pitched[..., :5], w, pad=(1, 0), stride=(1, 2)), ref)
    big = np.full((2, 7, 6, 5), -3.0, dtype=np.float32)
    big[:, 2:6] = x
    assert np.array_equal(oc.conv_forward(big[:, 2:6], w, pad=(1, 0), stride=(1, 2)), ref)
    # a transposed (H<->W swapped strides) view is a different logical tensor
    xt = np.ascontiguousarray(x.transpose(0, 1, 3, 2)).transpose(0, 1, 3, 2)
    assert np.array_equal(oc.conv_forward(xt, w, pad=(1, 0), stride=(1, 2)), ref)


def test_group_convolution_by_channel_slices():
    """Group convolution as the framework does it: several calls on channel slices."""
    x, w = rnd(22, 1, 4, 5, 5), rnd(23, 4, 2, 3, 3)   # 2 groups: 2 in-channels -> 2 filters each
    y0 = oc.conv_forward(x[:, 0:2], w[0:2], pad=(1, 1))
    y1 = oc.conv_forward(x[:, 2:4], w[2:4], pad=(1, 1))
    wfull = np.zeros((4, 4, 3, 3), dtype=np.float32)
    wfull[0:2, 0:2] = w[0:2]
    wfull[2:4, 2:4] = w[2:4]
    yfull = oc.conv_forward(x, wfull, pad=(1, 1))
    np.testing.assert_allclose(np.concatenate([y0, y1], axis=1), yfull, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- zero-border count
def test_all_ones_counts_inbounds_taps():
    """x = 1, w = 1: every output equals C * (#taps inside the image), a closed form
    per (p,q): rows_in(p) * cols_in(q)."""
    C, H, W, R, S = 3, 7, 6, 3, 4
    x = np.ones((1, C, H, W), dtype=np.float32)
    w = np.ones((2, C, R, S), dtype=np.float32)
    for pad, stride in (((0, 0), (1, 1)), ((1, 2), (1, 1)), ((2, 3), (2, 3))):
        for mode in (CONV, XCORR):
            y = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode)
            P, Q = y.shape[2:]
            for p in range(P):
                lo = p * stride[0] - pad[0]
                rows = len([h for h in range(lo, lo + R) if 0 <= h < H])
                for q in range(Q):
                    lo2 = q * stride[1] - pad[1]
                    cols = len([c for c in range(lo2, lo2 + S) if 0 <= c < W])
                    assert y[0, 0, p, q] == C * rows * cols
                    assert y[0, 1, p, q] == C * rows * cols


# ---------------------------------------------------------------- library routines the special cases reduce to
def test_against_scipy_correlate_and_convolve():
    from scipy.signal import convolve2d, correlate2d
    x, w = rnd(24, 1, 3, 9, 8), rnd(25, 2, 3, 3, 4)
    yx = oc.conv_forward(x, w, mode=XCORR)
    yc = oc.conv_forward(x, w, mode=CONV)
    for k in range(2):
        cx = sum(correlate2d(x[0, c].astype(np.float64), w[k, c].astype(np.float64), mode="valid") for c in range(3))
        cc = sum(convolve2d(x[0, c].astype(np.float64), w[k, c].astype(np.float64), mode="valid") for c in range(3))
        np.testing.assert_allclose(yx[0, k], cx, rtol=0, atol=1e-13)
        np.testing.assert_allclose(yc[0, k], cc, rtol=0, atol=1e-13)
    # "full" mode: pad R-1, S-1 (Section 2.1.1) is scipy's mode="full"
    yfull = oc.conv_forward(x, w, pad=(2, 3), mode=CONV)
    for k in range(2):
        cf = sum(convolve2d(x[0, c].astype(np.float64), w[k, c].astype(np.float64), mode="full") for c in range(3))
        np.testing.assert_allclose(yfull[0, k], cf, rtol=0, atol=1e-13)


def test_against_torch_cpu_conv2d_fp64():
    import torch
    x, w = rnd(26, 2, 5, 12, 10), rnd(27, 6, 5, 3, 5)
    got = oc.conv_forward(x, w, pad=(2, 1), stride=(2, 3), mode=XCORR)
    want = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                      stride=(2, 3), padding=(2, 1)).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_rejects_bad_problems():
    x, w = rnd(28, 1, 1, 3, 3), rnd(29, 1, 1, 5, 5)
    with pytest.raises(ValueError):
        oc.conv_forward(x, w)            # filter larger than padded image: no output
    with pytest.raises(ValueError):
        oc.conv_forward(x, rnd(30, 1, 1, 2, 2), beta=1.0)  # beta without y_old
