"""Seeded synthetic inputs for the convolution-forward workloads.

This module holds NO convolution arithmetic: it only names the problem shapes and
draws the input arrays.  Both the CPU oracle's tests and the HIP path's tests/bench
take their data from here, so the two sides see identical inputs without sharing
any other code.  Output sizes P, Q are stored as data (they are stated with the
workloads) and are cross-checked by the tests against both implementations.

Distributions per workload: x uniform on the stated interval, filters normal with
the stated standard deviation, optional y prefill uniform[-1,1]; dense tensors, no
sparsity.  Generator: numpy ``default_rng(seed)``, seed = 14100759*10 + index for
x, +100 for w, +200 for the y prefill.
"""
from dataclasses import dataclass, replace
import math

import numpy as np

CONVOLUTION = 0
CROSS_CORRELATION = 1


@dataclass(frozen=True)
class ConvWorkload:
    name: str
    index: int              # 1-based position in the workload list
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    pad_h: int
    pad_w: int
    u: int                  # vertical stride
    v: int                  # horizontal stride
    P: int
    Q: int
    dtype: str              # "f32" or "bf16" (inputs; output is always f32)
    x_layout: str           # "NCHW" or "NHWC": memory order behind the logical NCHW view
    y_layout: str
    x_dist: tuple           # ("uniform", lo, hi)
    w_std: float            # filters ~ normal(0, w_std)
    alpha: float = 1.0
    beta: float = 0.0
    mode: int = CROSS_CORRELATION

    @property
    def flops(self) -> int:
        """2 * N*K*P*Q*C*R*S (multiply-adds against the zero border included)."""
        return 2 * self.N * self.K * self.P * self.Q * self.C * self.R * self.S

    @property
    def algorithmic_bytes(self) -> int:
        """x once + w once + y written once (+ y read once when beta != 0)."""
        e = 4 if self.dtype == "f32" else 2
        xb = self.N * self.C * self.H * self.W * e
        wb = self.K * self.C * self.R * self.S * e
        yb = self.N * self.K * self.P * self.Q * 4
        return xb + wb + yb * (2 if self.beta != 0.0 else 1)


def _he(C, R, S):
    return math.sqrt(2.0 / (C * R * S))


WORKLOADS = (
    ConvWorkload("cfg1_tiny_f32", 1, 1, 3, 32, 32, 16, 3, 3, 1, 1, 1, 1, 32, 32,
                 "f32", "NCHW", "NCHW", ("uniform", -1.0, 1.0), None),
    ConvWorkload("cfg2_first_layer_11x11_s4_f32", 2, 64, 3, 227, 227, 96, 11, 11, 0, 0, 4, 4, 55, 55,
                 "f32", "NCHW", "NCHW", ("uniform", 0.0, 1.0), 0.01),
    ConvWorkload("cfg3_mid_layer_3x3_f32", 3, 128, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 56, 56,
                 "f32", "NCHW", "NCHW", ("uniform", -1.0, 1.0), _he(64, 3, 3)),
    ConvWorkload("cfg4_deep_3x3_f32_beta1", 4, 128, 384, 13, 13, 256, 3, 3, 1, 1, 1, 1, 13, 13,
                 "f32", "NCHW", "NCHW", ("uniform", -1.0, 1.0), _he(384, 3, 3), beta=1.0),
    ConvWorkload("cfg5_bf16_nhwc_3x3", 5, 32, 512, 14, 14, 512, 3, 3, 1, 1, 1, 1, 14, 14,
                 "bf16", "NHWC", "NHWC", ("uniform", -1.0, 1.0), _he(512, 3, 3)),
)


# The paper's own layer collection (Table 2: "Convolutional layer collection"; N = 128, unit
# stride, no padding), with synthetic data of the same recipe as the mid-layer workloads:
# x uniform[-1,1], w normal(0, sqrt(2/(C*R*S))).  Indices 11..15 keep their seeds apart.
def _table2(i, C, HW, K, RS):
    P = HW - RS + 1
    return ConvWorkload("table2_layer%d" % i, 10 + i, 128, C, HW, HW, K, RS, RS, 0, 0, 1, 1, P, P,
                        "f32", "NCHW", "NCHW", ("uniform", -1.0, 1.0), _he(C, RS, RS))


TABLE2_LAYERS = (
    _table2(1, 3, 128, 96, 11),
    _table2(2, 96, 64, 128, 9),
    _table2(3, 128, 32, 128, 9),
    _table2(4, 128, 16, 128, 7),
    _table2(5, 128, 13, 384, 3),
)
# What the paper reports for them (Table 3, TFLOP/s; hardware of 2014, context only).
TABLE3_PAPER_TFLOPS = {
    "K40 (peak 4.29)": (0.99, 1.52, 1.51, 1.38, 1.01),
    "GTX 980 (peak 4.95)": (1.46, 2.49, 2.42, 2.19, 1.87),
}


def by_index(i: int) -> ConvWorkload:
    return WORKLOADS[i - 1]


def shrink(wl: ConvWorkload, N: int) -> ConvWorkload:
    """Same layer with another number of images (every image is independent)."""
    return replace(wl, N=N, name="%s_N%d" % (wl.name, N))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32
    holding exactly representable bf16 values.  Data preparation only."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that already are bf16-representable."""
    bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(bits & 0xFFFF), "values are not bf16-representable"
    return (bits >> 16).astype(np.uint16).reshape(a.shape)


def with_layout(a: np.ndarray, layout: str) -> np.ndarray:
    """Return a logically-NCHW view of ``a`` whose memory order is ``layout``."""
    if layout == "NCHW":
        return np.ascontiguousarray(a)
    if layout == "NHWC":
        return np.ascontiguousarray(a.transpose(0, 2, 3, 1)).transpose(0, 3, 1, 2)
    raise ValueError(layout)


def make_inputs(wl: ConvWorkload):
    """Returns (x, w, y_prefill): float32 arrays with logical shapes (N,C,H,W),
    (K,C,R,S), (N,K,P,Q), x and y_prefill laid out in memory as the workload says
    (w is always packed K,C,R,S).  y_prefill is None when beta == 0.  For "bf16"
    workloads x and w are already rounded to bf16-representable values."""
    base = 14100759 * 10 + wl.index
    kind, lo, hi = wl.x_dist
    assert kind == "uniform"
    x = np.random.default_rng(base).uniform(lo, hi, size=(wl.N, wl.C, wl.H, wl.W)).astype(np.float32)
    rw = np.random.default_rng(base + 100)
    if wl.w_std is None:
        w = rw.uniform(-1.0, 1.0, size=(wl.K, wl.C, wl.R, wl.S)).astype(np.float32)
    else:
        w = (rw.standard_normal(size=(wl.K, wl.C, wl.R, wl.S)) * wl.w_std).astype(np.float32)
    if wl.dtype == "bf16":
        x, w = round_to_bf16(x), round_to_bf16(w)
    y0 = None
    if wl.beta != 0.0:
        y0 = np.random.default_rng(base + 200).uniform(
            -1.0, 1.0, size=(wl.N, wl.K, wl.P, wl.Q)).astype(np.float32)
        y0 = with_layout(y0, wl.y_layout)
    return with_layout(x, wl.x_layout), np.ascontiguousarray(w), y0


def random_problem(seed: int, N, C, H, W, K, R, S, x_layout="NCHW", dtype="f32"):
    """Small seeded problem for sweeps: x uniform[-1,1], w normal(0, sqrt(2/(CRS)))."""
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1.0, 1.0, size=(N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal(size=(K, C, R, S)) * _he(C, R, S)).astype(np.float32)
    if dtype == "bf16":
        x, w = round_to_bf16(x), round_to_bf16(w)
    return with_layout(x, x_layout), w
