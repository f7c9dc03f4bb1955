"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Bar: max|gpu - oracle| / max|oracle| <= 2e-5 for
fp32 and <= 1e-2 for bf16 inputs (the oracle consumes the already-rounded bf16 values).
"""
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


def _check(x, w, pad, stride, mode, dtype, alpha=1.0, beta=0.0, y0=None, y_layout="NCHW", kernel=None,
           tag=""):
    gu = _gpu()
    print("case", tag, x.shape, w.shape, pad, stride, mode, dtype, alpha, beta, y_layout, "kernel", kernel,
          flush=True)
    got, plan = gu.run(x, w, pad, stride, mode, alpha, beta, y0, dtype, y_layout, kernel)
    want = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode, alpha=alpha, beta=beta, y_old=y0)
    assert got.shape == want.shape
    assert np.all(np.isfinite(got)), "non-finite output (NaN prefill leaked or garbage)"
    err = gu.rel_err(got, want)
    assert err <= gu.BOUND[dtype], "rel err %.3g > %.3g (kernel %d)" % (err, gu.BOUND[dtype], plan.kernelId)
    return err, plan


# ------------------------------------------------------------------ small sweep, heuristic kernel choice
SWEEP = [
    # N, C, H, W, K, R, S, pad, stride
    (1, 1, 5, 5, 1, 1, 1, (0, 0), (1, 1)),
    (2, 3, 9, 11, 5, 3, 3, (1, 1), (1, 1)),
    (3, 5, 17, 19, 37, 3, 2, (1, 0), (1, 1)),
    (2, 4, 23, 21, 70, 5, 5, (2, 2), (2, 2)),
    (1, 3, 35, 35, 96, 11, 11, (0, 0), (4, 4)),
    (2, 7, 12, 40, 33, 1, 7, (0, 3), (1, 3)),
    (5, 9, 13, 13, 130, 3, 3, (1, 1), (1, 1)),
    (2, 2, 8, 8, 4, 4, 4, (3, 3), (1, 1)),      # "full" padding
    (1, 6, 30, 7, 20, 7, 1, (3, 0), (2, 1)),
    (4, 16, 14, 14, 64, 3, 3, (1, 1), (1, 1)),
]


@pytest.mark.parametrize("mode", [0, 1], ids=["conv", "xcorr"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SWEEP, ids=[str(i) for i in range(len(SWEEP))])
def test_small_sweep(shape, dtype, mode):
    N, C, H, W, K, R, S, pad, stride = shape
    x, w = wl.random_problem(1000 + hash(shape) % 1000, N, C, H, W, K, R, S, dtype=dtype)
    _check(x, w, pad, stride, mode, dtype, tag="sweep")


# ------------------------------------------------------------------ every kernel in the table
def _kernel_cases():
    # (dtype, needs CRS % vec == 0)
    import paper_1410_0759_amd as ig
    out = []
    for kid, name in enumerate(ig.kernel_names()):
        out.append((kid, name))
    return out


def _names():
    import paper_1410_0759_amd as ig
    return ig.kernel_names()


def test_every_kernel_variant():
    """Each kernel of the table, forced, on problems with tails in every GEMM dimension
    (K not a tile multiple, NPQ ragged, CRS not a multiple of the k tile; odd and even
    numbers of reduction steps)."""
    import paper_1410_0759_amd as ig
    for kid, name in _kernel_cases():
        if "wgrad" in name or name.startswith("f64"):   # backward-filter and double-precision kernels: covered by their own tests
            continue
        dtype = "bf16" if name.startswith("bf16") else "f32"
        vec = "vecw" in name
        swap = "swap" in name
        nopad = "nopad" in name or ("direct" in name and "border" not in name)
        taps9 = "taps9" in name
        vecn = 8 if dtype == "bf16" else 4
        problems = [
            (3, 8 if vec else 5, 15, 17, 150, 3, 3, (1, 1), (1, 1)),
            (2, 16 if vec else 3, 21, 9, 45, 2, 2 if vec else 3, (0, 1), (2, 1)),
            (2, 24 if vec else 13, 9, 11, 33, 1, 1, (0, 0), (1, 1)),
        ]
        if taps9:   # nine taps, channels in fours; odd and even step counts
            vec = True
            problems = [
                (3, 8, 15, 17, 150, 3, 3, (1, 1), (1, 1)),
                (2, 12, 21, 9, 45, 3, 3, (0, 2), (2, 1)),
                (2, 4, 9, 30, 33, 1, 9, (0, 4), (1, 2)),
                (1, 20, 12, 7, 70, 9, 1, (5, 0), (1, 1)),
            ]
            if "x72 " in name:   # steps of eight channels
                problems = [(n_, 8 * ((c_ + 7) // 8), h_, w_, k_, r_, s_, pd, st) for (n_, c_, h_, w_, k_, r_, s_, pd, st) in problems]
        if "direct" in name:   # the reduction cut among 8 or 16 wavefronts: long ones, a ragged end, wavefronts left without steps
            problems = problems + [(2, 40, 12, 9, 70, 5, 3, (0, 0), (1, 2)), (1, 24, 20, 21, 130, 7, 7, (0, 0), (1, 1)),
                                   (2, 8 if vec else 7, 9, 9, 40, 3, 3, (0, 0), (1, 1)), (1, 4 if vec else 1, 12, 12, 33, 2, 2, (0, 0), (1, 1))]
            if "border" in name:   # zero borders (wider than the image allows windows wholly outside it), at most 31 taps
                problems = [pr for pr in problems if pr[5] * pr[6] <= 31] + [
                    (2, 40, 12, 9, 70, 5, 3, (2, 1), (1, 2)), (1, 24, 20, 21, 130, 5, 5, (2, 2), (1, 1)),
                    (2, 8, 9, 9, 40, 3, 3, (1, 1), (1, 1)), (1, 4, 3, 4, 33, 2, 2, (3, 2), (1, 1)), (1, 12, 6, 7, 20, 5, 6, (4, 5), (2, 3))]
        if "teams" in name:   # long reductions: several steps per team, a ragged last step, a team left without steps
            problems = problems + ([(2, 40, 15, 17, 150, 3, 3, (1, 1), (1, 1)), (1, 136, 9, 11, 70, 3, 3, (1, 1), (2, 1))] if taps9 else
                                   [(2, 40, 12, 9, 70, 5, 3, (0, 0), (1, 2)), (1, 24, 20, 21, 130, 7, 7, (0, 0), (1, 1)), (2, 8, 9, 9, 40, 3, 3, (0, 0), (1, 1))])
        if "table short" in name:   # an even number of steps, the last one at most half full
            problems = [
                (3, 5, 15, 17, 150, 3, 3, (0, 0), (1, 1)),        # C*R*S = 45: 2 steps, 13 in the last
                (2, 3, 35, 33, 96, 11, 11, (0, 0), (4, 4)),       # 363: 12 steps, 11 in the last
                (2, 7, 12, 9, 70, 5, 3, (0, 0), (1, 2)),          # 105: 4 steps, 9 in the last
            ]
        if "table odd" in name:   # an odd number of steps (of 16): the step that rounds it up is not multiplied
            problems = [
                (3, 5, 15, 17, 150, 3, 3, (0, 0), (1, 1)),        # C*R*S = 45: 3 steps
                (2, 3, 35, 33, 96, 11, 11, (0, 0), (4, 4)),       # 363: 23 steps
                (2, 7, 12, 9, 70, 5, 3, (0, 0), (1, 2)),          # 105: 7 steps
                (2, 16, 9, 11, 40, 3, 1, (0, 0), (1, 1)),         # 48: 3 whole steps
            ]
        channels = "channels" in name or "patch" in name or "pointwise" in name
        if "pointwise" in name:   # 1x1 filters, channels in eights and contiguous; one step, several, a ragged last one; strides, a border
            vec = True
            problems = [
                (3, 16, 15, 17, 150, 1, 1, (0, 0), (1, 1)),
                (2, 72, 21, 9, 45, 1, 1, (0, 0), (2, 1)),
                (2, 200, 9, 30, 33, 1, 1, (1, 2), (1, 2)),
                (1, 8, 12, 7, 200, 1, 1, (0, 0), (1, 1)),
                (2, 128, 14, 14, 64, 1, 1, (0, 0), (1, 1)),
            ]
        elif channels:   # nine taps, channels in sixteens and contiguous; odd and even step counts
            vec = True
            problems = [
                (3, 16, 15, 17, 150, 3, 3, (1, 1), (1, 1)),
                (2, 48, 21, 9, 45, 3, 3, (0, 2), (2, 1)),
                (2, 32, 9, 30, 33, 1, 9, (0, 4), (1, 2)),
                (1, 80, 12, 7, 200, 9, 1, (5, 0), (1, 1)),
            ]
            if "x256x" in name:   # 256 strided columns would not fit the staged image patch
                problems = [pr[:8] + ((1, 1),) for pr in problems]
            if "two groups" in name:   # steps of 32 channels: one step, an odd and an even number of them
                problems = [(n_, 32 * ((c_ + 31) // 32), h_, w_, k_, r_, s_, pd, st) for (n_, c_, h_, w_, k_, r_, s_, pd, st) in problems]
                problems[3] = (1, 96, 12, 7, 200, 3, 3, (1, 1), (1, 1))   # (the 9x1 one's 22 padded rows exceed this kernel's smaller patch)
        for (N, C, H, W, K, R, S, pad, stride) in problems:
            if nopad:
                pad = (0, 0)
            if vec:
                assert (C * R * S) % vecn == 0
            x, w = wl.random_problem(7 + kid, N, C, H, W, K, R, S, dtype=dtype)
            if channels:
                x = wl.with_layout(x, "NHWC")
            y0 = np.random.default_rng(kid).uniform(-1, 1, size=(N, K, (H + 2 * pad[0] - R) // stride[0] + 1,
                                                                 (W + 2 * pad[1] - S) // stride[1] + 1)).astype(np.float32)
            lay = "NHWC" if swap else "NCHW"
            _, plan = _check(x, w, pad, stride, 1, dtype, kernel=kid, y_layout=lay, tag=name)
            assert plan.kernelId == kid
            _check(x, w, pad, stride, 0, dtype, alpha=0.5, beta=-1.5, y0=y0, kernel=kid, y_layout=lay, tag=name)


def test_gather_modes_are_chosen():
    """Nine taps and channels in fours -> tap table; more than 63 taps and enough channels -> tap-major order; few channels, unpadded -> unpadded gather in
    filter order; few channels, padded -> masked filter order (fp32, up to 63 taps) or generic; few output elements and a long reduction
    -> the reduction cut inside the workgroup, with a tap mask per column when there is a border."""
    x, w = wl.random_problem(3, 8, 32, 40, 40, 64, 3, 3)
    _, plan = _check(x, w, (1, 1), (1, 1), 1, "f32", tag="mode taps9")
    assert plan.gatherMode == 3 and plan.kSteps == 32 // (plan.tileK // 9)   # whole channels per step
    x, w = wl.random_problem(3, 2, 32, 12, 12, 8, 3, 3)
    _, plan = _check(x, w, (1, 1), (1, 1), 1, "f32", tag="mode direct border")
    assert plan.gatherMode == 16 and plan.tileM == 32 and plan.tileN == 32
    x, w = wl.random_problem(3, 2, 32, 14, 14, 8, 9, 8)
    _, plan = _check(x, w, (2, 1), (1, 1), 1, "f32", tag="mode tapmajor")
    assert plan.gatherMode == 1 and plan.kSteps == 72
    x, w = wl.random_problem(4, 2, 3, 12, 12, 8, 5, 5)
    _, plan = _check(x, w, (0, 0), (2, 1), 0, "f32", tag="mode nopad table")
    assert plan.gatherMode == 7 and plan.kSteps == 3      # short reduction: tap offsets tabulated in LDS
    x, w = wl.random_problem(4, 2, 3, 35, 33, 32, 11, 11)
    _, plan = _check(x, w, (0, 0), (4, 4), 1, "f32", tag="mode nopad table, short last step")
    assert plan.gatherMode == 11 and plan.kSteps == 12    # 363 = 11 * 32 + 11: the last step runs half of its k-groups
    x, w = wl.random_problem(4, 2, 1, 20, 20, 33, 7, 7)
    _, plan = _check(x, w, (0, 0), (2, 1), 1, "f32", tag="mode nopad table, 17 indices in the last step")
    assert plan.gatherMode == 7 and plan.kSteps == 2
    xp_, wp_ = wl.random_problem(5, 2, 64, 14, 14, 96, 1, 1, dtype="bf16")
    _, plan = _check(wl.with_layout(xp_, "NHWC"), wp_, (0, 0), (1, 1), 1, "bf16", y_layout="NHWC", tag="mode pointwise")
    assert plan.gatherMode == 12 and plan.kSteps == 1 and plan.swapOperands == 1
    xl, wl_ = wl.random_problem(4, 1, 100, 9, 9, 8, 5, 5)
    _, plan = _check(xl, wl_, (0, 0), (1, 1), 0, "f32", kernel=[i for i, n in enumerate(_names()) if n == "f32 32x128x32 nopad"][0],
                     tag="mode nopad")
    assert plan.gatherMode == 2 and plan.kSteps == 79     # (2500 indices would not fit the table)
    # padded, at most 63 taps, fp32: filter order with a per-column mask of the taps that fall outside
    _, plan = _check(x, w, (2, 2), (1, 1), 0, "f32", tag="mode masked")
    assert plan.gatherMode == 14
    _, plan = _check(x, w, (3, 1), (2, 1), 1, "f32", y_layout="NHWC", tag="mode masked swap")
    assert plan.gatherMode == 14 and plan.swapOperands == 1
    # more than 63 taps, or bf16: per-element bounds checks
    x, w = wl.random_problem(4, 2, 1, 20, 20, 33, 8, 8)
    _, plan = _check(x, w, (2, 2), (1, 1), 0, "f32", tag="mode generic")
    assert plan.gatherMode == 0
    _, plan = _check(x, w, (3, 1), (2, 1), 1, "f32", y_layout="NHWC", tag="mode generic swap")
    assert plan.gatherMode == 0 and plan.swapOperands == 1
    # bf16, nine taps, contiguous channels in sixteens: channel vectors from a staged image patch;
    # an image too wide for the patch: channel vectors gathered tap by tap
    x, w = wl.random_problem(5, 3, 48, 13, 11, 40, 3, 3, dtype="bf16")
    _, plan = _check(wl.with_layout(x, "NHWC"), w, (1, 1), (1, 1), 0, "bf16", y_layout="NHWC", tag="mode patch")
    assert plan.gatherMode == 5 and plan.kSteps == 3 and plan.swapOperands == 1
    x, w = wl.random_problem(6, 1, 16, 5, 300, 24, 3, 3, dtype="bf16")
    _, plan = _check(wl.with_layout(x, "NHWC"), w, (1, 1), (1, 1), 1, "bf16", tag="mode channels")
    assert plan.gatherMode == 4 and plan.kSteps == 1


def test_tapmajor_ragged_channel_chunks():
    """Tap-major kernels with C below, equal to and above the chunk size, ragged or not,
    including filters holding Inf in channels that a ragged chunk would otherwise touch."""
    import paper_1410_0759_amd as ig
    names = ig.kernel_names()
    for name in ("f32 64x128x32 tapmajor", "f32 128x128x32 tapmajor swap", "bf16 128x128x32 tapmajor"):
        kid = names.index(name)
        dtype = "bf16" if name.startswith("bf16") else "f32"
        lay = "NHWC" if "swap" in name else "NCHW"
        for C in (1, 7, 32, 33, 48, 64, 70):
            x, w = wl.random_problem(100 + C, 2, C, 9, 10, 40, 3, 2, dtype=dtype)
            _check(x, w, (1, 1), (1, 1), 1, dtype, kernel=kid, y_layout=lay, tag=name)
            _check(x, w, (0, 1), (2, 1), 0, dtype, kernel=kid, y_layout=lay, tag=name)
    # a huge weight right after a ragged row must not leak into the previous filter
    x, w = wl.random_problem(5, 1, 33, 6, 6, 3, 1, 1)
    w[1, 0, 0, 0] = np.float32(3.0e38)
    x[:, 0] = 0.0
    _check(x, w, (0, 0), (1, 1), 1, "f32", kernel=names.index("f32 64x128x32 tapmajor"), tag="big neighbour")


def test_tapmajor_ragged_channel_chunk_in_a_cut_reduction():
    """The same when a lent workspace cuts the reduction into ranges, some of which begin inside the
    ragged last channel chunk: C = 40 in chunks of 32 with 5x5 taps is 50 steps, the last 25 ragged.
    The channels 40..63 a ragged chunk of filter k would touch are filter k+1's first 24: they hold
    Inf (x is zero there, so filter 1's own outputs are NaN in the oracle too and are left out)."""
    import paper_1410_0759_amd as ig
    gu = _gpu()
    names = ig.kernel_names()
    x, w = wl.random_problem(77, 1, 40, 8, 8, 3, 5, 5)
    w[1, :24] = np.float32(np.inf)
    x[:, :24] = 0.0
    want = oc.conv_forward(x, w, pad=(2, 2), stride=(1, 1), mode=1)
    assert np.all(np.isnan(want[:, 1])) and np.all(np.isfinite(want[:, [0, 2]]))
    for lend in (False, True):
        g = gu.GpuConv(x, w, (2, 2), (1, 1), 1)
        g.handle.set_kernel_override(names.index("f32 64x128x32 tapmajor"))
        if lend:
            assert g.lend_workspace() >= 2 * want.size * 4, "the reduction of this problem should be cut"
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        got = g.result()
        assert gu.rel_err(got[:, [0, 2]], want[:, [0, 2]]) <= gu.BOUND["f32"], lend


# ------------------------------------------------------------------ layouts through strides
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("x_layout,y_layout", [("NCHW", "NCHW"), ("NHWC", "NHWC"), ("NHWC", "NCHW"),
                                               ("NCHW", "NHWC")])
def test_layouts(x_layout, y_layout, dtype):
    x, w = wl.random_problem(31, 3, 24, 10, 9, 40, 3, 3, x_layout=x_layout, dtype=dtype)
    _check(x, w, (1, 1), (1, 1), 1, dtype, y_layout=y_layout, tag="layout")


def test_pitched_and_sliced_views():
    """Sub-section indexing: x is a channel slice of a wider, row-padded buffer."""
    rng = np.random.default_rng(5)
    big = rng.uniform(-1, 1, size=(2, 9, 12, 20)).astype(np.float32)
    x = big[:, 2:7, :, 3:16]      # channels 2..6, columns 3..15, pitch 20
    w = rng.standard_normal((12, 5, 3, 3)).astype(np.float32) * 0.2
    _check(x, w, (1, 1), (1, 1), 1, "f32", tag="view")
    _check(x, w, (0, 2), (2, 1), 0, "f32", tag="view")


def test_group_convolution_by_slices():
    """Group convolution as several calls on channel slices (what the framework layer does)."""
    gu = _gpu()
    rng = np.random.default_rng(6)
    x = rng.uniform(-1, 1, size=(2, 8, 10, 10)).astype(np.float32)
    w = rng.standard_normal((6, 4, 3, 3)).astype(np.float32) * 0.2   # 2 groups of 4 channels -> 3 filters
    for g in range(2):
        xg = x[:, 4 * g:4 * g + 4]
        wg = w[3 * g:3 * g + 3]
        _check(xg, wg, (1, 1), (1, 1), 1, "f32", tag="group")


def test_alpha_beta_and_nan_prefill():
    x, w = wl.random_problem(41, 2, 6, 12, 12, 20, 3, 3)
    y0 = np.random.default_rng(42).uniform(-1, 1, size=(2, 20, 12, 12)).astype(np.float32)
    _check(x, w, (1, 1), (1, 1), 1, "f32", alpha=1.0, beta=1.0, y0=y0, tag="beta1")
    _check(x, w, (1, 1), (1, 1), 1, "f32", alpha=0.0, beta=2.0, y0=y0, tag="alpha0")
    _check(x, w, (1, 1), (1, 1), 1, "f32", alpha=-3.0, beta=0.0, tag="nan prefill")   # y prefilled with NaN


def test_deterministic_run_to_run():
    gu = _gpu()
    x, w = wl.random_problem(43, 4, 32, 14, 14, 64, 3, 3)
    a, _ = gu.run(x, w, (1, 1), (1, 1))
    b, _ = gu.run(x, w, (1, 1), (1, 1))
    assert np.array_equal(a, b)


def test_workspace_is_zero_and_no_device_allocation():
    import torch
    import paper_1410_0759_amd as ig
    gu = _gpu()
    x, w = wl.random_problem(44, 2, 8, 16, 16, 32, 3, 3)
    g = gu.GpuConv(x, w, (1, 1), (1, 1), 1)
    assert ig.get_workspace_size(g.handle, g.xdesc, g.wdesc, g.conv, g.ydesc) == 0
    g.prefill(value=0.0)
    g.launch()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(10):
        g.launch()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, "device memory changed across forward calls"


def test_two_threads_two_handles():
    """Section 2.1: the library is callable from different host threads."""
    import threading
    import torch
    gu = _gpu()
    x, w = wl.random_problem(45, 2, 8, 20, 20, 48, 3, 3)
    want = oc.conv_forward(x, w, pad=(1, 1))
    results = {}

    def work(i):
        torch.cuda.set_device(0)
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            g = gu.GpuConv(x, w, (1, 1), (1, 1), 1)
            g.prefill(value=float("nan"))
            for _ in range(20):
                g.launch()
            s.synchronize()
            results[i] = g.result()

    ts = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    [t.start() for t in ts]
    [t.join() for t in ts]
    for i in range(2):
        assert gu.rel_err(results[i], want) <= gu.BOUND["f32"]


# ------------------------------------------------------------------ the five workloads at full size
@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_workload_full_size(index):
    """Full-size parity on the whole output, in the launch configuration the bench times."""
    gu = _gpu()
    w_ = wl.by_index(index)
    x, w, y0 = wl.make_inputs(w_)
    print("workload", w_.name, flush=True)
    got, plan = gu.run(x, w, (w_.pad_h, w_.pad_w), (w_.u, w_.v), w_.mode, w_.alpha, w_.beta, y0, w_.dtype,
                       w_.y_layout)
    assert got.shape == (w_.N, w_.K, w_.P, w_.Q)
    want = oc.conv_forward(x, w, pad=(w_.pad_h, w_.pad_w), stride=(w_.u, w_.v), mode=w_.mode,
                           alpha=w_.alpha, beta=w_.beta, y_old=y0)
    err = gu.rel_err(got, want)
    print("workload", w_.name, "kernel", plan.kernelId, "rel err", err, flush=True)
    assert err <= gu.BOUND[w_.dtype]


# ------------------------------------------------------------------ the paper's Table-2 layers
@pytest.mark.parametrize("layer", [1, 2, 3, 4, 5])
def test_table2_layer_sampled(layer):
    """The paper's layer collection at full size (N = 128) on the GPU; the oracle checks the
    whole output of a sample of images (the first two and the last two - images are
    independent, eq. 3)."""
    gu = _gpu()
    w_ = wl.TABLE2_LAYERS[layer - 1]
    x, w, _ = wl.make_inputs(w_)
    print("workload", w_.name, flush=True)
    got, plan = gu.run(x, w, (0, 0), (1, 1), w_.mode)
    assert got.shape == (w_.N, w_.K, w_.P, w_.Q)
    assert np.all(np.isfinite(got))
    for sl in (slice(0, 2), slice(w_.N - 2, w_.N)):
        want = oc.conv_forward(x[sl], w, mode=w_.mode)
        err = gu.rel_err(got[sl], want)
        print("workload", w_.name, "kernel", plan.kernelId, "images", sl, "rel err", err, flush=True)
        assert err <= gu.BOUND["f32"]


# ------------------------------------------------------------------ fused epilogue
def test_fused_bias_and_activation():
    """y = f(alpha*conv + beta*y + bias[k]) in one kernel, against the composition of the
    oracles (convolution, tensor addition with broadcasting, activation); every epilogue
    variant: pixels or channels along the lanes, full and ragged tiles, fp32 and bf16 kernels."""
    from oracle import pointwise_oracle as po
    gu = _gpu()
    cases = [
        # N, C, H, W, K, R, S, pad, stride, dtype, x layout, y layout
        (2, 5, 15, 17, 150, 3, 3, (1, 1), (1, 1), "f32", "NCHW", "NCHW"),
        (2, 8, 15, 17, 130, 3, 3, (1, 1), (1, 1), "f32", "NCHW", "NHWC"),
        (4, 16, 16, 16, 64, 3, 3, (1, 1), (1, 1), "f32", "NCHW", "NCHW"),     # full tiles: the unmasked store path
        (2, 3, 31, 31, 96, 11, 11, (0, 0), (4, 4), "f32", "NCHW", "NCHW"),
        (3, 48, 13, 11, 70, 3, 3, (1, 1), (1, 1), "bf16", "NHWC", "NHWC"),    # channel-vector kernel
        (3, 32, 13, 11, 40, 3, 3, (1, 1), (1, 1), "bf16", "NHWC", "NCHW"),
        (2, 7, 9, 9, 33, 5, 5, (2, 2), (2, 2), "bf16", "NCHW", "NCHW"),
    ]
    for i, (N, C, H, W, K, R, S, pad, stride, dtype, xl, yl) in enumerate(cases):
        x, w = wl.random_problem(50 + i, N, C, H, W, K, R, S, x_layout=xl, dtype=dtype)
        bias = np.random.default_rng(60 + i).uniform(-1, 1, size=K).astype(np.float32)
        raw = oc.conv_forward(x, w, pad=pad, stride=stride, mode=1)
        y0 = np.random.default_rng(70 + i).uniform(-1, 1, size=raw.shape).astype(np.float32)
        for act, alpha, beta, with_bias in [(1, 1.0, 0.0, True), (0, 0.5, -1.5, True), (2, 2.0, 1.0, True),
                                            (-1, 1.0, 0.0, True), (1, 1.0, 0.0, False)]:
            print("fused", cases[i], act, alpha, beta, with_bias, flush=True)
            g = gu.GpuConv(x, w, pad, stride, 1, dtype=dtype, y_layout=yl)
            if beta != 0.0:
                g.prefill(y0=y0)
            else:
                g.prefill(value=float("nan"))
            g.launch_fused(alpha, beta, bias if with_bias else None, act)
            got = g.result()
            pre = alpha * raw + (beta * y0.astype(np.float64) if beta != 0.0 else 0.0)
            if with_bias:
                pre = pre + po.add_tensor(bias.reshape(1, K, 1, 1), raw.shape)
            want = pre if act < 0 else po.activation_forward(act, pre.astype(np.float32))
            # (the activation oracle takes float32 inputs: compare with the matching slack)
            assert np.all(np.isfinite(got))
            err = gu.rel_err(got, want)
            assert err <= gu.BOUND[dtype], (cases[i], act, err)


# ------------------------------------------------------------------ optional workspace (small problems)
@pytest.mark.gpu
def test_forward_tap_major_with_filter_workspace():
    """A problem that runs in tap-major order (padded, not nine taps, enough channels and plenty of tiles; float with more
    than 63 taps, or bfloat16):
    the optional workspace is the filter's size, the filter is rewritten there with the channel index innermost and
    read through those strides.  Same sums in the same order: the same bits as without the workspace."""
    import paper_1410_0759_amd as ig
    gu = _gpu()
    cases = [
        # N, C, H, W, K, R, S, pad, stride, mode, data type
        # (float layers of up to 63 taps run in filter order under a mask of the taps outside, and ask for nothing)
        (32, 64, 20, 20, 70, 9, 8, (4, 3), (1, 1), 1, "f32"),
        (64, 80, 21, 19, 150, 13, 5, (6, 2), (2, 1), 0, "f32"),     # ragged last channel chunk, eq. 2 order
        (64, 64, 20, 20, 70, 5, 5, (2, 2), (1, 1), 1, "bf16"),
        (64, 80, 21, 19, 150, 7, 3, (3, 1), (2, 1), 0, "bf16"),
    ]
    for i, (N, C, H, W, K, R, S, pad, stride, mode, dtype) in enumerate(cases):
        x, w = wl.random_problem(120 + i, N, C, H, W, K, R, S, dtype=dtype)
        want = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode)
        g = gu.GpuConv(x, w, pad, stride, mode, dtype=dtype)
        assert g.plan().gatherMode == 1
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        plain = g.result()
        asked = g.lend_workspace()
        assert asked == K * C * R * S * (4 if dtype == "f32" else 2)
        print("tap-major with filter workspace", (N, C, H, W, K, R, S, pad, stride, mode), dtype, flush=True)
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        got = g.result()
        g.ws.result()                                   # guard bands of the workspace
        assert gu.rel_err(got, want) <= gu.BOUND[dtype]
        assert np.array_equal(got, plain)
        g.lend_workspace(asked - 4)                      # too small: the filter is read in place
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        assert np.array_equal(g.result(), plain)


def test_forward_few_channels_zero_border_with_image_workspace():
    """Few channels and a zero border: the layer runs with the masked gather, or - lent a workspace for x with its
    border written out - as a layer without a border over that copy.  Both against the oracle, with alpha/beta,
    bias and activation passed through, channel-fastest x, and a workspace too small (ignored)."""
    gu = _gpu()
    cases = [
        # N, C, H, W, K, R, S, pad, stride, mode, x layout
        (8, 3, 40, 38, 64, 7, 7, (3, 3), (2, 2), 1, "NCHW"),
        (4, 3, 33, 35, 24, 3, 3, (1, 1), (1, 1), 0, "NHWC"),
        (6, 1, 28, 28, 20, 5, 5, (2, 1), (1, 2), 1, "NCHW"),
    ]
    for i, (N, C, H, W, K, R, S, pad, stride, mode, xl) in enumerate(cases):
        x, w = wl.random_problem(140 + i, N, C, H, W, K, R, S)
        xg = wl.with_layout(x, xl)
        want = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode)
        y0 = np.random.default_rng(150 + i).uniform(-1, 1, size=want.shape).astype(np.float32)
        want2 = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode, alpha=0.5, beta=-1.5, y_old=y0)
        g = gu.GpuConv(xg, w, pad, stride, mode)
        assert g.plan().gatherMode == 14
        asked = g.lend_workspace()
        assert asked == N * C * (H + 2 * pad[0]) * (W + 2 * pad[1]) * 4
        print("image workspace", cases[i], flush=True)
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        assert gu.rel_err(g.result(), want) <= gu.BOUND["f32"]
        g.ws.result()                                   # guard bands of the workspace
        g.prefill(y0=y0)
        g.launch(0.5, -1.5)
        assert gu.rel_err(g.result(), want2) <= gu.BOUND["f32"]
        bias = np.random.default_rng(160 + i).uniform(-1, 1, size=K).astype(np.float32)
        g.prefill(value=float("nan"))
        g.launch_fused(1.0, 0.0, bias, 1)
        assert gu.rel_err(g.result(), np.maximum(want + bias[None, :, None, None], 0.0)) <= gu.BOUND["f32"]
        g.lend_workspace(asked - 4)
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        assert gu.rel_err(g.result(), want) <= gu.BOUND["f32"]


def test_small_problems_run_with_the_reduction_cut_inside_the_workgroup():
    """Few output elements and a long reduction, no workspace: 32 x 32 tiles, the reduction cut among the wavefronts of
    a workgroup, operands straight from global memory.  Chosen by the library for such shapes; checked with eq. 2's
    inverted filter, strides, channel-fastest x and y, alpha/beta, and the fused bias + activation."""
    gu = _gpu()
    cases = [
        # N, C, H, W, K, R, S, pad, stride, mode, x layout, y layout
        (4, 128, 16, 16, 128, 7, 7, (0, 0), (1, 1), 1, "NCHW", "NCHW"),      # a deep layer of Table 2 at a mini-batch of 4
        (2, 96, 21, 19, 70, 5, 3, (0, 0), (2, 1), 0, "NHWC", "NHWC"),
        (1, 300, 9, 11, 33, 3, 4, (0, 0), (1, 2), 0, "NCHW", "NHWC"),
        # with a zero border (up to 31 taps): the window test from a tap mask per column
        (4, 256, 7, 7, 200, 3, 3, (1, 1), (1, 1), 1, "NCHW", "NCHW"),        # the last layers of a deep network at a small mini-batch
        (2, 96, 13, 11, 70, 5, 3, (2, 1), (2, 1), 0, "NHWC", "NHWC"),
        (1, 300, 5, 6, 33, 3, 4, (2, 3), (1, 2), 0, "NCHW", "NHWC"),
        (3, 64, 2, 3, 40, 5, 5, (4, 4), (1, 1), 0, "NCHW", "NCHW"),          # windows that lie wholly in the border
    ]
    for i, (N, C, H, W, K, R, S, pad, stride, mode, xl, yl) in enumerate(cases):
        x, w = wl.random_problem(170 + i, N, C, H, W, K, R, S)
        want = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode)
        y0 = np.random.default_rng(175 + i).uniform(-1, 1, size=want.shape).astype(np.float32)
        want2 = oc.conv_forward(x, w, pad=pad, stride=stride, mode=mode, alpha=0.5, beta=-1.5, y_old=y0)
        g = gu.GpuConv(wl.with_layout(x, xl), w, pad, stride, mode, y_layout=yl)
        print("direct", cases[i], flush=True)
        assert g.plan().gatherMode == (15 if pad == (0, 0) else 16)
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        assert gu.rel_err(g.result(), want) <= gu.BOUND["f32"]
        g.prefill(y0=y0)
        g.launch(0.5, -1.5)
        assert gu.rel_err(g.result(), want2) <= gu.BOUND["f32"]
        bias = np.random.default_rng(180 + i).uniform(-1, 1, size=K).astype(np.float32)
        g.prefill(value=float("nan"))
        g.launch_fused(1.0, 0.0, bias, 1)
        assert gu.rel_err(g.result(), np.maximum(want + bias[None, :, None, None], 0.0)) <= gu.BOUND["f32"]


def test_forward_with_optional_workspace():
    """Few output tiles and a long reduction: with a lent workspace the reduction is cut into
    ranges and summed in order.  Same result as without (to rounding), bitwise repeatable, any
    workspace size accepted, the mandatory workspace query still reports zero."""
    import paper_1410_0759_amd as ig
    gu = _gpu()
    cases = [
        # N, C, H, W, K, R, S, pad, stride, y layout
        (2, 128, 17, 17, 128, 7, 7, (0, 0), (1, 1), "NCHW"),     # unpadded, long filter rows
        (1, 256, 13, 13, 96, 3, 3, (1, 1), (1, 1), "NCHW"),      # nine-tap table
        (2, 200, 9, 9, 40, 5, 3, (2, 1), (1, 1), "NHWC"),        # tap-major, channels along the lanes
        (1, 300, 11, 11, 24, 3, 3, (1, 1), (2, 2), "NCHW"),
    ]
    for i, (N, C, H, W, K, R, S, pad, stride, yl) in enumerate(cases):
        x, w = wl.random_problem(90 + i, N, C, H, W, K, R, S)
        want = oc.conv_forward(x, w, pad=pad, stride=stride, mode=1)
        y0 = np.random.default_rng(95 + i).uniform(-1, 1, size=want.shape).astype(np.float32)
        want = oc.conv_forward(x, w, pad=pad, stride=stride, mode=1, alpha=0.5, beta=-1.5, y_old=y0)
        g = gu.GpuConv(x, w, pad, stride, 1, y_layout=yl)
        assert ig.get_workspace_size(g.handle, g.xdesc, g.wdesc, g.conv, g.ydesc) == 0
        outs = []
        asked = None
        for ws in ("none", "asked", "asked", "one part", "odd"):
            if ws == "none":
                pass
            elif ws == "asked":
                asked = g.lend_workspace()
                part = int(np.prod(want.shape)) * 4
                assert asked >= 2 * part and asked % part == 0, "this problem should be cut into ranges"
            elif ws == "one part":
                g.lend_workspace(part)               # too small to cut: runs as without
            else:
                g.lend_workspace(3 * part + 12)
            print("optional workspace", cases[i], ws, flush=True)
            g.prefill(y0=y0)
            g.launch(0.5, -1.5)
            got = g.result()
            if getattr(g, "ws", None) is not None:
                g.ws.result()                        # guard bands of the workspace
            assert gu.rel_err(got, want) <= gu.BOUND["f32"]
            outs.append(got)
        assert np.array_equal(outs[1], outs[2]), "same call, same bits"
        assert np.array_equal(outs[0], outs[3])
    # a problem with plenty of tiles is not cut; neither is one whose y has gaps
    x, w = wl.random_problem(99, 8, 16, 40, 40, 64, 3, 3)
    g = gu.GpuConv(x, w, (1, 1), (1, 1), 1)
    assert g.lend_workspace() == 0


def test_calls_can_be_captured_in_a_graph_and_replayed():
    """The library only enqueues kernels on the handle's stream (no allocation, no memset, no
    synchronisation), so a sequence of its calls can be captured in a HIP graph: forward with
    fused bias and rectifier, backward filter with its workspace and summing pass, backward data.
    Every replay, on new input contents and with eager work between the replays, must give the
    eager results bit for bit."""
    gu = _gpu()
    import torch
    import paper_1410_0759_amd as ig
    N, C, H, W, K, R, S, pad, stride = 4, 24, 20, 19, 40, 3, 3, (1, 1), (1, 1)
    P, Q = oc.output_dim(H, R, 1, 1), oc.output_dim(W, S, 1, 1)
    rng = np.random.default_rng(5)
    mk = lambda *s: torch.from_numpy(rng.uniform(-1, 1, size=s).astype(np.float32)).cuda()
    x, w, dy, bias = mk(N, C, H, W), mk(K, C, R, S), mk(N, K, P, Q), mk(K)
    y, dw, dx = torch.empty(N, K, P, Q, device="cuda"), torch.empty(K, C, R, S, device="cuda"), torch.empty(N, C, H, W, device="cuda")
    td = lambda t: ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, *t.shape, t.stride())
    xd, yd, dyd, dxd = td(x), td(y), td(dy), td(dx)
    wd = ig.FilterDescriptor().set(ig.IGC_DATA_FLOAT, K, C, R, S)
    conv = ig.ConvolutionDescriptor().set(1, 1, 1, 1, ig.IGC_CROSS_CORRELATION)
    h = ig.Handle()
    ws_bytes = ig.get_backward_filter_workspace_size(h, xd, dyd, conv, wd)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes // 4, device="cuda")

    def calls():
        h.set_stream(torch.cuda.current_stream().cuda_stream)
        ig.check(ig.convolution_bias_activation_forward(h, 1.0, xd, x.data_ptr(), wd, w.data_ptr(), conv, 0.0, bias.data_ptr(),
                                                        ig.IGC_ACTIVATION_RELU, yd, y.data_ptr()), "forward")
        ig.check(ig.convolution_backward_filter(h, 1.0, xd, x.data_ptr(), dyd, dy.data_ptr(), conv, 0.0, wd, dw.data_ptr(),
                                                ws.data_ptr(), ws_bytes), "backward filter")
        ig.check(ig.convolution_backward_data(h, 1.0, wd, w.data_ptr(), dyd, dy.data_ptr(), conv, 0.0, dxd, dx.data_ptr()), "backward data")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):      # (warm-up on the capture stream, as graph capture wants)
        calls()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        calls()
    for rep in range(3):
        for t in (x, w, dy, bias):
            t.copy_(mk(*t.shape))
        for t in (y, dw, dx):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (y, dw, dx)]
        for t in (y, dw, dx):
            t.fill_(float("nan"))
        calls()                         # eager, between the replays
        torch.cuda.synchronize()
        for g, e in zip(got, (y, dw, dx)):
            assert torch.equal(g, e), "replay %d differs from the eager result" % rep
    want = oc.conv_forward(x.cpu().numpy(), w.cpu().numpy(), pad=pad, stride=stride, mode=1)
    want = np.maximum(want + bias.cpu().numpy().astype(np.float64).reshape(1, -1, 1, 1), 0.0)
    assert gu.rel_err(y.cpu().numpy().astype(np.float64), want) <= gu.BOUND["f32"]
