"""The allocation-free backward-filter entry point (the library's own scratch array instead of
a workspace) against the ordinary one: same results on two calls in a row, the second on a
smaller problem, so that whatever the first call left in the scratch array is there to be
tripped over.  Collected last on purpose (the name sorts after the other test files)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import workloads as wl
from oracle import conv_oracle as oc


def _gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def _both(gu, x, dy, rs, pad, stride, dtype, alpha=1.0, beta=0.0, dw_old=None):
    """(dw from igcConvolutionBackwardFilter with its full workspace, dw from the allocation-free call)."""
    import torch
    import paper_1410_0759_amd as ig
    g = gu.GpuBackwardFilter(x, dy, rs, pad, stride, 1, dtype, "full")
    assert 0 < g.asked <= ig.NOALLOC_SCRATCH_BYTES, g.asked   # (a problem whose reduction is cut, and that fits)
    res = []
    for no_alloc in (False, True):
        if dw_old is not None:
            g.out.prefill(old=dw_old)
        else:
            g.out.prefill(value=float("nan"))
        g.handle.set_stream(torch.cuda.current_stream().cuda_stream)
        if no_alloc:
            before = torch.cuda.memory_allocated()
            st = ig.convolution_backward_filter_no_alloc(g.handle, alpha, g.xdesc, g.x_dev.data_ptr(), g.dydesc, g.dy_dev.data_ptr(),
                                                         g.conv, beta, g.dwdesc, g.out.ptr)
            ig.check(st, "igcConvolutionBackwardFilterNoAlloc")
            assert torch.cuda.memory_allocated() == before
        else:
            g.launch(alpha, beta)
        res.append(g.out.result())
    return res


def test_no_alloc_backward_filter_matches_on_two_calls_in_a_row():
    gu = _gpu()
    rng = np.random.default_rng(991)
    cases = [
        # (N, C, H, W, K, R, S, pad, stride, dtype, x layout): a larger problem, then a smaller one
        (16, 64, 28, 28, 96, 3, 3, (1, 1), (1, 1), "f32", "NCHW"),
        (4, 24, 13, 11, 40, 3, 3, (1, 1), (1, 1), "f32", "NCHW"),
        (8, 64, 14, 14, 64, 3, 3, (1, 1), (1, 1), "bf16", "NHWC"),
        (8, 3, 23, 23, 16, 5, 5, (0, 0), (2, 2), "f32", "NCHW"),
        (8, 130, 20, 20, 200, 3, 3, (1, 1), (1, 1), "f64", "NCHW"),   # (double: more ranges than resident workgroups)
        (4, 24, 13, 11, 40, 3, 3, (1, 1), (1, 1), "f64", "NCHW"),
    ]
    for (N, C, H, W, K, R, S, pad, stride, dtype, lay) in cases:
        print("no-alloc backward filter", N, C, H, W, K, R, S, pad, stride, dtype, lay, flush=True)
        x, _ = wl.random_problem(300 + N, N, C, H, W, K, R, S, x_layout=lay, dtype="f32" if dtype == "f64" else dtype)
        P, Q = oc.output_dim(H, R, stride[0], pad[0]), oc.output_dim(W, S, stride[1], pad[1])
        dy = rng.uniform(-1, 1, size=(N, K, P, Q)).astype(np.float32)
        if dtype == "bf16":
            dy = wl.round_to_bf16(dy)
        dy = wl.with_layout(dy, lay)
        old = rng.uniform(-1, 1, size=(K, C, R, S)).astype(np.float32)
        # (double precision: the same float-valued inputs as doubles)
        as_dev = (lambda a: None if a is None else a.astype(np.float64)) if dtype == "f64" else (lambda a: a)
        for alpha, beta, dw_old in ((1.0, 0.0, None), (0.5, -2.0, old)):
            ref, got = _both(gu, as_dev(x), as_dev(dy), (R, S), pad, stride, dtype, alpha, beta, as_dev(dw_old))
            assert np.array_equal(ref, got), "not bit for bit the ordinary entry point's result"
            want = oc.conv_backward_filter(x, dy, (R, S), pad=pad, stride=stride, mode=1, alpha=alpha, beta=beta, dw_old=dw_old)
            assert gu.rel_err(got, want) <= gu.BOUND[dtype]
