"""Benchmark: convolution forward effective TFLOP/s and fraction of the MI355X matrix peak.

A step is one igcConvolutionForward call (the whole hot path) on one batch of seeded
synthetic input already resident in HBM.  Prints ONE JSON line.  The headline workload
is the second entry of the workload list (large-kernel strided first layer, fp32); all five
workloads are timed and reported inside "roofline" ("per_config": mean, median and minimum
per launch, TFLOP/s, fraction of the matrix peak of the data type, parity error, kernel),
with the measured rate of a register-only MFMA loop ("achievable_peak") beside the datasheet
peaks.  The CPU oracle is timed beside it on a bounded sample of the same workload as a
stated baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2516.6, "f64": 78.6}   # MI355X dense matrix peaks (256 CUs x 2.4 GHz)
# acceptance bars of the parity measure max|gpu - oracle| / max|oracle|
TOL = {"f32": 2e-5, "bf16": 1e-2, "f64": 1e-12}
# The chip idles between the sections of this script (input generation, oracle runs) and needs
# some milliseconds of work to come back to its sustained engine and memory clocks; a timed region
# of 20 launches of 0.1 ms would otherwise measure the ramp (measured: 127 us per launch of the
# headline kernel right after an idle phase against 114 us from the hundredth launch on; a
# register-only MFMA loop does not do it, the memory clocks matter too).  Before every timed
# region the call itself is therefore repeated, untimed, for this long.
CLOCK_WARMUP_MS = 30
_warm = {"ms": CLOCK_WARMUP_MS}


def warm_clocks(call):
    import torch
    if _warm["ms"] <= 0:
        return
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < _warm["ms"]:
        for _ in range(10):
            call()
        torch.cuda.synchronize()


def time_calls(call, steps, warmup):
    """Times `steps` calls after `warmup` untimed ones, HIP events on the launch stream.
    Returns (mean, median, min) milliseconds per call: the mean from one pair of events
    around all the calls, median and minimum from a second pass with an event after every
    call (back-to-back launches on one stream: the gap between two events is one call)."""
    import torch
    warm_clocks(call)
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        call()
    e1.record()
    torch.cuda.synchronize()
    mean = e0.elapsed_time(e1) / steps
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        call()
        ev[i + 1].record()
    torch.cuda.synchronize()
    each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    return mean, each[len(each) // 2], each[0]


def time_gpu(g, alpha, beta, steps, warmup):
    """Mean milliseconds per call of g.launch(alpha, beta)."""
    return time_calls(lambda: g.launch(alpha, beta), steps, warmup)[0]


def run_config(index, steps, warmup, oracle_seconds, kernel=None, workload=None, lend_workspace=False):
    import numpy as np
    import workloads as wl
    from oracle import conv_oracle as oc
    from paper_1410_0759_amd import runner as gu
    import paper_1410_0759_amd as ig

    w_ = workload if workload is not None else wl.by_index(index)
    x, w, y0 = wl.make_inputs(w_)
    g = gu.GpuConv(x, w, (w_.pad_h, w_.pad_w), (w_.u, w_.v), w_.mode, dtype=w_.dtype, y_layout=w_.y_layout)
    if kernel is not None:
        g.handle.set_kernel_override(kernel)
    if lend_workspace:   # the optional workspace that lets a problem with few tiles cut its reduction
        g.lend_workspace()
    plan = g.plan()
    # parity run first (single call on the prefilled / NaN-poisoned output)
    if y0 is not None:
        g.prefill(y0=y0)
    else:
        g.prefill(value=float("nan"))
    g.launch(w_.alpha, w_.beta)
    got = g.result()
    # timed runs (beta != 0 keeps accumulating into y: same work every call)
    g.prefill(value=0.0)
    ms, median_ms, min_ms = time_calls(lambda: g.launch(w_.alpha, w_.beta), steps, warmup)
    tflops = w_.flops / (ms * 1e-3) / 1e12

    # oracle on a bounded sample: the first n images (images are independent)
    cores = len(os.sched_getaffinity(0))
    macs_per_image = w_.flops / 2 / w_.N
    rate_guess = 0.2e9 * cores                      # plain seven-loop code, MAC/s
    n = int(max(1, min(w_.N, oracle_seconds * rate_guess / macs_per_image)))
    t0 = time.perf_counter()
    want = oc.conv_forward(x[:n], w, pad=(w_.pad_h, w_.pad_w), stride=(w_.u, w_.v), mode=w_.mode,
                           alpha=w_.alpha, beta=w_.beta, y_old=None if y0 is None else y0[:n])
    cpu_s = time.perf_counter() - t0
    err = gu.rel_err(got[:n], want)
    cpu_tflops = (2 * macs_per_image * n) / cpu_s / 1e12
    return {
        "workload": w_.name, "dtype": w_.dtype, "gflop": w_.flops / 1e9, "ms": ms, "median_ms": median_ms, "min_ms": min_ms,
        "tflops": tflops,
        "peak_tflops": PEAK_TFLOPS[w_.dtype], "frac_of_peak": tflops / PEAK_TFLOPS[w_.dtype],
        "kernel": ig.kernel_names()[plan.kernelId], "grid": plan.gridX, "k_steps": plan.kSteps,
        "rel_err": err, "tolerance": TOL[w_.dtype], "parity_images": n,
        "oracle_seconds": cpu_s, "oracle_tflops": cpu_tflops, "oracle_threads": oc.max_threads(),
        "host_cores": cores, "algorithmic_bytes": w_.algorithmic_bytes,
    }


def run_backward(index, steps, warmup, oracle_seconds, workload=None):
    """Backward data and backward filter at one workload's size: seeded dy of the forward
    output's shape, timing of each pass, parity against the oracle's backward forms on the
    first n images (backward data: those images of dx; backward filter: the same pass run
    on those images alone, since every image contributes to every filter element)."""
    import numpy as np
    import workloads as wl
    from oracle import conv_oracle as oc
    from paper_1410_0759_amd import runner as gu

    w_ = workload if workload is not None else wl.by_index(index)
    x, w, _ = wl.make_inputs(w_)
    pad, stride = (w_.pad_h, w_.pad_w), (w_.u, w_.v)
    dy = np.random.default_rng(14100759 * 10 + w_.index + 300).uniform(-1, 1, size=(w_.N, w_.K, w_.P, w_.Q)).astype(np.float32)
    if w_.dtype == "bf16":
        dy = wl.round_to_bf16(dy)
    dy = wl.with_layout(dy, w_.y_layout)
    cores = len(os.sched_getaffinity(0))
    macs_per_image = w_.flops / 2 / w_.N
    n = int(max(1, min(w_.N, oracle_seconds * 0.2e9 * cores / macs_per_image)))
    out = {"workload": w_.name, "dtype": w_.dtype, "gflop": w_.flops / 1e9, "parity_images": n,
           "tolerance": TOL[w_.dtype]}

    class _Timed:   # adapts the backward objects to time_gpu
        def __init__(self, g):
            self.g = g

        def launch(self, alpha, beta):
            self.g.launch(alpha, beta)

    g = gu.GpuBackwardData(dy, w, (w_.H, w_.W), pad, stride, w_.mode, w_.dtype, w_.x_layout)
    g.out.prefill(value=float("nan"))
    g.launch(1.0, 0.0)
    got = g.out.result()
    t0 = time.perf_counter()
    want = oc.conv_backward_data(dy[:n], w, (w_.H, w_.W), pad=pad, stride=stride, mode=w_.mode)
    cpu_s = time.perf_counter() - t0
    ms = time_gpu(_Timed(g), 1.0, 0.0, steps, warmup)
    out["backward_data"] = {"ms": ms, "tflops": w_.flops / ms / 1e9, "frac_of_peak": w_.flops / ms / 1e9 / PEAK_TFLOPS[w_.dtype],
                            "workspace_bytes": g.asked, "rel_err": gu.rel_err(got[:n], want), "oracle_seconds": cpu_s}
    del g

    g = gu.GpuBackwardFilter(x, dy, (w_.R, w_.S), pad, stride, w_.mode, w_.dtype)
    g.out.prefill(value=float("nan"))
    ms = time_gpu(_Timed(g), 1.0, 0.0, steps, warmup)
    assert np.all(np.isfinite(g.out.result()))
    got, _ = gu.run_backward_filter(x[:n], dy[:n], (w_.R, w_.S), pad, stride, w_.mode, dtype=w_.dtype)
    t0 = time.perf_counter()
    want = oc.conv_backward_filter(x[:n], dy[:n], (w_.R, w_.S), pad=pad, stride=stride, mode=w_.mode)
    cpu_s = time.perf_counter() - t0
    out["backward_filter"] = {"ms": ms, "tflops": w_.flops / ms / 1e9, "frac_of_peak": w_.flops / ms / 1e9 / PEAK_TFLOPS[w_.dtype],
                              "workspace_bytes": g.asked, "rel_err": gu.rel_err(got, want), "oracle_seconds": cpu_s}
    return out


def run_double_precision(steps, warmup, index=3):
    """The three passes in double precision at the shape of one workload on 64 images
    (float32-valued inputs held as doubles, so that the oracle, which takes float32 values and
    works in double, gives the expected result directly; parity on the first image)."""
    import numpy as np
    import workloads as wl
    from oracle import conv_oracle as oc
    from paper_1410_0759_amd import runner as gu

    w_ = wl.shrink(wl.by_index(index), 64)
    x, w, _ = wl.make_inputs(w_)
    pad, stride = (w_.pad_h, w_.pad_w), (w_.u, w_.v)
    dy = np.random.default_rng(14100759 * 10 + 640 + index).uniform(-1, 1, size=(w_.N, w_.K, w_.P, w_.Q)).astype(np.float32)
    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    out = {"workload": w_.name + " in double precision", "dtype": "f64", "gflop": w_.flops / 1e9, "tolerance": TOL["f64"]}

    class _Timed:
        def __init__(self, g):
            self.g = g

        def launch(self, alpha, beta):
            self.g.launch(alpha, beta)

    def entry(ms, err):
        return {"ms": ms, "tflops": w_.flops / ms / 1e9, "frac_of_peak": w_.flops / ms / 1e9 / PEAK_TFLOPS["f64"], "rel_err": err}

    g = gu.GpuConv(x64, w64, pad, stride, w_.mode, dtype="f64")
    g.prefill(value=float("nan"))
    g.launch(1.0, 0.0)
    err = gu.rel_err(g.result()[:1], oc.conv_forward(x[:1], w, pad=pad, stride=stride, mode=w_.mode))
    out["forward"] = entry(time_gpu(g, 1.0, 0.0, steps, warmup), err)
    import paper_1410_0759_amd as ig
    out["forward"]["kernel"] = ig.kernel_names()[g.plan().kernelId]
    del g
    g = gu.GpuBackwardData(dy64, w64, (w_.H, w_.W), pad, stride, w_.mode, "f64")
    g.out.prefill(value=float("nan"))
    g.launch(1.0, 0.0)
    err = gu.rel_err(g.out.result()[:1], oc.conv_backward_data(dy[:1], w, (w_.H, w_.W), pad=pad, stride=stride, mode=w_.mode))
    out["backward_data"] = entry(time_gpu(_Timed(g), 1.0, 0.0, steps, warmup), err)
    del g
    g = gu.GpuBackwardFilter(x64, dy64, (w_.R, w_.S), pad, stride, w_.mode, "f64")
    g.out.prefill(value=float("nan"))
    ms = time_gpu(_Timed(g), 1.0, 0.0, steps, warmup)
    got, _ = gu.run_backward_filter(x64[:1], dy64[:1], (w_.R, w_.S), pad, stride, w_.mode, dtype="f64")
    err = gu.rel_err(got, oc.conv_backward_filter(x[:1], dy[:1], (w_.R, w_.S), pad=pad, stride=stride, mode=w_.mode))
    out["backward_filter"] = entry(ms, err)
    out["backward_filter"]["workspace_bytes"] = g.asked
    return out


def run_padded_filters(steps, warmup):
    """Layers outside the paper's collection whose filters are neither nine taps nor unpadded (a 5x5 and a 7x7
    layer with zero borders): forward and backward data without a workspace (filter order, the window test read from
    a tap mask per column) and with whatever the optional-workspace query asks for (nothing for these float layers;
    the keys are kept so that a workspace-dependent route would show).  Parity on the first image against the oracle."""
    import numpy as np
    import workloads as wl
    from oracle import conv_oracle as oc
    from paper_1410_0759_amd import runner as gu
    import paper_1410_0759_amd as ig

    out = []
    for (N, C, H, W, K, R, S, pad) in ((128, 96, 27, 27, 256, 5, 5, (2, 2)), (128, 64, 56, 56, 64, 7, 7, (3, 3))):
        x, w = wl.random_problem(700 + R, N, C, H, W, K, R, S)
        flops = 2.0 * N * K * H * W * C * R * S
        entry = {"shape": "N%d C%d %dx%d K%d %dx%d pad %d" % (N, C, H, W, K, R, S, pad[0]), "gflop": flops / 1e9}
        g = gu.GpuConv(x, w, pad, (1, 1), 1)
        entry["kernel"] = ig.kernel_names()[g.plan().kernelId]
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        entry["rel_err"] = gu.rel_err(g.result()[:1], oc.conv_forward(x[:1], w, pad=pad, stride=(1, 1), mode=1))
        ms = time_gpu(g, 1.0, 0.0, steps, warmup)
        entry["forward"] = {"ms": ms, "tflops": flops / ms / 1e9}
        entry["workspace_bytes"] = g.lend_workspace()
        ms = time_gpu(g, 1.0, 0.0, steps, warmup)
        entry["forward_with_workspace"] = {"ms": ms, "tflops": flops / ms / 1e9}
        del g
        dy = np.random.default_rng(710 + R).uniform(-1, 1, size=(N, K, H, W)).astype(np.float32)

        class _Timed:
            def __init__(self, g):
                self.g = g

            def launch(self, alpha, beta):
                self.g.launch(alpha, beta)

        for ws, key in (("none", "backward_data"), ("full", "backward_data_with_workspace")):
            g = gu.GpuBackwardData(dy, w, (H, W), pad, (1, 1), 1, "f32", "NCHW", ws)
            ms = time_gpu(_Timed(g), 1.0, 0.0, steps, warmup)
            entry[key] = {"ms": ms, "tflops": flops / ms / 1e9}
            del g
        out.append(entry)
    return out


def run_small_layers(steps, warmup):
    """Padded layers at the mini-batches of serving (a handful of images, 7x7 to 28x28 pixels, long reductions): few
    output elements, so that tiles of 64 x 64 and more leave most compute units idle.  The library runs them with 32 x 32
    tiles and the reduction cut among the wavefronts of a workgroup (no workspace); beside it the same call with the
    pipelined nine-tap kernel forced, and parity of the whole output against the oracle."""
    import workloads as wl
    from oracle import conv_oracle as oc
    from paper_1410_0759_amd import runner as gu
    import paper_1410_0759_amd as ig

    names = ig.kernel_names()
    out = []
    for (N, C, HW, K, RS) in ((4, 512, 7, 512, 3), (1, 256, 14, 256, 3), (1, 512, 28, 512, 3), (2, 128, 28, 128, 5)):
        pad = (RS // 2, RS // 2)
        x, w = wl.random_problem(800 + HW + RS, N, C, HW, HW, K, RS, RS)
        flops = 2.0 * N * K * HW * HW * C * RS * RS
        g = gu.GpuConv(x, w, pad, (1, 1), 1)
        entry = {"shape": "N%d C%d %dx%d K%d %dx%d pad %d" % (N, C, HW, HW, K, RS, RS, pad[0]), "gflop": flops / 1e9,
                 "kernel": names[g.plan().kernelId]}
        g.prefill(value=float("nan"))
        g.launch(1.0, 0.0)
        entry["rel_err"] = gu.rel_err(g.result(), oc.conv_forward(x, w, pad=pad, stride=(1, 1), mode=1))
        ms = time_gpu(g, 1.0, 0.0, steps, warmup)
        entry.update({"ms": ms, "tflops": flops / ms / 1e9})
        other = "f32 64x64x72 taps9" if RS == 3 else "f32 32x128x32 tapmajor"
        g.handle.set_kernel_override(names.index(other))
        ms = time_gpu(g, 1.0, 0.0, steps, warmup)
        entry["pipelined_kernel"] = {"kernel": other, "ms": ms, "tflops": flops / ms / 1e9}
        out.append(entry)
    return out


def run_other_functions(steps, warmup):
    """The bandwidth-bound functions (activations, bias addition and bias gradient, softmax, pooling) on
    layer-sized float tensors: time per call, algorithmic bytes (each tensor once) per second
    against the 8 TB/s HBM peak, parity against the oracle on the first image(s)."""
    import numpy as np
    import torch
    import paper_1410_0759_amd as ig
    from oracle import pointwise_oracle as po
    from paper_1410_0759_amd import runner as gu

    HBM_PEAK = 8000.0   # GB/s
    rng = np.random.default_rng(14100759 * 10 + 900)
    h = ig.Handle()
    h.set_stream(torch.cuda.current_stream().cuda_stream)
    out = []

    def timed(call, steps=steps, warmup=warmup):
        return time_calls(call, steps, warmup)[0]

    def dev(a):
        t = torch.from_numpy(a).cuda()
        n, c, hh, ww = a.shape
        return t, ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, n, c, hh, ww, (c * hh * ww, hh * ww, ww, 1))

    def record(name, shape, nbytes, ms, err):
        out.append({"function": name, "shape": list(shape), "ms": ms, "algorithmic_bytes": nbytes,
                    "gb_per_s": nbytes / ms / 1e6, "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK, "rel_err": err})

    shape = (128, 64, 56, 56)
    x = rng.uniform(-3, 3, size=shape).astype(np.float32)
    xt, xd = dev(x)
    yt, yd = dev(np.zeros(shape, np.float32))
    nb = x.nbytes
    for mode, nm in ((ig.IGC_ACTIVATION_RELU, "relu"), (ig.IGC_ACTIVATION_TANH, "tanh")):
        call = lambda: ig.check(ig.activation_forward(h, mode, 1.0, xd, xt.data_ptr(), 0.0, yd, yt.data_ptr()), nm)
        ms = timed(call)
        err = gu.rel_err(yt[:2].cpu().numpy().astype(np.float64), po.activation_forward(mode, x[:2]))
        record("activation forward " + nm, shape, 2 * nb, ms, err)
    dyt, dyd = dev(rng.uniform(-1, 1, size=shape).astype(np.float32))
    dxt, dxd = dev(np.zeros(shape, np.float32))
    call = lambda: ig.check(ig.activation_backward(h, ig.IGC_ACTIVATION_TANH, 1.0, yd, yt.data_ptr(), dyd, dyt.data_ptr(),
                                                   xd, xt.data_ptr(), 0.0, dxd, dxt.data_ptr()), "tanh backward")
    ms = timed(call)
    err = gu.rel_err(dxt[:2].cpu().numpy().astype(np.float64),
                     po.activation_backward(po.TANH, yt[:2].cpu().numpy(), dyt[:2].cpu().numpy(), x[:2]))
    record("activation backward tanh", shape, 3 * nb, ms, err)
    bias = rng.uniform(-1, 1, size=(1, 64, 1, 1)).astype(np.float32)
    bt = torch.from_numpy(bias).cuda()
    bd = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, 1, 64, 1, 1, (64, 1, 1, 1))
    yt.copy_(xt)
    ig.check(ig.add_tensor(h, 1.0, bd, bt.data_ptr(), 1.0, yd, yt.data_ptr()), "bias")
    err = gu.rel_err(yt[:2].cpu().numpy().astype(np.float64), po.add_tensor(bias, (2,) + shape[1:], 1.0, 1.0, x[:2]))
    ms = timed(lambda: ig.check(ig.add_tensor(h, 1.0, bd, bt.data_ptr(), 1.0, yd, yt.data_ptr()), "bias"))
    record("bias addition in place (1,C,1,1)", shape, 2 * nb, ms, err)
    # the gradient with respect to that bias: dy summed per feature map (dy read once), with the workspace it asks for
    dbt = torch.zeros(64, dtype=torch.float32, device="cuda")
    dy_np = dyt.cpu().numpy()
    want_db = po.bias_backward(dy_np[:4])
    nhwc_dy = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, *shape, (shape[2] * shape[3] * shape[1], 1, shape[3] * shape[1], shape[1]))
    dy_nhwc = torch.from_numpy(np.ascontiguousarray(dy_np.transpose(0, 2, 3, 1))).cuda()
    for nm, desc, t in (("NCHW", dyd, dyt), ("NHWC", nhwc_dy, dy_nhwc)):
        few = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, 4, *shape[1:], desc.get()[2])   # (parity on four images)
        ws_bytes = ig.get_backward_bias_workspace_size(h, desc, bd)
        ws = torch.empty(max(ws_bytes, 8), dtype=torch.uint8, device="cuda")
        ig.check(ig.convolution_backward_bias(h, 1.0, few, t.data_ptr(), 0.0, bd, dbt.data_ptr(), ws.data_ptr(), ws_bytes), "bias gradient")
        err = gu.rel_err(dbt.cpu().numpy().astype(np.float64), want_db)
        ms = timed(lambda: ig.check(ig.convolution_backward_bias(h, 1.0, desc, t.data_ptr(), 0.0, bd, dbt.data_ptr(), ws.data_ptr(), ws_bytes),
                                    "bias gradient"))
        record("bias gradient, dy " + nm, shape, nb, ms, err)
    del dy_nhwc
    # change of layout: NCHW -> NHWC and back
    nhwc = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, *shape, (shape[2] * shape[3] * shape[1], 1, shape[3] * shape[1], shape[1]))
    ig.check(ig.transform_tensor(h, 1.0, xd, xt.data_ptr(), 0.0, nhwc, yt.data_ptr()), "to NHWC")
    ms = timed(lambda: ig.check(ig.transform_tensor(h, 1.0, xd, xt.data_ptr(), 0.0, nhwc, yt.data_ptr()), "to NHWC"))
    got = torch.as_strided(yt.view(-1), shape, (shape[2] * shape[3] * shape[1], 1, shape[3] * shape[1], shape[1]))[:2].cpu().numpy()
    record("tensor transformation NCHW -> NHWC", shape, 2 * nb, ms, gu.rel_err(got.astype(np.float64), po.add_tensor(x[:2], (2,) + shape[1:])))
    ms = timed(lambda: ig.check(ig.transform_tensor(h, 1.0, nhwc, yt.data_ptr(), 0.0, dxd, dxt.data_ptr()), "to NCHW"))
    record("tensor transformation NHWC -> NCHW", shape, 2 * nb, ms, gu.rel_err(dxt[:2].cpu().numpy().astype(np.float64), po.add_tensor(x[:2], (2,) + shape[1:])))
    del xt, yt, dyt, dxt

    for mode, nm, shape in ((ig.IGC_SOFTMAX_MODE_CHANNEL, "softmax per location", (32, 21, 128, 128)),
                            (ig.IGC_SOFTMAX_MODE_INSTANCE, "softmax per image", (256, 1000, 1, 1))):
        x = rng.uniform(-8, 8, size=shape).astype(np.float32)
        xt, xd = dev(x)
        yt, yd = dev(np.zeros(shape, np.float32))
        ms = timed(lambda: ig.check(ig.softmax_forward(h, mode, 1.0, xd, xt.data_ptr(), 0.0, yd, yt.data_ptr()), nm))
        err = gu.rel_err(yt[:2].cpu().numpy().astype(np.float64), po.softmax_forward(mode, x[:2]))
        record(nm, shape, 2 * x.nbytes, ms, err)
        dy = rng.uniform(-1, 1, size=shape).astype(np.float32)
        dyt, dyd = dev(dy)
        dxt, dxd = dev(np.zeros(shape, np.float32))
        ms = timed(lambda: ig.check(ig.softmax_backward(h, mode, 1.0, yd, yt.data_ptr(), dyd, dyt.data_ptr(), 0.0, dxd,
                                                        dxt.data_ptr()), nm))
        err = gu.rel_err(dxt[:2].cpu().numpy().astype(np.float64), po.softmax_backward(mode, yt[:2].cpu().numpy(), dy[:2]))
        record(nm + ", backward", shape, 3 * x.nbytes, ms, err)
        del xt, yt, dyt, dxt

    # bias addition and rectifier fused into the convolution's epilogue, against the three calls
    # one after the other, on the mid-layer workload
    import workloads as wl
    from oracle import conv_oracle as oc
    w_ = wl.by_index(3)
    cx, cw, _ = wl.make_inputs(w_)
    g = gu.GpuConv(cx, cw, (w_.pad_h, w_.pad_w), (w_.u, w_.v), w_.mode, dtype=w_.dtype, y_layout=w_.y_layout, handle=h)
    cb = rng.uniform(-1, 1, size=w_.K).astype(np.float32)
    g.prefill(value=float("nan"))
    g.launch_fused(1.0, 0.0, cb, ig.IGC_ACTIVATION_RELU)
    n = 2
    want = po.activation_forward(po.RELU, (oc.conv_forward(cx[:n], cw, pad=(w_.pad_h, w_.pad_w), stride=(w_.u, w_.v), mode=w_.mode)
                                           + po.add_tensor(cb.reshape(1, -1, 1, 1), (n, w_.K, w_.P, w_.Q))).astype(np.float32))
    err = gu.rel_err(g.result()[:n], want)
    bdev = g.bias_dev
    fused_call = lambda: ig.check(ig.convolution_bias_activation_forward(
        h, 1.0, g.xdesc, g.x_dev.data_ptr(), g.wdesc, g.w_dev.data_ptr(), g.conv, 0.0, bdev.data_ptr(),
        ig.IGC_ACTIVATION_RELU, g.ydesc, g.y_ptr), "fused")
    bdesc = ig.TensorDescriptor().set(ig.IGC_DATA_FLOAT, 1, w_.K, 1, 1, (w_.K, 1, 1, 1))

    def separate_calls():
        g.launch(1.0, 0.0)
        ig.check(ig.add_tensor(h, 1.0, bdesc, bdev.data_ptr(), 1.0, g.ydesc, g.y_ptr), "bias")
        ig.check(ig.activation_forward(h, ig.IGC_ACTIVATION_RELU, 1.0, g.ydesc, g.y_ptr, 0.0, g.ydesc, g.y_ptr), "relu")

    # (compute-bound: the clocks need about a hundred launches to settle)
    ms_fused, ms_sep = timed(fused_call, 150, 100), timed(separate_calls, 150, 100)
    out.append({"function": "convolution + bias + rectifier, fused epilogue (" + w_.name + ")", "ms": ms_fused,
                "ms_as_three_calls": ms_sep, "tflops": w_.flops / ms_fused / 1e9, "rel_err": err})
    del g

    shape = (128, 96, 55, 55)
    x = rng.uniform(-3, 3, size=shape).astype(np.float32)
    xt, xd = dev(x)
    for mode, nm in ((ig.IGC_POOLING_MAX, "max"), (ig.IGC_POOLING_AVERAGE, "average")):
        pool = ig.PoolingDescriptor().set(mode, 3, 3, 0, 0, 2, 2)
        oshape = ig.get_pooling_output_dim(pool, xd)
        yt, yd = dev(np.zeros(oshape, np.float32))
        ms = timed(lambda: ig.check(ig.pooling_forward(h, pool, 1.0, xd, xt.data_ptr(), 0.0, yd, yt.data_ptr()), nm))
        err = gu.rel_err(yt[:2].cpu().numpy().astype(np.float64), po.pooling_forward(mode, x[:2], (3, 3), (0, 0), (2, 2)))
        record("pooling 3x3 stride 2 " + nm, shape, x.nbytes + yt.numel() * 4, ms, err)
        dy = rng.uniform(-1, 1, size=oshape).astype(np.float32)
        dyt, dyd = dev(dy)
        dxt, dxd = dev(np.zeros(shape, np.float32))
        ms = timed(lambda: ig.check(ig.pooling_backward(h, pool, 1.0, dyd, dyt.data_ptr(), xd, xt.data_ptr(), 0.0, dxd,
                                                        dxt.data_ptr()), nm))
        err = gu.rel_err(dxt[:2].cpu().numpy().astype(np.float64), po.pooling_backward(mode, x[:2], dy[:2], (3, 3), (0, 0), (2, 2)))
        # (the average does not read x)
        record("pooling 3x3 stride 2 " + nm + ", backward", shape, (2 if mode == ig.IGC_POOLING_MAX else 1) * x.nbytes + dy.nbytes, ms, err)
        del yt, dyt, dxt
    del xt

    # the double-precision forms (same kernels compiled for double): one element-wise function and pooling
    def dev64(a):
        t = torch.from_numpy(a).cuda()
        n, c, hh, ww = a.shape
        return t, ig.TensorDescriptor().set(ig.IGC_DATA_DOUBLE, n, c, hh, ww, (c * hh * ww, hh * ww, ww, 1))

    shape = (128, 64, 56, 56)
    x = rng.uniform(-3, 3, size=shape)
    xt, xd = dev64(x)
    yt, yd = dev64(np.zeros(shape))
    ms = timed(lambda: ig.check(ig.activation_forward(h, ig.IGC_ACTIVATION_TANH, 1.0, xd, xt.data_ptr(), 0.0, yd, yt.data_ptr()), "tanh f64"))
    record("activation forward tanh, double precision", shape, 2 * x.nbytes, ms,
           gu.rel_err(yt[:1].cpu().numpy(), po.activation_forward(po.TANH, x[:1])))
    del xt, yt
    shape = (128, 96, 55, 55)
    x = rng.uniform(-3, 3, size=shape)
    xt, xd = dev64(x)
    pool = ig.PoolingDescriptor().set(ig.IGC_POOLING_MAX, 3, 3, 0, 0, 2, 2)
    oshape = ig.get_pooling_output_dim(pool, xd)
    yt, yd = dev64(np.zeros(oshape))
    ms = timed(lambda: ig.check(ig.pooling_forward(h, pool, 1.0, xd, xt.data_ptr(), 0.0, yd, yt.data_ptr()), "pool f64"))
    record("pooling 3x3 stride 2 max, double precision", shape, x.nbytes + yt.numel() * 8, ms,
           gu.rel_err(yt[:1].cpu().numpy(), po.pooling_forward(po.POOL_MAX, x[:1], (3, 3), (0, 0), (2, 2))))
    dy = rng.uniform(-1, 1, size=oshape)
    dyt, dyd = dev64(dy)
    dxt, dxd = dev64(np.zeros(shape))
    ms = timed(lambda: ig.check(ig.pooling_backward(h, pool, 1.0, dyd, dyt.data_ptr(), xd, xt.data_ptr(), 0.0, dxd, dxt.data_ptr()), "pool bwd f64"))
    record("pooling 3x3 stride 2 max, backward, double precision", shape, 2 * x.nbytes + dy.nbytes, ms,
           gu.rel_err(dxt[:1].cpu().numpy(), po.pooling_backward(po.POOL_MAX, x[:1], dy[:1], (3, 3), (0, 0), (2, 2))))
    return out


def run_batch_sweep(steps, warmup):
    """The paper's Table-2 layers at mini-batches of 16 .. 256 (its Section 4 reports 86 % of the
    best throughput at 16): mean TFLOP/s over the five layers per batch size, without a workspace
    and with the optional one.  Inputs are drawn once per layer for 256 images and the smaller
    batches take the first images; parity per (layer, batch) on one output row of the last image
    (computed by the oracle from the R input rows it depends on)."""
    import numpy as np
    import workloads as wl
    from oracle import conv_oracle as oc
    from paper_1410_0759_amd import runner as gu

    sizes = (16, 32, 64, 128, 256)
    rates = {nb: [] for nb in sizes}
    rates_ws = {nb: [] for nb in sizes}
    worst = 0.0
    for layer in wl.TABLE2_LAYERS:
        big = wl.shrink(layer, sizes[-1])
        x, w, _ = wl.make_inputs(big)
        for nb in sizes:
            w_ = wl.shrink(layer, nb)
            g = gu.GpuConv(x[:nb], w, (0, 0), (1, 1), w_.mode)
            g.prefill(value=float("nan"))
            g.launch(1.0, 0.0)
            prow = (7 * nb) % w_.P
            got = g.y_view()[nb - 1, :, prow, :].cpu().numpy().astype(np.float64)
            want = oc.conv_forward(x[nb - 1:nb, :, prow:prow + w_.R, :], w, pad=(0, 0), stride=(1, 1), mode=w_.mode)[0, :, 0, :]
            worst = max(worst, gu.rel_err(got, want))
            ms = time_calls(lambda: g.launch(1.0, 0.0), steps, warmup)[0]
            rates[nb].append(w_.flops / ms / 1e9)
            g.lend_workspace()
            ms = time_calls(lambda: g.launch(1.0, 0.0), steps, warmup)[0]
            rates_ws[nb].append(w_.flops / ms / 1e9)
            del g
    mean = {nb: sum(v) / len(v) for nb, v in rates.items()}
    mean_ws = {nb: sum(v) / len(v) for nb, v in rates_ws.items()}
    top, top_ws = max(mean.values()), max(mean_ws.values())
    return {
        "layers": "the paper's Table-2 layers, synthetic data", "mini_batches": list(sizes),
        "mean_tflops": [mean[nb] for nb in sizes], "fraction_of_best": [mean[nb] / top for nb in sizes],
        "mean_tflops_with_optional_workspace": [mean_ws[nb] for nb in sizes],
        "fraction_of_best_with_optional_workspace": [mean_ws[nb] / top_ws for nb in sizes],
        "per_layer_tflops": {str(nb): rates[nb] for nb in sizes},
        "per_layer_tflops_with_optional_workspace": {str(nb): rates_ws[nb] for nb in sizes},
        "worst_rel_err": worst, "paper": "86 % of its best throughput at a mini-batch of 16 (Section 4, Tesla K40)",
    }


def measured_traffic(workload, kernel):
    """HBM bytes per launch of the workload's kernel from the committed counter summary
    (profiles/hbm_traffic.json, written by bench_traffic.py from two rocprofv3 --pmc runs of this
    script: counters cannot be read from inside a timed run).  None when the summary is for another
    kernel than the one that just ran."""
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(tpath):
        return None
    with open(tpath) as fh:
        entry = json.load(fh).get(workload)
    if not entry or entry.get("kernel") != kernel:
        return None
    return entry.get("bytes_per_launch")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=2, help="headline workload (1-5)")
    ap.add_argument("--only", action="store_true", help="time the headline workload only")
    ap.add_argument("--no-batch-sweep", action="store_true", help="skip the mini-batch sweep over the Table-2 layers")
    ap.add_argument("--batch-sweep-only", action="store_true", help="time only that sweep")
    ap.add_argument("--no-table2", action="store_true", help="skip the paper's Table-2 layer collection")
    ap.add_argument("--no-backward", action="store_true", help="skip the backward-data / backward-filter section")
    ap.add_argument("--backward-only", type=int, default=0, help="time only the backward passes of this workload (1-5)")
    ap.add_argument("--no-other", action="store_true", help="skip the section on activations, softmax, pooling, bias addition")
    ap.add_argument("--other-only", action="store_true", help="time only that section")
    ap.add_argument("--f64-only", action="store_true", help="time only the double-precision section")
    ap.add_argument("--table2-only", action="store_true", help="time only the paper's Table-2 layer collection")
    ap.add_argument("--padded-only", action="store_true", help="time only the padded 5x5 / 7x7 layers")
    ap.add_argument("--small-only", action="store_true", help="time only the padded layers at serving mini-batches")
    ap.add_argument("--kernel", type=int, default=None, help="force a kernel id for the headline workload")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (a known-size reference "
                         "for the profiler's HBM byte counters)")
    ap.add_argument("--oracle-seconds", type=float, default=12.0, help="CPU budget of the headline oracle run")
    ap.add_argument("--clock-warmup-ms", type=int, default=CLOCK_WARMUP_MS,
                    help="milliseconds of untimed repetitions of the call before every timed region (0: none)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    _warm["ms"] = args.clock_warmup_ms

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    import paper_1410_0759_amd as ig
    import workloads as wl

    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.backward_only:
        big = wl.shrink(wl.by_index(5), 256) if args.backward_only == 6 else None     # (6: the bf16 workload at a mini-batch of 256)
        print(json.dumps(run_backward(args.backward_only, args.steps, args.warmup, 1.0, workload=big)))
        return
    if args.other_only:
        print(json.dumps(run_other_functions(max(20, args.steps // 5), max(10, args.warmup // 5))))
        return
    if args.f64_only:
        print(json.dumps([run_double_precision(max(20, args.steps // 10), max(10, args.warmup // 5), i) for i in (3, 4)]))
        return
    if args.table2_only:
        print(json.dumps([run_config(None, args.steps, args.warmup, 1.0, workload=w_) for w_ in wl.TABLE2_LAYERS]))
        return
    if args.padded_only:
        print(json.dumps(run_padded_filters(max(10, args.steps // 10), max(10, args.warmup // 5))))
        return
    if args.small_only:
        print(json.dumps(run_small_layers(max(10, args.steps // 10), max(10, args.warmup // 5))))
        return
    if args.batch_sweep_only:
        print(json.dumps(run_batch_sweep(max(10, args.steps // 10), max(5, args.warmup // 10))))
        return

    # The arithmetic ceiling at the clocks this chip sustains: a register-only loop of each data
    # type's MFMA instruction (no memory traffic), beside the datasheet peaks the fractions use.
    h = ig.Handle()
    h.set_stream(torch.cuda.current_stream().cuda_stream)
    cus, khz = ig.get_device_properties(h)
    # The same loop with pseudo-random operands that change with every instruction, as a real product's do: the matrix
    # pipes draw more power and the chip sustains lower clocks (bf16: about 0.7 of the rate with uniform operands).
    achievable, achievable_random = {}, {}
    if not args.only:
        for name, dt in (("f32", ig.IGC_DATA_FLOAT), ("bf16", ig.IGC_DATA_BFLOAT16), ("f64", ig.IGC_DATA_DOUBLE)):
            ig.measure_matrix_rate(h, dt, 30)
            achievable[name] = ig.measure_matrix_rate(h, dt, 100)
            ig.measure_matrix_rate_operands(h, dt, 30, 1)
            achievable_random[name] = ig.measure_matrix_rate_operands(h, dt, 100, 1)

    head = run_config(args.config, args.steps, args.warmup, args.oracle_seconds, args.kernel)
    per_config = []
    if not args.only:
        for i in range(1, 6):
            per_config.append(head if i == args.config else run_config(i, args.steps, args.warmup, 3.0))

    # The bf16 workload again at a mini-batch of 256: at N = 32 it has 200 tiles for 256 compute
    # units and 12 us of work at peak; this shows the same kernels with the chip filled.
    bf16_large = None
    if not args.only:
        bf16_large = run_config(None, max(30, args.steps // 3), max(20, args.warmup // 2), 1.0,
                                workload=wl.shrink(wl.by_index(5), 256))

    # The paper's own layer collection (its Table 2) with synthetic data, beside the numbers
    # its Table 3 reports for 2014 hardware.
    table2 = []
    if not args.only and not args.no_table2:
        for i, w_ in enumerate(wl.TABLE2_LAYERS):
            r = run_config(None, max(20, args.steps // 10), max(10, args.warmup // 5), 1.0, workload=w_)
            r["paper_tflops"] = {hw: v[i] for hw, v in wl.TABLE3_PAPER_TFLOPS.items()}
            table2.append(r)

    # The two backward passes at the sizes of workloads 2-5 (same FLOP count as forward).
    backward = []
    if not args.only and not args.no_backward:
        for i in (2, 3, 4, 5):
            backward.append(run_backward(i, max(20, args.steps // 2), max(10, args.warmup // 2), 1.0))
        backward.append(run_backward(None, max(20, args.steps // 5), max(10, args.warmup // 5), 1.0, workload=wl.shrink(wl.by_index(5), 256)))

    padded = []
    if not args.only and not args.no_backward and not args.no_table2:
        padded = run_padded_filters(max(10, args.steps // 10), max(10, args.warmup // 5))

    small = []
    if not args.only and not args.no_table2:
        small = run_small_layers(max(10, args.steps // 10), max(10, args.warmup // 5))

    other = []
    double_precision = None
    if not args.only and not args.no_other:
        other = run_other_functions(max(20, args.steps // 5), max(10, args.warmup // 5))
        double_precision = [run_double_precision(max(20, args.steps // 10), max(10, args.warmup // 5), i) for i in (3, 4)]

    batch_sweep = None
    if not args.only and not args.no_batch_sweep and not args.no_table2:
        batch_sweep = run_batch_sweep(max(10, args.steps // 10), max(5, args.warmup // 10))

    def compact(r):
        return {"workload": r["workload"], "dtype": r["dtype"], "ms": r["ms"], "median_ms": r["median_ms"], "min_ms": r["min_ms"],
                "tflops": r["tflops"], "peak": r["peak_tflops"], "frac": r["frac_of_peak"],
                "frac_at_median": r["gflop"] / r["median_ms"] / r["peak_tflops"],
                "frac_of_achievable_with_random_operands": (r["tflops"] / achievable_random[r["dtype"]]) if achievable_random.get(r["dtype"]) else None,
                "rel_err": r["rel_err"], "tolerance": r["tolerance"], "kernel": r["kernel"], "workspace_bytes": 0}

    roofline = {"bound": "mfma", "achieved": head["tflops"], "peak": head["peak_tflops"],
                "unit": "TFLOP/s", "frac": head["frac_of_peak"], "traffic": measured_traffic(head["workload"], head["kernel"]),
                "algorithmic_bytes": head["algorithmic_bytes"], "kernel": head["kernel"],
                "ms_mean": head["ms"], "ms_median": head["median_ms"], "ms_min": head["min_ms"],
                "per_config": [compact(r) for r in per_config],
                "target": ">= 0.5 of the matrix peak on cfg 2-4",
                "target_met": bool(per_config) and all(r["frac_of_peak"] >= 0.5 for r in per_config[1:4]),
                "achievable_peak": achievable,
                "achievable_peak_note": "register-only MFMA loop, two wavefronts per SIMD, measured in this run (TFLOP/s)",
                "achievable_peak_random_operands": achievable_random,
                "achievable_peak_random_operands_note": "the same loop with pseudo-random operands, another register set with every "
                                                        "instruction: the ceiling with real data at the clocks the chip then sustains"}
    if bf16_large:
        roofline["bf16_workload_at_mini_batch_256"] = compact(bf16_large)
    if batch_sweep:
        roofline["table2_mini_batch_16_fraction_of_best"] = batch_sweep["fraction_of_best"][0]
        roofline["table2_mini_batch_16_fraction_of_best_with_optional_workspace"] = batch_sweep["fraction_of_best_with_optional_workspace"][0]

    out = {
        "metric": "conv forward effective TFLOP/s and fraction of MI355X matrix peak",
        "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic (seeded)",
        "config": {"workload": head["workload"], "kernel": head["kernel"], "grid": head["grid"],
                   "parallelism": "single GPU", "workspace_bytes": 0, "copy_probe_mib": args.copy_probe_mib,
                   "clock_warmup_ms": args.clock_warmup_ms,
                   "clock_warmup": "the call itself repeated for that long before the warm-up steps of each timed region, untimed (the chip idles while inputs are drawn and the oracle runs)"},
        "frac_of_peak": head["frac_of_peak"], "rel_err_vs_oracle": head["rel_err"],
        "roofline": roofline,
        "cpu_baseline": {"value": head["oracle_tflops"], "unit": "TFLOP/s", "cores": head["oracle_threads"],
                         "kind": "oracle",
                         "sample": "first %d of the workload's images, whole output of those images, %.2f s"
                                   % (head["parity_images"], head["oracle_seconds"])},
        "device": {"name": props.name, "compute_units": cus, "clock_mhz": khz / 1e3},
        "per_config": per_config,
        "bf16_workload_at_mini_batch_256": bf16_large,
        "table2_layers": table2,
        "table2_batch_sweep": batch_sweep,
        "backward": backward,
        "padded_filter_layers": padded,
        "small_mini_batch_layers": small,
        "other_functions": other,
        "double_precision": double_precision,
        "paper_context": "paper Table 3: 0.99-1.52 TFLOP/s (23-35% of 4.29) on Tesla K40, 1.46-2.49 (30-51% of 4.95) "
                         "on GTX 980, fp32, its own Table-2 layers",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
