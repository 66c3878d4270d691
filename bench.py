#!/usr/bin/env python3
"""Benchmark: VGG-16 per-layer training compute (conv + FC, forward and backward) at the
strong-scaling per-GPU batches 1..32 on one MI355X.

A step = one pass of the whole hot path: for every per-GPU batch N in {1,2,4,8,16,32}: forward
through the 16 compute layers (bias+ReLU fused), then backward from the last layer: per layer
backward-data, whose epilogue also applies the backward of the ReLU in front of the layer
(dx *= [x > 0], DP_RELU_IN), and, on a side stream, backward-filter with the bias gradient.  The
gradient a layer receives is therefore already masked by its own output: every ReLU of the network is
differentiated once, by the layer behind it, and no layer needs a pointwise pass of its own.  The first
layer needs no backward-data (a training step never uses the gradient of the input image).  Inputs are
seeded synthetic tensors already resident in HBM.
value = nominal flops of the step / time (TFLOP/s); nominal flops per pass =
2*N*Ho*Wo*K*R*S*C (padding taps counted), three passes per layer (two for the first).

Prints ONE JSON line: metric, value (TFLOP/s), ms_per_step, per_batch, roofline, cpu_baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a 1 GiB copy kernel), averaged over
# the launches of each kernel at one per-GPU batch: profiles/vgg16_hbm_traffic.md
TRAFFIC_BYTES_PER_LAUNCH = {   # key: "<kernel as the profiler prints it>@<per-GPU batch>"
    "k_wgrad_dma<128, 128, 32, 2, 2, 2>@32": 275078599,
    "k_reduce_flat@32": 60161969,
    "k_wgrad_dma<256, 256, 64, 2, 4, 2>@32": 177667828,
    "k_wgrad_dma<128, 128, 64, 2, 2, 2>@32": 259377408,
    "k_reduce_pixel_major@32": 27174872,
    "k_conv_strip<true, 224, 256>@32": 171644633,
    "k_conv_strip<false, 224, 256>@32": 121469231,
    "k_wgrad_halo9<true>@32": 320878204,
    "k_conv_strip<true, 256, 128>@32": 185911535,
    "k_halo_ws<0, false>@32": 283800783,
    "k_dgrad_dma<64, 128, 64, 2, 2, 2, 1>@32": 164571708,
    "k_halo_ws<1, true>@32": 618192570,
    "k_fwd_dma<128, 128, 64, 2, 2, 2, 1>@32": 146734142,
    "k_fwd_dma<64, 128, 64, 2, 2, 2, 1>@32": 95860080,
    "k_dgrad_dma<64, 64, 64, 2, 2, 2, 2>@32": 157534286,
    "k_conv_strip<false, 256, 128>@32": 147696706,
    "k_conv_strip<true, 128, 256>@32": 132799145,
    "k_reduce_flat_wide@32": 48001240,
    "k_fwd_dma<64, 64, 64, 2, 2, 3, 1>@32": 99755382,
    "k_wgrad_dma<64, 256, 32, 1, 4, 2>@32": 424924068,
    "k_dgrad_dma<64, 64, 64, 2, 2, 3, 1>@32": 114982045,
    "k_fwd_rgb3@32": 230225985,
    "k_fwd_dma<64, 64, 64, 2, 2, 2, 4>@32": 74369407,
    "k_wgrad_rgb3<true>@32": 220898337,
    "k_dense_wgrad<true>@32": 69690728,
    "k_dense_wgrad<false>@32": 18710094,
    "k_dense_dgrad@32": 9297571,
    "k_wgrad_direct_sum@32": 4291674,
    "k_wgrad_dma<128, 128, 32, 2, 2, 2>@2": 131164048,
    "k_wgrad_dma<128, 64, 32, 2, 2, 2>@2": 80393531,
    "k_reduce_flat@2": 27498692,
    "k_dgrad_dma<64, 64, 64, 2, 2, 2, 2>@2": 54995695,
    "k_wgrad_dma<64, 128, 64, 2, 2, 2>@2": 39431809,
    "k_reduce_pixel_major@2": 9790902,
    "k_reduce_flat_wide@2": 22073797,
    "k_wgrad_dma<64, 64, 32, 2, 2, 2>@2": 35385434,
    "k_dgrad_dma<64, 64, 64, 2, 2, 2, 4>@2": 42727728,
    "k_dgrad_dma<128, 64, 64, 2, 2, 2, 1>@2": 53431899,
    "k_dgrad_dma<64, 64, 64, 2, 2, 3, 1>@2": 45686533,
    "k_dgrad_dma<128, 64, 64, 2, 2, 2, 2>@2": 56822772,
    "k_fwd_dma<64, 64, 64, 2, 2, 2, 2>@2": 31871907,
    "k_conv_fast<0, 64, 64, 64, 2, 2>@2": 28739201,
    "k_dense_fwd<1>@2": 82874842,
    "k_fwd_dma<64, 64, 64, 2, 2, 2, 4>@2": 33982470,
    "k_conv_fast<1, 128, 64, 64, 2, 2>@2": 68977417,
    "k_fwd_dma<128, 64, 64, 2, 2, 2, 1>@2": 30056766,
    "k_dgrad_dma<128, 64, 128, 2, 2, 2, 1>@2": 79696568,
    "k_wgrad_halo@2": 45397162,
    "k_fwd_dma<64, 64, 64, 2, 2, 3, 1>@2": 25019716,
    "k_wgrad_halo9<true>@2": 34065730,
    "k_dense_wgrad<true>@2": 67487480,
    "k_conv_fast<0, 128, 64, 64, 2, 2>@2": 19960021,
    "k_halo<0, 64, 1, 4, 3>@2": 17366213,
    "k_halo<1, 64, 1, 4, 4>@2": 39682413,
    "k_dgrad_dma<64, 64, 128, 2, 2, 3, 1>@2": 17234433,
    "k_halo_ws<1, true>@2": 39764571,
    "k_fwd_dma<64, 128, 128, 2, 2, 2, 1>@2": 14300926,
    "k_fwd_dma<64, 64, 128, 2, 2, 3, 1>@2": 20039705,
    "k_halo<0, 64, 1, 4, 2>@2": 20847855,
    "k_dgrad_dma<64, 128, 128, 2, 2, 2, 1>@2": 18350732,
    "k_dense_wgrad<false>@2": 16628633,
    "k_fwd_rgb3@2": 14118188,
    "k_wgrad_rgb3<true>@2": 15733105,
    "k_dense_dgrad@2": 8326932,
    "k_wgrad_direct_sum@2": 1706703,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batches", type=str, default="1,2,4,8,16,32")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--side-streams", type=int, default=2, help="streams that run the filter gradients beside the backward chain (0: everything on one stream)")
    ap.add_argument("--launch", type=str, default="auto", choices=["auto", "eager", "graph"],
                    help="auto: per batch, one small HIP graph per sub-step if it replays faster than launching the kernels one by one")
    ap.add_argument("--no-graph", action="store_true", help="same as --launch eager")
    ap.add_argument("--no-table", action="store_true", help="skip the dp_profile_layer table")
    ap.add_argument("--fg-batch", type=int, default=2, help="--multiplex: per-GPU batch of the foreground VGG-16 step")
    ap.add_argument("--bg-batch", type=int, default=64, help="--multiplex: batch of the background ResNet-50 step")
    ap.add_argument("--pace", type=int, default=2, help="--multiplex: most un-finished launches the background queue may hold")
    ap.add_argument("--graph-piece", type=int, default=8, help="--multiplex: library calls per small foreground graph")
    ap.add_argument("--multiplex", action="store_true",
                    help="single-GPU multiplexing run instead of the sweep: foreground VGG-16 step at batch 2 beside a background ResNet-50 step at batch 64")
    ap.add_argument("--workload", type=str, default="vgg16", choices=["vgg16", "resnet50", "inception", "wrn101_2"],
                    help="layer list; the metric and the default run are VGG-16, the others emit their own tables")
    ap.add_argument("--layers", type=str, default="", help="comma-separated layer names: run only these (profiling aid)")
    ap.add_argument("--calibrate-copy-mb", type=int, default=0,
                    help="profiling aid: also run an elementwise fp32 copy kernel that reads and writes this many MiB")
    ap.add_argument("--autotune", type=str, default="cold", choices=["warm", "cold"],
                    help="measured kernel choice: time the candidates back to back (warm) or with the caches flushed before every timed launch (cold: "
                         "the state a layer meets inside a step)")
    ap.add_argument("--no-autotune", action="store_true",
                    help="keep the analytic kernel choice instead of timing the candidates once per layer shape before the warm-up")
    ap.add_argument("--no-glue", action="store_true", help="skip the separate timing of pooling, loss and SGD update")
    ap.add_argument("--table", type=str, default="", help="also write the per-layer time-vs-batch table (JSON) here")
    args = ap.parse_args()
    if args.no_graph:
        args.launch = "eager"
    return args


class _BindProxy:
    """Stands in for the binding module: every dp_* call is turned into a pre-marshalled callable."""

    def __init__(self, dp, out):
        self._dp, self._out = dp, out

    def __getattr__(self, name):
        attr = getattr(self._dp, name)
        if not name.startswith("dp_"):
            return attr

        def rec(*args, **kw):
            import inspect
            ba = inspect.signature(attr).bind(*args, **kw)
            ba.apply_defaults()
            self._out.append(self._dp.bind(name, *ba.args))
        return rec


class Layer:
    """Device tensors of one layer at the largest batch; smaller batches use the leading samples."""

    def __init__(self, torch, dp, spec, nmax, gen, dev, is_conv):
        self.spec, self.is_conv, self.name = spec, is_conv, spec.name
        bf = torch.bfloat16
        if is_conv:
            l = spec
            self.ho = (l.h + 2 * l.ph - l.r) // l.sh + 1
            self.wo = (l.w + 2 * l.pw - l.s) // l.sw + 1
            fan_in = l.r * l.s * l.c
            self.x = torch.randn((nmax, l.h, l.w, l.c), generator=gen, device=dev, dtype=torch.float32).to(bf)
            self.w = (torch.randn((l.k, l.r, l.s, l.c), generator=gen, device=dev) * (2.0 / fan_in) ** 0.5).to(bf)
            self.dy = torch.randn((nmax, self.ho, self.wo, l.k), generator=gen, device=dev, dtype=torch.float32).to(bf)
            self.y = torch.empty((nmax, self.ho, self.wo, l.k), device=dev, dtype=bf)
            self.dx_f32 = l.c < 8   # first layer: input gradient kept in fp32 (bf16 cannot resolve it to the parity tolerance; a training step never needs it)
            self.dx = torch.empty((nmax, l.h, l.w, l.c), device=dev, dtype=torch.float32 if self.dx_f32 else bf)
            self.dw = torch.empty((l.k, l.r, l.s, l.c), device=dev, dtype=torch.float32)
            self.k = l.k
        else:
            l = spec
            self.x = torch.randn((nmax, l.in_f), generator=gen, device=dev, dtype=torch.float32).to(bf)
            self.w = (torch.randn((l.out_f, l.in_f), generator=gen, device=dev) * (2.0 / l.in_f) ** 0.5).to(bf)
            self.dy = torch.randn((nmax, l.out_f), generator=gen, device=dev, dtype=torch.float32).to(bf)
            self.y = torch.empty((nmax, l.out_f), device=dev, dtype=bf)
            self.dx = torch.empty((nmax, l.in_f), device=dev, dtype=bf)
            self.dw = torch.empty((l.out_f, l.in_f), device=dev, dtype=torch.float32)
            self.k = l.out_f
        self.bias = (torch.rand((self.k,), generator=gen, device=dev) * 0.2 - 0.1).float()
        self.db = torch.empty((self.k,), device=dev, dtype=torch.float32)
        self.needs_dx = not (is_conv and spec.c < 8)  # the network input needs no gradient

    def desc(self, dp, n):
        l = self.spec
        if self.is_conv:
            flags = (dp.DP_BIAS if l.bias else 0) | dp.DP_RELU | (dp.DP_DX_F32 if self.dx_f32 else 0)
            flags |= dp.DP_RELU_IN if self.needs_dx else 0
            return dp.conv_desc(n, l.h, l.w, l.c, l.k, l.r, l.s, (l.sh, l.sw), (l.ph, l.pw), dp.DP_BF16, flags)
        return dp.linear_desc(n, l.in_f, l.out_f, dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU | dp.DP_RELU_IN)

    def flops(self, n):
        l = self.spec
        if self.is_conv:
            return 2.0 * n * self.ho * self.wo * l.k * l.r * l.s * l.c
        return 2.0 * n * l.in_f * l.out_f

    def ws_bytes(self, dp, n):
        d = self.desc(dp, n)
        rb = dp.dp_relu_bias_grad_workspace_bytes(self.rows(n), self.k)
        if self.is_conv:
            return max(rb, *(dp.dp_conv2d_workspace_bytes(d, p) for p in range(3)))
        return max(rb, dp.dp_linear_workspace_bytes(d))

    def rows(self, n):
        return n * self.ho * self.wo if self.is_conv else n

    # the three passes; each is one library call
    def fwd(self, dp, d, ws, stream=None):
        if self.is_conv:
            dp.dp_conv2d_fwd(d, self.x, self.w, self.bias if self.spec.bias else None, self.y, ws, stream)
        else:
            dp.dp_linear_fwd_bwd(d, x=self.x, W=self.w, bias=self.bias, y=self.y, ws=ws, stream=stream)

    # Every layer but the first reads the output of a ReLU (directly or max-pooled).  Its backward-data call
    # applies that ReLU's backward in its epilogue (DP_RELU_IN: dx *= [x > 0]), so the gradient a layer
    # receives (dy here) is already masked by its own output and no layer runs a pointwise pass of its own;
    # each of the 15 ReLUs of the network is differentiated exactly once, by the layer behind it.
    def dgrad(self, dp, d, ws, stream=None):
        if self.is_conv:
            dp.dp_conv2d_bwd_data_relu(d, self.dy, None, self.w, self.x, self.dx, ws, stream)
        else:
            dp.dp_linear_fwd_bwd(d, x=self.x, W=self.w, dy=self.dy, dx=self.dx, ws=ws, stream=stream)

    def wgrad(self, dp, d, ws, stream=None):
        """Filter and bias gradient from the (already masked) incoming gradient."""
        if self.is_conv:
            dp.dp_conv2d_bwd_filter(d, self.x, self.dy, None, self.dw, self.db, ws, stream)
        else:
            dp.dp_linear_fwd_bwd(d, x=self.x, dy=self.dy, dW=self.dw, dbias=self.db, ws=ws, stream=stream)

    def bound(self, which, dp, d, ws, stream):
        """Zero-argument callable issuing the C call of pass `which` (arguments marshalled once)."""
        rec = []
        getattr(self, which)(_BindProxy(dp, rec), d, ws, stream)
        return rec[0]

    def passes(self):
        """(name, method, counts nominal flops) of the calls that make up this layer's share of a step."""
        out = [("fwd", self.fwd, True)]
        if self.needs_dx:
            out.append(("dgrad", self.dgrad, True))
        out.append(("wgrad", self.wgrad, True))
        return out

    def step_flops(self, n):
        return self.flops(n) * sum(1 for _, _, c in self.passes() if c)


def glue_times(dp, torch, dev, batches):
    """The layers between the conv/FC layers of a whole VGG-16 step, timed apart from the headline step
    (they carry no nominal flops): the five 2x2 max-pools forward + backward per batch, the loss, and one
    SGD-with-momentum update of all 138 M parameters.  HIP events around 10 back-to-back launches each."""
    pools = [(224, 64), (112, 128), (56, 256), (28, 512), (14, 512)]
    stream = torch.cuda.current_stream()

    def timed(fn, reps=10):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    out = {"pool_fwd_bwd_us": {}, "loss_us": {}}
    nmax = max(batches)
    bufs = []
    for hw, c in pools:
        x = torch.relu(torch.randn((nmax, hw, hw, c), device=dev)).to(torch.bfloat16)
        dy = torch.randn((nmax, hw // 2, hw // 2, c), device=dev).to(torch.bfloat16)
        bufs.append((hw, c, x, dy, torch.empty_like(dy), torch.empty_like(x)))
    z = torch.randn((nmax, 1000), device=dev).to(torch.bfloat16)
    labels = torch.arange(nmax, device=dev, dtype=torch.int32) % 1000
    loss, dz = torch.zeros(4, device=dev), torch.empty_like(z)
    for n in batches:
        def pool_pass():
            for hw, c, x, dy, y, dx in bufs:
                dp.dp_maxpool2x2_fwd(n, hw, hw, c, dp.DP_BF16, x, y)
                dp.dp_maxpool2x2_bwd(n, hw, hw, c, dp.DP_BF16, x, dy, dx)
        out["pool_fwd_bwd_us"][str(n)] = timed(pool_pass)
        out["loss_us"][str(n)] = timed(lambda: dp.dp_softmax_xent(n, 1000, dp.DP_BF16, z, labels, loss, dz))
    # HBM figure of the largest pool at the largest batch: forward reads x and writes y (1.25 x), backward
    # reads x and dy and writes dx (2.25 x)
    hw, c, x, dy, y, dx = bufs[0]
    t = timed(lambda: (dp.dp_maxpool2x2_fwd(nmax, hw, hw, c, dp.DP_BF16, x, y), dp.dp_maxpool2x2_bwd(nmax, hw, hw, c, dp.DP_BF16, x, dy, dx)))
    out["pool1_gb_per_s"] = 3.5 * x.numel() * 2 / t / 1e3
    del bufs, x, dy, y, dx
    from paper_2112_10065_amd import workloads as W
    count = W.vgg16_param_count()
    g = torch.randn(count, device=dev)
    m, w32, w16 = torch.zeros_like(g), torch.randn(count, device=dev), torch.empty(count, device=dev, dtype=torch.bfloat16)
    t = timed(lambda: dp.dp_sgd_update(count, 0.01, 0.9, g, m, w32, w16))
    out["sgd_update_us"] = t
    out["sgd_gb_per_s"] = 22.0 * count / t / 1e3   # reads grad, momentum, weights; writes momentum, weights, bf16 copy
    out["hbm_peak_gb_per_s"] = 8000.0
    return out


def cpu_baseline():
    """Time the fp64 oracle (as it stands) on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    from paper_2112_10065_amd import synth
    sample = [("conv2_2", 112, 128, 128, 2), ("conv3_2", 56, 256, 256, 8), ("conv4_2", 28, 512, 512, 8), ("conv5_1", 14, 512, 512, 8)]
    flops, secs = 0.0, 0.0
    for name, hw, c, k, n in sample:
        x, w, b = synth.conv_tensors(f"vgg/{name}", n, hw, hw, c, k, 3, 3)
        x, w = synth.round_bf16(x), synth.round_bf16(w)
        dy = synth.round_bf16(synth.upstream_grad(f"vgg/{name}", (n, hw, hw, k)))
        t0 = time.perf_counter()
        y = oracle.conv2d_fwd(x, w, b, relu=True, pad=(1, 1))
        oracle.conv2d_bwd_data(dy, w, x.shape, y_saved=y, pad=(1, 1))
        oracle.conv2d_bwd_filter(x, dy, w.shape, y_saved=y, pad=(1, 1), want_db=True)
        secs += time.perf_counter() - t0
        flops += 3 * 2.0 * n * hw * hw * k * 9 * c
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": "fp64 nested-loop oracle, fwd+dgrad+wgrad of VGG-16 " + ", ".join(f"{nm} (N={n})" for nm, _, _, _, n in sample) + "; "
                      f"{flops / 1e9:.1f} GFLOP nominal in {secs:.1f} s"}


def median(v):
    v = sorted(v)
    return v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2])


def algorithmic_bytes(l, n, pname):
    """Algorithmic HBM bytes of one pass (bf16 tensors, fp32 filter / bias gradients): what the pass must read and write."""
    sp = l.spec
    if l.is_conv:
        xe, we, ye = n * sp.h * sp.w * sp.c, sp.k * sp.r * sp.s * sp.c, n * l.ho * l.wo * sp.k
    else:
        xe, we, ye = n * sp.in_f, sp.out_f * sp.in_f, n * sp.out_f
    if pname == "fwd":
        return 2.0 * (xe + we + ye) + 4.0 * l.k
    if pname == "dgrad":
        return 2.0 * (ye + we + xe) + 2.0 * xe      # + the saved input read by the fused ReLU backward
    return 2.0 * (xe + ye) + 4.0 * we + 4.0 * l.k


RIDGE_FLOP_PER_BYTE = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)


def roofline_objects(trace, layers, n):
    """The two roofline objects of per-GPU batch n from the per-kernel trace.  A call (layer, pass) is bound by the
    matrix cores when its flops / algorithmic bytes exceed the ridge of the two peaks, else by HBM; the calls of each
    class are grouped by the kernel name the profiler prints.  Dominant = largest summed main-kernel duration over
    all layers and passes of the class."""
    groups = {"mfma": {}, "hbm": {}}
    total_us = 0.0
    for l in layers:
        for pname, _, _ in l.passes():
            rows = trace.get((l.name, n, pname))
            if not rows:
                continue
            fl, by = l.flops(n), algorithmic_bytes(l, n, pname)
            bound = "mfma" if fl / by >= RIDGE_FLOP_PER_BYTE else "hbm"
            g = groups[bound].setdefault(rows[0]["kernel"], {"us": 0.0, "launches": 0, "flops": 0.0, "bytes": 0.0, "calls": []})
            main = median([r["main_us"] for r in rows])
            total_us += main
            g["us"] += main
            g["launches"] += 1
            g["flops"] += fl
            g["bytes"] += by
            g["calls"].append(f"{l.name}.{pname}")
    out = {}
    for bound in ("mfma", "hbm"):
        if not groups[bound]:
            out[bound] = None
            continue
        kname, g = max(groups[bound].items(), key=lambda kv: kv[1]["us"])
        if bound == "mfma":
            achieved, peak, unit = g["flops"] / g["us"] / 1e6, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
        else:
            achieved, peak, unit = g["bytes"] / g["us"] / 1e3, HBM_PEAK_GBS, "GB/s"
        out[bound] = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                      "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(f"{kname}@{n}"),
                      "kernel": kname, "samples_per_launch": n, "avg_launch_us": g["us"] / g["launches"], "launches_per_step": g["launches"],
                      "flops_per_launch_avg": g["flops"] / g["launches"], "algorithmic_bytes_per_launch_avg": g["bytes"] / g["launches"],
                      "share_of_batch_kernel_time": g["us"] / total_us, "calls": g["calls"]}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1).", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2112_10065_amd import binding as dp, workloads as W

    if not torch.cuda.is_available():
        print("no GPU visible: the HIP library cannot run", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.multiplex:
        from paper_2112_10065_amd import multiplex
        print(json.dumps(multiplex.run(args, dp, torch, dev, Layer)))
        return
    gen = torch.Generator(device=dev)
    gen.manual_seed(20211210)
    batches = [int(b) for b in args.batches.split(",")]
    nmax = max(batches)

    keep = set(args.layers.split(",")) if args.layers else None
    convs = {"vgg16": W.vgg16_convs, "resnet50": W.resnet50_convs, "inception": W.inception_convs, "wrn101_2": W.wrn101_2_convs}[args.workload]()
    linears = W.vgg16_linears() if args.workload == "vgg16" else []
    layers = [Layer(torch, dp, l, nmax, gen, dev, True) for l in convs if keep is None or l.name in keep]
    layers += [Layer(torch, dp, l, nmax, gen, dev, False) for l in linears if keep is None or l.name in keep]
    # Measured kernel choice: the first call per (layer, batch, pass) times the planner's candidates.
    # It is switched on before the workspace query (the query then covers every candidate).
    dp.dp_set_autotune(0 if args.no_autotune else 2 if args.autotune == "cold" else 1)
    ws_bytes = max(l.ws_bytes(dp, n) for l in layers for n in batches)
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=dev)
    descs = {(l.name, n): l.desc(dp, n) for l in layers for n in batches}

    if not args.no_autotune:
        # one call of every pass, alone on the GPU, so that each measurement sees an idle device
        for n in batches:
            for l in layers:
                for _, fn, _ in l.passes():
                    fn(dp, descs[(l.name, n)], ws)
                    torch.cuda.synchronize()

    if args.calibrate_copy_mb > 0:
        # known-size traffic for scaling the profiler's FETCH_SIZE / WRITE_SIZE counters; in a kernel
        # trace it also separates the measured-choice launches above from the steps below
        n_el = args.calibrate_copy_mb * (1 << 20) // 4
        src = torch.ones(n_el, device=dev, dtype=torch.float32)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    n_side = max(0, args.side_streams)
    ws_side = [torch.empty(ws_bytes + 256, dtype=torch.uint8, device=dev) for _ in range(n_side)]
    side_streams = [torch.cuda.Stream() for _ in range(n_side)]   # default priority

    def build_batch(n, main):
        """Pre-marshalled launch list of the sub-step of per-GPU batch n on stream `main` (+ the side streams):
        forward through the layers, then backward from the last layer; a layer's filter gradient depends only on
        that layer's (already masked) incoming gradient, so it runs on a side stream beside the data-gradient
        chain, after an event that stands for "the layer behind has produced this gradient"."""
        ops = []   # (kind, payload): "call" zero-arg launch, "fork" (event, side stream), "join"
        for l in layers:
            ops.append(("call", l.bound("fwd", dp, descs[(l.name, n)], ws, main)))
        for li, l in enumerate(reversed(layers)):
            d = descs[(l.name, n)]
            if n_side > 0:
                side, wss = side_streams[li % n_side], ws_side[li % n_side]
                ops.append(("fork", (torch.cuda.Event(), side)))
                ops.append(("call", l.bound("wgrad", dp, d, wss, side)))
            else:
                ops.append(("call", l.bound("wgrad", dp, d, ws, main)))
            if l.needs_dx:
                ops.append(("call", l.bound("dgrad", dp, d, ws, main)))
        if n_side > 0:
            ops.append(("join", None))
        return ops

    def run_ops(ops, main):
        for kind, payload in ops:
            if kind == "call":
                payload()
            elif kind == "fork":
                ev, side = payload
                ev.record(main)
                side.wait_event(ev)
            else:
                for side in side_streams:
                    main.wait_stream(side)

    _ops_cache = {}

    def eager_batch(n):
        main = torch.cuda.current_stream()
        key = (n, main.cuda_stream)
        if key not in _ops_cache:
            _ops_cache[key] = build_batch(n, main)
        run_ops(_ops_cache[key], main)

    def timed(fn, reps):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / reps

    # Launch mode per batch.  The paper runs whole iterations as device graphs and splits them into small graphs
    # (section 5, "Multiplexing"); here every per-GPU batch's sub-step is one small graph, captured with its side
    # streams, and a step replays the six of them in order.  A batch keeps the graph only if it replays faster than
    # launching its kernels one by one (measured in the warm-up, same kernels, same data).
    runners, launch = {}, {}
    reps = max(2, args.warmup)
    for n in batches:
        eager = (lambda n=n: eager_batch(n))
        for _ in range(max(1, args.warmup)):
            eager()                     # also runs the library's one-time initialisation
        runners[n], launch[n] = eager, "eager"
        if args.launch != "eager":
            cap = torch.cuda.Stream()
            cap.wait_stream(torch.cuda.current_stream())
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=cap):
                eager_batch(n)
            graph.replay()
            torch.cuda.synchronize()
            # best of three short runs each: a single short run of either mode is noisy enough to pick the slower one
            if args.launch == "graph" or min(timed(graph.replay, max(5, reps)) for _ in range(3)) < min(timed(eager, max(5, reps)) for _ in range(3)):
                runners[n], launch[n] = graph.replay, "hip_graph"

    def step():
        for n in batches:
            runners[n]()

    flops_step = sum(l.step_flops(n) for l in layers for n in batches)
    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    value = flops_step / (elapsed / args.steps) / 1e12

    # ---- per batch: wall time of that batch's sub-step alone, launched as in the step ----
    per_batch = {}
    for n in batches:
        us = min(timed(runners[n], max(3, args.steps)) for _ in range(3)) * 1e6
        fl = sum(l.step_flops(n) for l in layers)
        per_batch[str(n)] = {"tflops": fl / us / 1e6, "frac_mfma_peak": fl / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, "us": us, "launch": launch[n]}

    # ---- per kernel: the library's own trace (HIP events on the launch stream before / after the main kernel of every
    # pass and after its last kernel); calls issued one after another on one stream ----
    trace = {}
    for _ in range(max(3, min(args.steps, 10))):
        for n in batches:
            layers[0].passes()[0][1](dp, descs[(layers[0].name, n)], ws)   # untraced: absorbs the idle queue's start-up latency
            dp.dp_trace_begin()
            order = []
            for l in layers:
                for pname, fn, _ in l.passes():
                    fn(dp, descs[(l.name, n)], ws)
                    order.append((l.name, n, pname))
            rows = dp.dp_trace_end()
            assert len(rows) == len(order), (len(rows), len(order))
            for key, r in zip(order, rows):
                trace.setdefault(key, []).append(r)
    for n in batches:
        per_batch[str(n)]["us_sum_of_calls"] = sum(median([r["total_us"] for r in trace[(l.name, n, p)]]) for l in layers for p, _, _ in l.passes())
        per_batch[str(n)]["us_sum_of_main_kernels"] = sum(median([r["main_us"] for r in trace[(l.name, n, p)]]) for l in layers for p, _, _ in l.passes())
    kernels = {}
    for (lname, n, pname), rows in trace.items():
        kernels.setdefault(lname, {}).setdefault(str(n), {})[pname] = {
            "kernel": rows[0]["kernel"], "splits": rows[0]["splits"], "main_us": median([r["main_us"] for r in rows]),
            "total_us": median([r["total_us"] for r in rows])}

    rf_max = roofline_objects(trace, layers, nmax)
    rf_small = roofline_objects(trace, layers, 2) if 2 in batches and nmax != 2 else {"mfma": None, "hbm": None}

    # ---- the planner's table comp(i, g): dp_profile_layer per layer over the batches (paper section 4.1) ----
    table = {}
    if not args.no_table:
        for l in layers:
            d = descs[(l.name, batches[0])]
            rows = dp.dp_profile_layer(conv=d, batches=batches, warmup=2, iters=10) if l.is_conv else \
                dp.dp_profile_layer(linear=d, batches=batches, warmup=2, iters=10)
            table[l.name] = {str(r["batch"]): {"fwd_us": r["fwd_us"], "dgrad_us": r["dgrad_us"] if l.needs_dx else 0.0, "wgrad_us": r["wgrad_us"],
                                               "flops_per_pass": r["flops_per_pass"]} for r in rows}

    out = {
        "metric": "conv+FC fwd/bwd TFLOP/s and % bf16 MFMA peak vs per-GPU batch 1-32 (VGG-16)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "strong", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (seeded N(0,1) activations/gradients, He-normal weights)",
        "config": {"workload": {"vgg16": "VGG-16 13 conv + 3 FC layers, 224x224x3 input", "resnet50": "ResNet-50 conv layers (23 unique shapes), 224x224x3 input",
                                "inception": "Inception-v3-style conv layers (18 shapes), 299x299x3 input",
                                "wrn101_2": "wide ResNet-101-2 conv layers (24 unique shapes), 400x400x3 input"}[args.workload]
                               + ", per layer fwd (bias + ReLU fused) + dgrad (backward of the ReLU in front of the layer fused, "
                               "so incoming gradients are already masked) + wgrad with bias gradient (first layer: no dgrad), "
                               + ("layers " + args.layers + ", " if args.layers else "")
                               + "per-GPU batches " + args.batches + " (strong-scaling shards of global batch 32)",
                   "batches": batches, "flops_per_step": flops_step},
        "frac_mfma_peak": value / MFMA_BF16_PEAK_TFLOPS, "launch": launch if len(set(launch.values())) > 1 else next(iter(launch.values())),
        "kernel_choice": "model" if args.no_autotune else "measured (" + args.autotune + ")",
        "per_batch": per_batch,
        "roofline": rf_max["mfma"] or rf_max["hbm"],
        "roofline_hbm": rf_max["hbm"],
        "roofline_batch2": rf_small["mfma"],
        "roofline_hbm_batch2": rf_small["hbm"],
    }
    if table:
        out["layer_table_us"] = {ln: {b: [round(v["fwd_us"], 2), round(v["dgrad_us"], 2), round(v["wgrad_us"], 2)] for b, v in t.items()} for ln, t in table.items()}
        out["layer_table_source"] = "dp_profile_layer (fwd, dgrad, wgrad microseconds per layer and per-GPU batch; comp(i,g) of the planner = their sum at batch 32/g)"
    if args.workload == "vgg16" and not args.layers and not args.no_glue:
        out["glue"] = glue_times(dp, torch, dev, batches)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    if args.table:
        with open(args.table, "w") as f:
            json.dump({"source": "dp_profile_layer", "layers": table, "kernels": kernels}, f, indent=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
