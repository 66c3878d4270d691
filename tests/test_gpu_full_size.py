"""Full-size layers of the benchmark workload (VGG-16, paper Table 1) at the per-GPU batches the benchmark
times, spot-checked against the oracle's per-element evaluators.

Every (layer, batch) point is run the way bench.py's step issues it -- measured kernel choice on, forward with
bias + ReLU, backward-data with the fused backward of the input ReLU and no saved output (the incoming gradient
counts as already masked), backward-filter with the bias gradient and no saved output -- so the grids, split
counts and row widths checked here are the ones that are timed.  The saved-output (y_saved) forms of the two
backward calls are checked at two batches per layer.  A second group forces every kernel family the benchmark
reports onto the full-size layers it is eligible for and asserts, through dp_conv2d_kernel_info, that this
family is what ran.  Samples always include the first and the last elements (first / last tile, image borders).
Tolerances: the bf16 bar (rel-L2 <= 2e-2, max-abs <= 5e-2); bias gradients rel-L2 <= 1e-5 against the oracle.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

NMAX = 32
BATCHES = (1, 2, 4, 8, 16, 32)
MASKED_BATCHES = (2, 32)   # batches at which the y_saved forms of the backward calls are checked as well


@pytest.fixture(scope="module")
def env(orc):
    from paper_2112_10065_amd import binding as dp
    import gpu_util as U
    assert torch.cuda.is_available()
    yield dp, U, orc
    dp.dp_set_autotune(False)
    for p in range(3):
        dp.dp_set_override(p, -1, 0)


def _convs():
    from paper_2112_10065_amd import workloads
    return workloads.vgg16_convs()


def _linears():
    from paper_2112_10065_amd import workloads
    return workloads.vgg16_linears()


class FullConv:
    """Seeded tensors of one VGG conv layer at batch 32 (smaller batches are the leading samples: the sample
    index is part of the generator's counter).  The input of every layer but the first is what a ReLU leaves."""

    def __init__(self, U, l):
        from paper_2112_10065_amd import synth
        self.l, self.first = l, l.c < 8
        x, w, b = synth.conv_tensors(f"vgg/{l.name}", NMAX, l.h, l.w, l.c, l.k, l.r, l.s)
        if not self.first:
            np.maximum(x, 0.0, out=x)
        dy = synth.upstream_grad(f"vgg/{l.name}", (NMAX, l.h, l.w, l.k))
        xb, wb, dyb = (synth.f32_to_bf16_bits(a) for a in (x, w, dy))
        self.x, self.w, self.dy, self.b = synth.bf16_bits_to_f32(xb), synth.bf16_bits_to_f32(wb), synth.bf16_bits_to_f32(dyb), b
        self.xd, self.wd, self.dyd = U.bf16_dev(xb), U.bf16_dev(wb), U.bf16_dev(dyb)
        self.bd = torch.from_numpy(b).to(U.DEV)

    def desc(self, dp, n, relu_in):
        l = self.l
        flags = dp.DP_BIAS | dp.DP_RELU | (dp.DP_DX_F32 if self.first else 0) | (dp.DP_RELU_IN if relu_in else 0)
        return dp.conv_desc(n, l.h, l.w, l.c, l.k, l.r, l.s, (1, 1), (1, 1), dp.DP_BF16, flags)


_cache = {}


def full_conv(U, name):
    """One layer's tensors stay resident at a time (the largest is 0.8 GB on the host)."""
    if name not in _cache:
        _cache.clear()
        _cache[name] = FullConv(U, {l.name: l for l in _convs()}[name])
    return _cache[name]


def _sample(rng, size, count, edge):
    idx = rng.integers(0, size, count)
    edge = min(edge, size, count // 2)
    idx[:edge] = np.arange(edge)
    idx[edge:2 * edge] = size - 1 - np.arange(edge)
    return idx


def check_conv_point(dp, U, orc, L, n, what, masked_forms, passes=(0, 1, 2)):
    """The three calls of bench.py's step on the first n samples, sampled against the oracle."""
    l = L.l
    rng = np.random.default_rng(1000 * n + l.h + l.c)
    x, dy, xd, dyd = L.x[:n], L.dy[:n], L.xd[:n], L.dyd[:n]
    d = L.desc(dp, n, relu_in=not L.first)
    ws = U.workspace(max(dp.dp_conv2d_workspace_bytes(d, p) for p in range(3)))
    y = torch.empty((n, l.h, l.w, l.k), dtype=torch.bfloat16, device=U.DEV)
    dx = torch.full((n, l.h, l.w, l.c), 3.0, dtype=torch.float32 if L.first else torch.bfloat16, device=U.DEV)
    dw = torch.empty((l.k, l.r, l.s, l.c), dtype=torch.float32, device=U.DEV)
    db = torch.empty((l.k,), dtype=torch.float32, device=U.DEV)
    if 0 in passes or masked_forms:
        dp.dp_conv2d_fwd(d, xd, L.wd, L.bd, y, ws)
    if 1 in passes:
        dp.dp_conv2d_bwd_data_relu(d, dyd, None, L.wd, xd, dx, ws)
    if 2 in passes:
        dp.dp_conv2d_bwd_filter(d, xd, dyd, None, dw, db, ws)
    torch.cuda.synchronize()
    y_np = U.to_np(y)
    if 0 in passes:
        idx = _sample(rng, y_np.size, 3000, 64)
        U.assert_bf16_close(y_np.ravel()[idx], orc.conv2d_fwd_at(x, L.w, L.b, True, (1, 1), (1, 1), idx), f"{what} y")
    if 1 in passes:
        dx_np = U.to_np(dx)
        idx = _sample(rng, dx_np.size, 3000, 64)
        want = orc.conv2d_bwd_data_at(dy, L.w, x.shape, None, (1, 1), (1, 1), idx)
        if not L.first:
            want = orc.relu_in_backward(want, x.ravel()[idx])
            assert not dx_np.ravel()[idx][x.ravel()[idx] <= 0].any(), f"{what}: dx not zero behind a closed ReLU"
        U.assert_bf16_close(dx_np.ravel()[idx], want, f"{what} dx")
    if 2 in passes:
        dw_np = U.to_np(dw)
        idx = _sample(rng, dw_np.size, 600, 32)
        U.assert_bf16_close(dw_np.ravel()[idx], orc.conv2d_bwd_filter_at(x, dy, L.w.shape, None, (1, 1), (1, 1), idx), f"{what} dw")
        _, rdb = orc.relu_bias_grad(dy, np.ones_like(dy))   # no mask: the plain column sum, by the oracle
        rel, mx = U.errs(U.to_np(db), rdb)
        assert rel <= 1e-5, f"{what} db rel_l2={rel:.3e} max_abs={mx:.3e}"
    if masked_forms:
        # the forms that take the layer's saved output: g = dy * [y_saved > 0] inside the calls
        dm = L.desc(dp, n, relu_in=False)
        wsm = U.workspace(max(dp.dp_conv2d_workspace_bytes(dm, p) for p in range(3)))
        dp.dp_conv2d_bwd_data(dm, dyd, y, L.wd, dx, wsm)
        dp.dp_conv2d_bwd_filter(dm, xd, dyd, y, dw, db, wsm)
        torch.cuda.synchronize()
        dx_np, dw_np = U.to_np(dx), U.to_np(dw)
        idx = _sample(rng, dx_np.size, 2000, 32)
        U.assert_bf16_close(dx_np.ravel()[idx], orc.conv2d_bwd_data_at(dy, L.w, x.shape, y_np, (1, 1), (1, 1), idx), f"{what} dx (y_saved)")
        idx = _sample(rng, dw_np.size, 400, 16)
        U.assert_bf16_close(dw_np.ravel()[idx], orc.conv2d_bwd_filter_at(x, dy, L.w.shape, y_np, (1, 1), (1, 1), idx), f"{what} dw (y_saved)")
        _, rdb = orc.relu_bias_grad(dy, y_np)
        rel, mx = U.errs(U.to_np(db), rdb)
        assert rel <= 1e-5, f"{what} db (y_saved) rel_l2={rel:.3e} max_abs={mx:.3e}"
    return [dp.dp_conv2d_kernel_info(d, p) for p in range(3)]


@pytest.mark.parametrize("name", [l.name for l in _convs()])
def test_vgg_conv_layer_every_batch_measured_choice(env, name):
    """All six per-GPU batches of one layer under the measured kernel choice: the plans bench.py times."""
    dp, U, orc = env
    L = full_conv(U, name)
    dp.dp_set_autotune(True)
    try:
        for n in BATCHES:
            names = check_conv_point(dp, U, orc, L, n, f"{name} N={n}", masked_forms=n in MASKED_BATCHES)
            print(f"{name} N={n}: " + "; ".join(f"{nm} x{sp}" for nm, sp in names))
    finally:
        dp.dp_set_autotune(False)


@pytest.mark.parametrize("name", ["conv1_1", "conv1_2", "conv3_2", "conv5_1"])
def test_vgg_conv_layer_model_choice(env, name):
    """The analytic kernel choice (no measurement, what DP_DETERMINISTIC callers get) at the smallest and largest batch."""
    dp, U, orc = env
    L = full_conv(U, name)
    for n in (1, 32):
        check_conv_point(dp, U, orc, L, n, f"{name} N={n} model", masked_forms=False)


# (layer, batch, pass, variant code, splits, kernel name the profiler prints)
FORCED = [
    # pixel-strip kernels, forward and backward-data: every tile shape on a layer it is offered for
    ("conv2_2", 32, 0, 232, 1, "k_conv_strip<false, 256, 128>"), ("conv2_2", 32, 1, 232, 1, "k_conv_strip<true, 256, 128>"),
    ("conv2_2", 4, 0, 232, 1, "k_conv_strip<false, 256, 128>"),
    ("conv3_1", 32, 1, 232, 1, "k_conv_strip<true, 256, 128>"), ("conv3_1", 32, 0, 233, 1, "k_conv_strip<false, 224, 256>"),
    ("conv3_2", 32, 0, 233, 1, "k_conv_strip<false, 224, 256>"), ("conv3_2", 32, 1, 233, 1, "k_conv_strip<true, 224, 256>"),
    ("conv3_2", 32, 0, 230, 1, "k_conv_strip<false, 256, 256>"), ("conv3_2", 32, 1, 230, 1, "k_conv_strip<true, 256, 256>"),
    ("conv3_2", 16, 0, 233, 1, "k_conv_strip<false, 224, 256>"), ("conv3_2", 8, 1, 231, 1, "k_conv_strip<true, 128, 256>"),
    ("conv4_2", 32, 0, 233, 1, "k_conv_strip<false, 224, 256>"), ("conv4_2", 32, 1, 233, 1, "k_conv_strip<true, 224, 256>"),
    ("conv4_2", 16, 0, 231, 1, "k_conv_strip<false, 128, 256>"), ("conv4_2", 16, 1, 231, 1, "k_conv_strip<true, 128, 256>"),
    ("conv5_1", 32, 0, 231, 2, "k_conv_strip<false, 128, 256>"), ("conv5_1", 32, 1, 231, 2, "k_conv_strip<true, 128, 256>"),
    ("conv5_1", 32, 0, 230, 4, "k_conv_strip<false, 256, 256>"),
    # filter gradient on the shared x strip (rows of at most 62 pixels) and its split counts
    ("conv3_2", 32, 2, 316, 8, "k_wgrad_strip"), ("conv3_2", 16, 2, 316, 4, "k_wgrad_strip"), ("conv4_2", 32, 2, 316, 8, "k_wgrad_strip"),
    ("conv4_2", 16, 2, 316, 5, "k_wgrad_strip"), ("conv5_1", 32, 2, 316, 5, "k_wgrad_strip"), ("conv3_1", 32, 2, 316, 16, "k_wgrad_strip"),
    # input patch resident in LDS (64 reduction channels per tap): conv1_2 forward / backward-data / filter gradient, conv2_1
    ("conv1_2", 32, 0, 403, 0, "k_halo<0, 64, 1, 4, 4>"), ("conv1_2", 2, 0, 400, 0, "k_halo<0, 64, 1, 4, 2>"),
    ("conv1_2", 16, 0, 404, 0, "k_halo_ws<0, false>"), ("conv1_2", 32, 1, 403, 0, "k_halo<1, 64, 1, 4, 4>"),
    ("conv2_1", 32, 0, 403, 0, "k_halo<0, 64, 1, 4, 4>"), ("conv2_1", 2, 0, 401, 0, "k_halo<0, 128, 2, 2, 2>"),
    ("conv1_2", 32, 2, 410, 0, "k_wgrad_halo"), ("conv2_1", 32, 2, 410, 0, "k_wgrad_halo"), ("conv1_2", 2, 2, 410, 0, "k_wgrad_halo"),
    ("conv1_2", 32, 2, 411, 0, "k_wgrad_halo9<true>"), ("conv2_1", 16, 2, 411, 0, "k_wgrad_halo9<true>"), ("conv1_2", 1, 2, 411, 0, "k_wgrad_halo9<true>"),
    # pipelined tiles of the large batches and their filter-gradient forms with many splits
    ("conv2_2", 32, 0, 200, 1, "k_fwd_dma<128, 128, 64, 2, 2, 2, 1>"), ("conv4_2", 32, 1, 208, 1, "k_dgrad_dma<256, 256, 64, 2, 4, 2, 1>"),
    ("conv2_2", 32, 2, 300, 16, "k_wgrad_dma<128, 128, 32, 2, 2, 2>"), ("conv4_2", 32, 2, 312, 8, "k_wgrad_dma<256, 256, 64, 2, 4, 2>"),
    ("conv4_2", 2, 2, 305, 1, "k_wgrad_dma<64, 64, 32, 2, 2, 2>"), ("conv5_1", 1, 2, 305, 1, "k_wgrad_dma<64, 64, 32, 2, 2, 2>"),
    # small-batch tiles: reduction groups inside a block, reduction splits with the second kernel
    ("conv3_2", 2, 0, 228, 1, "k_fwd_dma<64, 128, 64, 2, 2, 2, 2>"), ("conv3_2", 2, 1, 228, 1, "k_dgrad_dma<64, 128, 64, 2, 2, 2, 2>"),
    ("conv3_2", 1, 0, 226, 1, "k_fwd_dma<64, 64, 64, 2, 2, 2, 4>"), ("conv4_2", 1, 1, 226, 2, "k_dgrad_dma<64, 64, 64, 2, 2, 2, 4>"),
    ("conv4_2", 2, 0, 227, 2, "k_fwd_dma<64, 64, 64, 2, 2, 2, 2>"), ("conv4_2", 2, 1, 206, 5, "k_dgrad_dma<128, 64, 64, 2, 2, 2, 1>"),
    ("conv5_1", 2, 0, 207, 12, "k_fwd_dma<64, 64, 64, 2, 2, 3, 1>"), ("conv5_1", 2, 1, 229, 9, "k_dgrad_dma<128, 64, 64, 2, 2, 2, 2>"),
    ("conv5_1", 1, 0, 226, 6, "k_fwd_dma<64, 64, 64, 2, 2, 2, 4>"),
]


@pytest.mark.parametrize("name,n,pas,variant,splits,kernel", FORCED, ids=[f"{f[0]}_n{f[1]}_p{f[2]}_v{f[3]}_s{f[4]}" for f in FORCED])
def test_kernel_family_at_full_size(env, name, n, pas, variant, splits, kernel):
    """Each kernel family the benchmark reports, forced onto a full-size layer: the name the profiler would print is
    asserted, then the pass is sampled against the oracle."""
    dp, U, orc = env
    L = full_conv(U, name)
    dp.dp_set_override(pas, variant, splits)
    try:
        got, got_splits = dp.dp_conv2d_kernel_info(L.desc(dp, n, relu_in=not L.first), pas)
        assert got == kernel, (got, got_splits)
        if splits > 0 and "k_wgrad_strip" not in kernel:
            assert got_splits == splits
        check_conv_point(dp, U, orc, L, n, f"{name} N={n} {kernel} x{got_splits}", masked_forms=False, passes=(pas,))
    finally:
        dp.dp_set_override(pas, -1, 0)


@pytest.mark.parametrize("name", [l.name for l in _linears()])
def test_vgg_dense_layer_full_size(env, name):
    """fc6 / fc7 / fc8 at batches 1, 2 and 32 as bench.py's step calls them (forward; dx with the fused backward of
    the input ReLU; dW + db), plus the y_saved forms at batch 32; measured kernel choice."""
    dp, U, orc = env
    from paper_2112_10065_amd import synth
    l = {q.name: q for q in _linears()}[name]
    i, o = l.in_f, l.out_f
    x, W, b = synth.linear_tensors(f"vgg/{name}", NMAX, i, o)
    np.maximum(x, 0.0, out=x)
    dy = synth.upstream_grad(f"vgg/{name}", (NMAX, o))
    xb, Wb, dyb = (synth.f32_to_bf16_bits(a) for a in (x, W, dy))
    x, W, dy = (synth.bf16_bits_to_f32(a) for a in (xb, Wb, dyb))
    xd, Wd, dyd = U.bf16_dev(xb), U.bf16_dev(Wb), U.bf16_dev(dyb)
    bd = torch.from_numpy(b).to(U.DEV)
    dW = torch.empty((o, i), dtype=torch.float32, device=U.DEV)
    db = torch.empty((o,), dtype=torch.float32, device=U.DEV)
    dp.dp_set_autotune(True)
    try:
        for n in (1, 2, 32):
            rng = np.random.default_rng(n + o)
            desc = dp.linear_desc(n, i, o, dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU | dp.DP_RELU_IN)
            ws = U.workspace(dp.dp_linear_workspace_bytes(desc))
            y = torch.empty((n, o), dtype=torch.bfloat16, device=U.DEV)
            dx = torch.full((n, i), 3.0, dtype=torch.bfloat16, device=U.DEV)
            dp.dp_linear_fwd_bwd(desc, x=xd[:n], W=Wd, bias=bd, y=y, ws=ws)
            dp.dp_linear_fwd_bwd(desc, x=xd[:n], W=Wd, dy=dyd[:n], dx=dx, ws=ws)
            dp.dp_linear_fwd_bwd(desc, x=xd[:n], dy=dyd[:n], dW=dW, dbias=db, ws=ws)
            torch.cuda.synchronize()
            y_np, dx_np = U.to_np(y), U.to_np(dx)
            idx = _sample(rng, n * o, min(4000, 2 * n * o), 32)
            U.assert_bf16_close(y_np.ravel()[idx], orc.linear_fwd_at(x[:n], W, b, True, idx), f"{name} N={n} y")
            idx = _sample(rng, n * i, 4000, 32)
            want = orc.relu_in_backward(orc.linear_dx_at(W, dy[:n], None, idx), x[:n].ravel()[idx])
            U.assert_bf16_close(dx_np.ravel()[idx], want, f"{name} N={n} dx")
            assert not dx_np.ravel()[idx][x[:n].ravel()[idx] <= 0].any()
            idx = _sample(rng, o * i, 20000, 64)
            U.assert_bf16_close(U.to_np(dW).ravel()[idx], orc.linear_dw_at(x[:n], dy[:n], None, idx), f"{name} N={n} dW")
            _, rdb = orc.relu_bias_grad(dy[:n], np.ones_like(dy[:n]))
            rel, mx = U.errs(U.to_np(db), rdb)
            assert rel <= 1e-5, f"{name} N={n} db rel_l2={rel:.3e}"
            if n == 32:
                dm = dp.linear_desc(n, i, o, dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU)
                wsm = U.workspace(dp.dp_linear_workspace_bytes(dm))
                dp.dp_linear_fwd_bwd(dm, x=xd[:n], W=Wd, dy=dyd[:n], y_saved=y, dx=dx, dW=dW, dbias=db, ws=wsm)
                torch.cuda.synchronize()
                idx = _sample(rng, n * i, 4000, 32)
                U.assert_bf16_close(U.to_np(dx).ravel()[idx], orc.linear_dx_at(W, dy[:n], y_np, idx), f"{name} dx (y_saved)")
                idx = _sample(rng, o * i, 20000, 64)
                U.assert_bf16_close(U.to_np(dW).ravel()[idx], orc.linear_dw_at(x[:n], dy[:n], y_np, idx), f"{name} dW (y_saved)")
                _, rdb = orc.relu_bias_grad(dy[:n], y_np)
                rel, mx = U.errs(U.to_np(db), rdb)
                assert rel <= 1e-5, f"{name} db (y_saved) rel_l2={rel:.3e}"
    finally:
        dp.dp_set_autotune(False)
