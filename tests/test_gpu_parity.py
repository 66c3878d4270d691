"""GPU parity: the HIP library against the fp64 CPU oracle on the same seeded inputs.

Tolerances are the spec ones: fp32 path rel-L2 <= 1e-5; bf16-input path (fp32
accumulation) rel-L2 <= 2e-2 and max-abs <= 5e-2.  Backward passes take the GPU forward's
stored output as the saved activation on both sides, so a ReLU mask never differs.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(orc):
    from paper_2112_10065_amd import binding as dp
    import gpu_util as U
    assert torch.cuda.is_available()
    yield dp, U, orc
    for p in range(3):
        dp.dp_set_override(p, -1, 0)


def check_case(dp, U, orc, case, what):
    n, h, w, c, k, r, s = case.shape
    st, pd = case.stride, case.pad
    y = case.run_fwd()
    dx = case.run_dgrad(y if case.relu else None)
    dw, db = case.run_wgrad(y if case.relu else None)
    torch.cuda.synchronize()
    y_np = U.to_np(y)
    ys = y_np if case.relu else None
    ref_y = orc.conv2d_fwd(case.x, case.w, case.b, relu=case.relu, stride=st, pad=pd)
    ref_dx = orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=ys, stride=st, pad=pd)
    ref_dw, ref_db = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=ys, stride=st, pad=pd, want_db=True)
    chk = U.assert_bf16_close if case.bf16 else U.assert_f32_close
    chk(y_np, ref_y, f"{what} y")
    chk(U.to_np(dx), ref_dx, f"{what} dx")
    chk(U.to_np(dw), ref_dw, f"{what} dw")
    chk(U.to_np(db), ref_db, f"{what} db")


def test_rgb_stem_kernels_are_chosen_and_filter_gradient_without_bias_gradient(env):
    """The RGB 3x3 stem with rows of whole 32-pixel segments runs the segment kernels (names as the profiler shows them); the filter gradient
    alone (no bias gradient asked for) equals the oracle's."""
    dp, U, orc = env
    case = U.ConvCase("rgb_seg", 2, 6, 64, 3, 64, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=False, dx_f32=True)
    assert dp.dp_conv2d_kernel_info(case.desc, 0)[0] == "k_fwd_rgb3"
    assert dp.dp_conv2d_kernel_info(case.desc, 2)[0] == "k_wgrad_rgb3<true>"
    other = U.ConvCase("rgb_noseg", 2, 6, 40, 3, 64, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=False, dx_f32=True)
    assert dp.dp_conv2d_kernel_info(other.desc, 0)[0] == "k_fwd_direct"
    assert dp.dp_conv2d_kernel_info(other.desc, 2)[0] == "k_wgrad_direct"
    dw, db = case.run_wgrad(None, want_db=False)
    torch.cuda.synchronize()
    assert db is None
    ref_dw, _ = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=None, stride=(1, 1), pad=(1, 1), want_db=True)
    U.assert_bf16_close(U.to_np(dw), ref_dw, "stem filter gradient without bias gradient")


# ---- configuration 1: single 3x3 layer in fp32 ------------------------------------------
@pytest.mark.parametrize("bias", [False, True])
def test_config1_fp32(env, bias):
    dp, U, orc = env
    case = U.ConvCase("cfg1", 2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1), bf16=False, dist="he_uniform", bias=bias, relu=True)
    check_case(dp, U, orc, case, f"config1 bias={bias}")


def test_fp32_strided_asymmetric(env):
    dp, U, orc = env
    case = U.ConvCase("f32s", 3, 13, 11, 5, 7, 3, 5, (2, 1), (1, 2), bf16=False, dist="he_uniform", bias=True, relu=True)
    check_case(dp, U, orc, case, "fp32 strided")


# ---- bf16 matrix-core path: shapes that span several tiles with ragged tails ---------------
BF16_CASES = [
    # tag, n, h, w, c, k, r, s, stride, pad, bias, relu, dx_f32
    ("vgg_like_64", 2, 28, 28, 64, 64, 3, 3, (1, 1), (1, 1), True, True, False),
    ("vgg_like_64_dx_f32", 2, 28, 28, 64, 64, 3, 3, (1, 1), (1, 1), True, True, True),
    ("vgg_like_128_256", 3, 14, 14, 128, 256, 3, 3, (1, 1), (1, 1), True, True, False),
    ("rgb_3x3", 2, 20, 22, 3, 64, 3, 3, (1, 1), (1, 1), True, True, True),
    ("stem_7x7_s2", 2, 30, 30, 3, 64, 7, 7, (2, 2), (3, 3), False, False, True),
    ("rgb_3x3_s2_k32", 3, 23, 21, 3, 32, 3, 3, (2, 2), (0, 0), False, True, True),
    ("rgb_3x3_k136", 1, 37, 19, 3, 136, 3, 3, (1, 1), (1, 1), True, True, True),
    # rows of whole 32-pixel segments: the RGB stem kernels (unmasked filter gradient, forward); with ReLU the saved output masks dy
    ("rgb_3x3_w32", 2, 5, 32, 3, 64, 3, 3, (1, 1), (1, 1), True, False, True),
    ("rgb_3x3_w64_relu_k128", 3, 7, 64, 3, 128, 3, 3, (1, 1), (1, 1), True, True, True),
    ("rgb_3x3_w96_k128", 1, 9, 96, 3, 128, 3, 3, (1, 1), (1, 1), False, False, True),
    ("rgb_3x3_one_row", 2, 1, 32, 3, 64, 3, 3, (1, 1), (1, 1), True, False, True),
    ("gray_5x5", 2, 18, 18, 1, 16, 5, 5, (1, 1), (2, 2), True, False, True),
    ("res_1x1", 2, 14, 14, 256, 64, 1, 1, (1, 1), (0, 0), False, False, False),
    ("res_1x1_s2", 2, 14, 14, 128, 256, 1, 1, (2, 2), (0, 0), False, False, False),
    ("res_3x3_s2", 2, 15, 15, 64, 64, 3, 3, (2, 2), (1, 1), False, True, False),
    ("inc_1x7", 2, 17, 17, 128, 160, 1, 7, (1, 1), (0, 3), False, True, False),
    ("inc_7x1", 2, 17, 17, 160, 128, 7, 1, (1, 1), (3, 0), False, False, False),
    ("inc_c80", 1, 19, 19, 80, 192, 3, 3, (1, 1), (0, 0), False, True, False),
    ("inc_3x3_s2_p0", 2, 17, 17, 32, 96, 3, 3, (2, 2), (0, 0), False, False, False),
    ("odd_channels", 2, 9, 10, 24, 40, 3, 3, (1, 1), (1, 1), True, True, False),
    ("k_not_mult8", 1, 8, 8, 16, 12, 3, 3, (1, 1), (1, 1), True, True, False),
    ("tiny", 1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0), True, True, True),
]


@pytest.mark.parametrize("spec", BF16_CASES, ids=[c[0] for c in BF16_CASES])
def test_bf16_conv_parity(env, spec):
    dp, U, orc = env
    tag, n, h, w, c, k, r, s, st, pd, bias, relu, dxf = spec
    case = U.ConvCase(tag, n, h, w, c, k, r, s, st, pd, bf16=True, bias=bias, relu=relu, dx_f32=dxf)
    check_case(dp, U, orc, case, tag)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("splits", [1, 3])
def test_every_tile_variant_and_split(env, variant, splits):
    dp, U, orc = env
    for p in range(3):
        dp.dp_set_override(p, variant, splits)
    try:
        case = U.ConvCase("variants", 2, 13, 12, 72, 136, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True)
        check_case(dp, U, orc, case, f"variant {variant} splits {splits}")
        case = U.ConvCase("variants_rgb", 1, 12, 12, 3, 40, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True, dx_f32=True)
        check_case(dp, U, orc, case, f"variant {variant} splits {splits} rgb")
    finally:
        for p in range(3):
            dp.dp_set_override(p, -1, 0)


@pytest.mark.parametrize("variant", [100, 101, 102, 103])
@pytest.mark.parametrize("splits", [1, 3])
def test_every_fast_variant_and_split(env, variant, splits):
    """Fast-path kernels (buffer loads, LDS transpose reads), every tile shape, split and unsplit."""
    dp, U, orc = env
    for p in range(3):
        dp.dp_set_override(p, variant, splits)
    try:
        # c_in % 64 == 0 and c_out % 32 == 0 (reduction step 64 forward, 32 backward-data), ragged tiles
        case = U.ConvCase("fastv", 2, 13, 12, 64, 96, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True)
        names = [dp.dp_conv2d_kernel_info(case.desc, p)[0] for p in range(3)]
        assert all("fast" in n for n in names), names
        check_case(dp, U, orc, case, f"fast variant {variant} splits {splits}")
        # c_in % 32 == 0 only, 1x7 filter, backward-filter with stride 2 falls on the fast path too
        case = U.ConvCase("fastv2", 2, 11, 17, 96, 64, 1, 7, (1, 1), (0, 3), bf16=True, bias=False, relu=False)
        check_case(dp, U, orc, case, f"fast variant {variant} splits {splits} 1x7")
        case = U.ConvCase("fastv3", 3, 15, 14, 32, 40, 3, 3, (2, 2), (1, 1), bf16=True, bias=True, relu=True)
        check_case(dp, U, orc, case, f"fast variant {variant} splits {splits} stride 2")
    finally:
        for p in range(3):
            dp.dp_set_override(p, -1, 0)


@pytest.mark.parametrize("variant", [200, 201, 202, 203, 204, 205, 206, 207, 208, 209, 210, 211, 212, 213, 214, 215, 216, 217, 218, 219, 220, 221, 222, 223, 224, 225, 226, 227, 228, 229])
@pytest.mark.parametrize("splits", [1, 2])
def test_pipelined_forward_variants(env, variant, splits):
    """Forward and backward-data kernels with the multi-stage direct-to-LDS pipeline: every stage
    count / tile shape, reductions shorter and longer than the pipeline depth, ragged tails."""
    dp, U, orc = env
    dp.dp_set_override(0, variant, splits)
    dp.dp_set_override(1, variant, splits)
    try:
        for tag, n, h, w, c, k, r, s_, pd in (("pipe_a", 2, 13, 12, 64, 96, 3, 3, (1, 1)), ("pipe_b", 1, 9, 9, 128, 200, 1, 1, (0, 0)),
                                              ("pipe_c", 3, 10, 17, 64, 264, 1, 7, (0, 3)), ("pipe_d", 2, 12, 13, 192, 128, 3, 3, (1, 1)),
                                              ("pipe_e", 2, 11, 9, 256, 128, 3, 3, (1, 1))):
            if 221 <= variant <= 225 and c % 128 != 0:
                continue   # these variants reduce 128 channels per step
            case = U.ConvCase(tag, n, h, w, c, k, r, s_, (1, 1), pd, bf16=True, bias=True, relu=True)
            assert "fwd_dma" in dp.dp_conv2d_kernel_info(case.desc, 0)[0]
            y = case.run_fwd()
            torch.cuda.synchronize()
            ref = orc.conv2d_fwd(case.x, case.w, case.b, relu=True, stride=(1, 1), pad=pd)
            U.assert_bf16_close(U.to_np(y), ref, f"{tag} variant {variant} splits {splits}")
            if k % 64 == 0 or (k % 32 == 0 and "32, 2, 2" in dp.dp_conv2d_kernel_info(case.desc, 0)[0]):
                assert "dgrad_dma" in dp.dp_conv2d_kernel_info(case.desc, 1)[0]
            dx = case.run_dgrad(y)
            torch.cuda.synchronize()
            y_np = U.to_np(y)
            U.assert_bf16_close(U.to_np(dx), orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=y_np, pad=pd),
                                f"{tag} variant {variant} splits {splits} dx")
    finally:
        dp.dp_set_override(0, -1, 0)
        dp.dp_set_override(1, -1, 0)


@pytest.mark.parametrize("variant", [200, 203, 207, 210, 214, 219, 221, 226, 227, 229])
@pytest.mark.parametrize("splits", [2, 5])
def test_split_reduction_fused_into_the_pipelined_kernels(env, variant, splits):
    """Forced variant 1000 + v: the last block that finishes a tile sums the splits' partial tiles itself (in split
    order, so the result equals the two-kernel path bit for bit) and applies bias / ReLU / the input-ReLU mask.
    Two calls in a row per case: the tile counters return to zero after a call."""
    dp, U, orc = env
    for tag, n, h, w, c, k, r, s_, pd, f32 in (("fr_a", 2, 13, 12, 128, 192, 3, 3, (1, 1), False), ("fr_b", 1, 9, 9, 256, 200, 1, 1, (0, 0), True),
                                               ("fr_c", 3, 10, 17, 128, 264, 1, 7, (0, 3), False), ("fr_d", 1, 14, 14, 512, 512, 3, 3, (1, 1), True)):
        if 221 <= variant <= 225 and c % 128 != 0:
            continue   # these variants reduce 128 channels per step
        case = U.ConvCase(tag, n, h, w, c, k, r, s_, (1, 1), pd, bf16=True, bias=True, relu=True, dx_f32=f32)
        out, plain = {}, {}
        for fused in (0, 1000):
            dp.dp_set_override(0, variant + fused, splits)
            dp.dp_set_override(1, variant + fused, splits)
            try:
                for p in (0, 1):   # a negative split count reports that no reduction kernel follows
                    nm, sp = dp.dp_conv2d_kernel_info(case.desc, p)
                    if not fused:
                        plain[p] = sp   # the planner may lower the forced split count to one that divides the reduction steps
                    assert "_dma" in nm or p == 1, nm
                    assert sp == (-plain[p] if fused and "_dma" in nm and plain[p] > 1 else plain[p]), (nm, sp, plain[p])
                ys = [case.run_fwd() for _ in range(2)]
                dxs = [case.run_dgrad(ys[0]) for _ in range(2)]
                dxm = case.run_dgrad_relu_in(ys[0])
                torch.cuda.synchronize()
            finally:
                dp.dp_set_override(0, -1, 0)
                dp.dp_set_override(1, -1, 0)
            assert torch.equal(ys[0], ys[1]) and torch.equal(dxs[0], dxs[1]), f"{tag} {variant} second call differs"
            out[fused] = (ys[0], dxs[0], dxm)
        for a, b, what in zip(out[0], out[1000], ("y", "dx", "dx masked")):
            assert torch.equal(a, b), f"{tag} variant {variant} splits {splits}: fused {what} differs from the two-kernel path"
        y, dx, dxm = out[1000]
        U.assert_bf16_close(U.to_np(y), orc.conv2d_fwd(case.x, case.w, case.b, relu=True, stride=(1, 1), pad=pd), f"{tag} fused y")
        ref = orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=U.to_np(y), pad=pd)
        U.assert_bf16_close(U.to_np(dx), ref, f"{tag} fused dx")


@pytest.mark.parametrize("tag,n,h,w,c,k,r,s_,st,pd", [
    ("sd_3x3_s2", 2, 15, 15, 64, 64, 3, 3, (2, 2), (1, 1)), ("sd_1x1_s2", 1, 14, 17, 128, 128, 1, 1, (2, 2), (0, 0)),
    ("sd_3x3_s21", 2, 13, 12, 64, 192, 3, 3, (2, 1), (1, 0)), ("sd_5x5_s3", 1, 20, 20, 256, 128, 5, 5, (3, 3), (2, 2))])
def test_strided_backward_data_pipelined(env, tag, n, h, w, c, k, r, s_, st, pd):
    """Strided layers run backward-data on the pipelined kernel: taps that miss the stride grid of an input
    pixel are masked out (zero rows), the rest address dy at (hb/sh - r/sh, wb/sw - s/sw)."""
    dp, U, orc = env
    case = U.ConvCase(tag, n, h, w, c, k, r, s_, st, pd, bf16=True, bias=False, relu=True)
    assert "dgrad_dma" in dp.dp_conv2d_kernel_info(case.desc, 1)[0]
    y = case.run_fwd()
    dx = case.run_dgrad(y)
    torch.cuda.synchronize()
    U.assert_bf16_close(U.to_np(dx), orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=U.to_np(y), stride=st, pad=pd), f"{tag} dx")


PHASE_CASES = [
    # tag, n, h, w, c, k, r, s, stride, pad : stride 2 in one or both directions, odd and even sizes, pads that shift the phases
    ("ph_3x3_s2_p1", 2, 15, 14, 64, 64, 3, 3, (2, 2), (1, 1)), ("ph_3x3_s2_p0", 3, 17, 17, 32, 96, 3, 3, (2, 2), (0, 0)),
    ("ph_1x1_s2", 2, 14, 17, 128, 128, 1, 1, (2, 2), (0, 0)), ("ph_3x3_s21", 2, 13, 12, 64, 192, 3, 3, (2, 1), (1, 0)),
    ("ph_3x3_s12", 1, 9, 20, 40, 64, 3, 3, (1, 2), (1, 1)), ("ph_7x7_s2", 1, 21, 22, 16, 64, 7, 7, (2, 2), (3, 3)),
    ("ph_2x2_s2", 2, 8, 8, 64, 64, 2, 2, (2, 2), (0, 0)), ("ph_1x3_s2", 1, 6, 30, 64, 128, 1, 3, (2, 2), (0, 1)),
    ("ph_tiny", 1, 1, 3, 8, 64, 1, 1, (2, 2), (0, 0)),
]


@pytest.mark.parametrize("spec", PHASE_CASES, ids=[c[0] for c in PHASE_CASES])
def test_strided_backward_data_by_phase(env, spec):
    """Stride-2 backward-data without a reduction split walks the input pixels phase by phase ((h % sh, w % sw)) and
    multiplies only the taps that can hit the output grid; with a split, or fp32 gradients, the masked form runs.
    All must agree with the oracle, with and without the fused input ReLU."""
    dp, U, orc = env
    tag, n, h, w, c, k, r, s_, st, pd = spec
    case = U.ConvCase(tag, n, h, w, c, k, r, s_, st, pd, bf16=True, bias=False, relu=True)
    x = np.maximum(case.x, 0.0).astype(np.float32)
    case.x = x
    case.xd = U.bf16_dev(U.synth.f32_to_bf16_bits(x))
    y = case.run_fwd()
    torch.cuda.synchronize()
    want = orc.conv2d_bwd_data(case.dy, case.w, x.shape, y_saved=U.to_np(y), stride=st, pad=pd)
    for variant, splits in ((-1, 0), (200, 1), (204, 1), (207, 1), (212, 1), (226, 1), (200, 2), (207, 3)):
        dp.dp_set_override(1, variant, splits)
        try:
            name = dp.dp_conv2d_kernel_info(case.desc, 1)[0]
            dx = case.run_dgrad(y)
            dxm = case.run_dgrad_relu_in(y)
            torch.cuda.synchronize()
        finally:
            dp.dp_set_override(1, -1, 0)
        U.assert_bf16_close(U.to_np(dx), want, f"{tag} {variant}/{splits} {name}")
        U.assert_bf16_close(U.to_np(dxm), orc.relu_in_backward(want, x), f"{tag} {variant}/{splits} {name} with the input ReLU")
    # fp32 gradients take the same plan in natural pixel order
    case32 = U.ConvCase(tag, n, h, w, c, k, r, s_, st, pd, bf16=True, bias=False, relu=True, dx_f32=True)
    dp.dp_set_override(1, 200, 1)
    try:
        dx32 = case32.run_dgrad(y)
        torch.cuda.synchronize()
    finally:
        dp.dp_set_override(1, -1, 0)
    U.assert_bf16_close(U.to_np(dx32), orc.conv2d_bwd_data(case32.dy, case32.w, case32.x.shape, y_saved=U.to_np(y), stride=st, pad=pd), f"{tag} fp32 dx")


@pytest.mark.parametrize("blocks", [0, 3, 40])
def test_input_patch_filter_gradient_all_taps_per_wave(env, blocks):
    """The 3x3 form of the input-patch filter gradient with all nine taps in one wave (four waves: two pixel groups x two halves of
    c_in; sums of the pixel groups meet in LDS at the end): both tile shapes, ragged edges, c_out below / above one 64-row tile,
    padding 0 and 1, one block with many tiles and more blocks than tiles, with and without the fused bias gradient."""
    dp, U, orc = env
    dp.dp_set_override(2, 411, blocks)
    try:
        for tag, n, h, w, k, pd in (("tapsw_a", 2, 13, 12, 96, (1, 1)), ("tapsw_b", 1, 37, 40, 64, (1, 1)), ("tapsw_c", 3, 20, 70, 40, (0, 0)),
                                    ("tapsw_d", 2, 33, 31, 136, (1, 1)), ("tapsw_e", 5, 16, 16, 64, (1, 1))):
            case = U.ConvCase(tag, n, h, w, 64, k, 3, 3, (1, 1), pd, bf16=True, bias=True, relu=True)
            assert dp.dp_conv2d_kernel_info(case.desc, 2)[0] == "k_wgrad_halo9<true>"
            y = case.run_fwd()
            dw, db = case.run_wgrad(y)   # saved output given: dy is masked first, the bias gradient comes from that pass
            torch.cuda.synchronize()
            rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=U.to_np(y), pad=pd, want_db=True)
            U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} blocks {blocks} dw")
            U.assert_bf16_close(U.to_np(db), rdb, f"{tag} blocks {blocks} db")
            dw, db = case.run_wgrad(None)   # no saved output: the c_in-half-0 waves also sum the bias gradient
            db.fill_(7.0)
            dw, db = case.run_wgrad(None)
            torch.cuda.synchronize()
            rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=None, pad=pd, want_db=True)
            U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} blocks {blocks} dw, unmasked")
            U.assert_bf16_close(U.to_np(db), rdb, f"{tag} blocks {blocks} db, fused")
            dw2, _ = case.run_wgrad(None, want_db=False)
            torch.cuda.synchronize()
            assert torch.equal(dw, dw2), f"{tag}: filter gradient differs when the bias gradient is not asked for"
        # other filter shapes stay with the wave-per-tap kernel
        case = U.ConvCase("tapsw_1x7", 2, 9, 33, 64, 64, 1, 7, (1, 1), (0, 3), bf16=True, bias=True, relu=True)
        assert "halo9" not in dp.dp_conv2d_kernel_info(case.desc, 2)[0]
    finally:
        dp.dp_set_override(2, -1, 0)


@pytest.mark.parametrize("blocks", [0, 3, 40])
def test_input_patch_filter_gradient(env, blocks):
    """Filter gradient with the input patch in LDS and persistent blocks (64 input channels, stride 1): both
    tile shapes, ragged edges, c_out below / above one 64-row tile, 1xS filters, more blocks than tiles."""
    dp, U, orc = env
    dp.dp_set_override(2, 410, blocks)
    try:
        for tag, n, h, w, k, r, s_, pd in (("patchw_a", 2, 13, 12, 96, 3, 3, (1, 1)), ("patchw_b", 1, 37, 40, 64, 3, 3, (1, 1)),
                                           ("patchw_c", 2, 9, 33, 136, 1, 7, (0, 3)), ("patchw_d", 3, 20, 70, 40, 3, 3, (0, 0))):
            case = U.ConvCase(tag, n, h, w, 64, k, r, s_, (1, 1), pd, bf16=True, bias=True, relu=True)
            assert "k_wgrad_halo" in dp.dp_conv2d_kernel_info(case.desc, 2)[0]
            y = case.run_fwd()
            dw, db = case.run_wgrad(y)
            torch.cuda.synchronize()
            rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=U.to_np(y), pad=pd, want_db=True)
            U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} blocks {blocks} dw")
            U.assert_bf16_close(U.to_np(db), rdb, f"{tag} blocks {blocks} db")
            dw, db = case.run_wgrad(None)   # no saved output: two of the tap waves also sum the bias gradient
            torch.cuda.synchronize()
            rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=None, pad=pd, want_db=True)
            U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} blocks {blocks} dw, unmasked")
            U.assert_bf16_close(U.to_np(db), rdb, f"{tag} blocks {blocks} db, fused")
    finally:
        dp.dp_set_override(2, -1, 0)


@pytest.mark.parametrize("variant", [400, 401, 402, 403])
def test_input_patch_variants(env, variant):
    """Kernels that keep the input patch (with halo) of a 256-pixel tile in LDS: 64 reduction channels per
    tap, stride 1; both tile shapes (8x32, 16x16), ragged image edges, several c_out / c_in tiles, 1xS filters."""
    dp, U, orc = env
    dp.dp_set_override(0, variant, 0)
    dp.dp_set_override(1, variant, 0)
    try:
        # forward: c_in = 64
        for tag, n, h, w, k, r, s_, pd in (("patch_a", 2, 13, 12, 96, 3, 3, (1, 1)), ("patch_b", 1, 37, 40, 64, 3, 3, (1, 1)),
                                           ("patch_c", 2, 9, 33, 136, 1, 7, (0, 3)), ("patch_d", 3, 20, 70, 200, 3, 3, (0, 0))):
            case = U.ConvCase(tag, n, h, w, 64, k, r, s_, (1, 1), pd, bf16=True, bias=True, relu=True)
            assert "k_halo<0" in dp.dp_conv2d_kernel_info(case.desc, 0)[0]
            y = case.run_fwd()
            torch.cuda.synchronize()
            U.assert_bf16_close(U.to_np(y), orc.conv2d_fwd(case.x, case.w, case.b, relu=True, stride=(1, 1), pad=pd), f"{tag} variant {variant}")
        # backward-data: c_out = 64
        for tag, n, h, w, c, r, s_, pd in (("patchd_a", 2, 13, 12, 96, 3, 3, (1, 1)), ("patchd_b", 1, 37, 40, 64, 3, 3, (1, 1)),
                                           ("patchd_c", 2, 9, 33, 136, 1, 7, (0, 3)), ("patchd_d", 3, 20, 70, 200, 3, 3, (0, 0))):
            case = U.ConvCase(tag, n, h, w, c, 64, r, s_, (1, 1), pd, bf16=True, bias=True, relu=True)
            assert "k_halo<1" in dp.dp_conv2d_kernel_info(case.desc, 1)[0]
            y = case.run_fwd()
            dx = case.run_dgrad(y)
            torch.cuda.synchronize()
            U.assert_bf16_close(U.to_np(dx), orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=U.to_np(y), pad=pd), f"{tag} variant {variant} dx")
        # a patch that does not fit (5x5 filter) falls back to another kernel
        case = U.ConvCase("patch_big", 1, 20, 20, 64, 64, 5, 5, (1, 1), (2, 2), bf16=True, bias=True, relu=True)
        assert "k_halo" not in dp.dp_conv2d_kernel_info(case.desc, 0)[0]
    finally:
        dp.dp_set_override(0, -1, 0)
        dp.dp_set_override(1, -1, 0)


RELU_IN_CASES = [
    # tag, n, h, w, c, k, r, s, stride, pad, bf16, dx_f32, (variant, splits) overrides of the backward-data pass
    ("mask_pipe", 2, 13, 12, 72, 128, 3, 3, (1, 1), (1, 1), True, False, [(-1, 0), (200, 1), (200, 3), (204, 1), (226, 1), (100, 1), (103, 2), (0, 1), (2, 3)]),
    ("mask_patch", 2, 20, 33, 96, 64, 3, 3, (1, 1), (1, 1), True, False, [(-1, 0), (400, 0), (403, 0), (404, 0)]),
    ("mask_stride2", 2, 15, 15, 64, 64, 3, 3, (2, 2), (1, 1), True, False, [(-1, 0), (200, 1), (200, 2)]),
    ("mask_1x1", 3, 14, 14, 256, 64, 1, 1, (1, 1), (0, 0), True, False, [(-1, 0), (207, 2)]),
    ("mask_odd_channels", 2, 9, 10, 24, 40, 3, 3, (1, 1), (1, 1), True, False, [(-1, 0), (1, 2)]),
    ("mask_c12", 1, 8, 8, 12, 16, 3, 3, (1, 1), (1, 1), True, False, [(-1, 0)]),
    ("mask_dx_f32", 2, 13, 12, 72, 64, 3, 3, (1, 1), (1, 1), True, True, [(-1, 0), (200, 1), (200, 3), (404, 0)]),
    ("mask_fp32", 2, 9, 8, 5, 7, 3, 3, (1, 1), (1, 1), False, False, [(-1, 0)]),
]


@pytest.mark.parametrize("spec", RELU_IN_CASES, ids=[c[0] for c in RELU_IN_CASES])
def test_backward_data_with_fused_input_relu(env, spec):
    """DP_RELU_IN: dx * [x > 0] leaves in the epilogue of every backward-data kernel family (staged and direct
    stores, split reductions, input-patch kernels; the stationary-weight kernel hands over to another one)."""
    dp, U, orc = env
    tag, n, h, w, c, k, r, s_, st, pd, bf16, dxf, overrides = spec
    case = U.ConvCase(tag, n, h, w, c, k, r, s_, st, pd, bf16=bf16, bias=True, relu=True, dx_f32=dxf)
    # the layer's input as a ReLU would leave it: about half zeros
    x = np.maximum(case.x, 0.0).astype(np.float32)
    case.x = x
    case.xd = U.bf16_dev(U.synth.f32_to_bf16_bits(x)) if bf16 else torch.from_numpy(x).to(U.DEV)
    y = case.run_fwd()
    torch.cuda.synchronize()
    want = orc.relu_in_backward(orc.conv2d_bwd_data(case.dy, case.w, x.shape, y_saved=U.to_np(y), stride=st, pad=pd), x)
    assert (want == 0).mean() > 0.3
    for variant, splits in overrides:
        dp.dp_set_override(1, variant, splits)
        try:
            dx = case.run_dgrad_relu_in(y)
            torch.cuda.synchronize()
        finally:
            dp.dp_set_override(1, -1, 0)
        got = U.to_np(dx)
        assert np.array_equal(got == 0, want == 0) or np.abs(got[(got == 0) != (want == 0)]).max() < 1e-30, f"{tag} {variant}/{splits}: mask differs"
        if bf16:
            U.assert_bf16_close(got, want, f"{tag} variant {variant} splits {splits}")
        else:
            U.assert_f32_close(got, want, f"{tag} fp32")
    # without the flag the saved input is ignored; the flag without a saved input is an error
    dx_plain = torch.empty_like(dx)
    dp.dp_conv2d_bwd_data_relu(case.desc, case.dyd, y, case.wd, case.xd, dx_plain, case.ws())
    torch.cuda.synchronize()
    ref_plain = orc.conv2d_bwd_data(case.dy, case.w, x.shape, y_saved=U.to_np(y), stride=st, pad=pd)
    (U.assert_bf16_close if bf16 else U.assert_f32_close)(U.to_np(dx_plain), ref_plain, f"{tag} unmasked")
    d = dp.dp_conv_desc.from_buffer_copy(case.desc)
    d.flags |= dp.DP_RELU_IN
    with pytest.raises(dp.DpError):
        dp.dp_conv2d_bwd_data(d, case.dyd, y, case.wd, dx_plain, case.ws())


def test_dense_backward_with_fused_input_relu(env):
    dp, U, orc = env
    for n, i, o in ((4, 256, 72), (32, 1024, 1000), (1, 4096, 1000)):
        x, W, b = U.synth.linear_tensors(f"fcmask/{n}/{i}/{o}", n, i, o)
        x = np.maximum(U.synth.round_bf16(x), 0.0)
        W = U.synth.round_bf16(W)
        dy = U.synth.round_bf16(U.synth.upstream_grad(f"fcmask/{n}/{i}/{o}", (n, o)))
        xd, Wd, dyd = (U.bf16_dev(U.synth.f32_to_bf16_bits(a)) for a in (x, W, dy))
        d = dp.linear_desc(n, i, o, dp.DP_BF16, dp.DP_RELU_IN)
        dx = torch.empty((n, i), dtype=torch.bfloat16, device=U.DEV)
        ws = U.workspace(dp.dp_linear_workspace_bytes(d))
        dp.dp_linear_fwd_bwd(d, x=xd, W=Wd, dy=dyd, dx=dx, ws=ws)
        torch.cuda.synchronize()
        want = orc.relu_in_backward(orc.linear_bwd(x, W, dy)[0], x)
        U.assert_bf16_close(U.to_np(dx), want, f"dense {n}x{i}x{o}")
        assert np.array_equal(U.to_np(dx) == 0, want == 0)


@pytest.mark.parametrize("blocks", [0, 1, 7])
def test_input_patch_stationary_weights(env, blocks):
    """3x3, stride 1, 64 reduction channels: persistent kernel with the weight fragments in registers.  Block
    counts below the tile count make every block walk several tiles (both patch buffers, delayed stores)."""
    dp, U, orc = env
    dp.dp_set_override(0, 404, blocks)
    dp.dp_set_override(1, 404, blocks)
    try:
        for tag, n, h, w, k, pd in (("ws_a", 2, 13, 12, 96, (1, 1)), ("ws_b", 1, 37, 40, 64, (1, 1)), ("ws_c", 3, 20, 70, 200, (0, 0)),
                                    ("ws_d", 2, 16, 16, 8, (2, 2))):
            case = U.ConvCase(tag, n, h, w, 64, k, 3, 3, (1, 1), pd, bf16=True, bias=True, relu=True)
            assert "k_halo_ws<0, false>" in dp.dp_conv2d_kernel_info(case.desc, 0)[0]
            y = case.run_fwd()
            torch.cuda.synchronize()
            U.assert_bf16_close(U.to_np(y), orc.conv2d_fwd(case.x, case.w, case.b, relu=True, stride=(1, 1), pad=pd), f"{tag} blocks {blocks}")
        for tag, n, h, w, c, pd in (("wsd_a", 2, 13, 12, 96, (1, 1)), ("wsd_b", 1, 37, 40, 64, (1, 1)), ("wsd_c", 3, 20, 70, 200, (0, 0)),
                                    ("wsd_d", 2, 16, 16, 8, (2, 2))):
            case = U.ConvCase(tag, n, h, w, c, 64, 3, 3, (1, 1), pd, bf16=True, bias=True, relu=True)
            assert "k_halo_ws<1, " in dp.dp_conv2d_kernel_info(case.desc, 1)[0]
            y = case.run_fwd()
            dx = case.run_dgrad(y)
            torch.cuda.synchronize()
            U.assert_bf16_close(U.to_np(dx), orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=U.to_np(y), pad=pd), f"{tag} blocks {blocks} dx")
        # other filter shapes and fp32 gradients are not this kernel's
        case = U.ConvCase("ws_1x7", 1, 9, 33, 64, 64, 1, 7, (1, 1), (0, 3), bf16=True, bias=True, relu=True)
        assert "k_halo_ws" not in dp.dp_conv2d_kernel_info(case.desc, 0)[0]
        case = U.ConvCase("ws_f32", 2, 13, 12, 72, 64, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True, dx_f32=True)
        assert "k_halo" not in dp.dp_conv2d_kernel_info(case.desc, 1)[0]
        y = case.run_fwd()
        dx = case.run_dgrad(y)
        torch.cuda.synchronize()
        assert dx.dtype == torch.float32
        U.assert_bf16_close(U.to_np(dx), orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=U.to_np(y), pad=(1, 1)), "ws_f32 dx")
    finally:
        dp.dp_set_override(0, -1, 0)
        dp.dp_set_override(1, -1, 0)


@pytest.mark.parametrize("splits", [1, 2])
@pytest.mark.parametrize("tile", [(256, 256), (128, 256), (256, 128), (224, 256)])
def test_forward_pixel_strip_kernel(env, tile, splits):
    """3x3, stride 1, pad 1, c_in % 128 == 0: the forward kernel that keeps one strip of input pixels in LDS for the three
    taps of a filter row and redirects (pixel, tap) pairs outside the image to rows of zeros.  Ragged last tiles in
    both directions, tiles that span several images, images narrower than the filter, one and several channel
    blocks, with and without the epilogue; tiles of 256 x 256 (two weight stages), 128 pixel rows and 128 channels (three), and
    224 pixel rows (each wave 64 channels x 224 pixels)."""
    dp, U, orc = env
    rows, chans = tile
    dp.dp_set_override(0, {(256, 256): 230, (128, 256): 231, (256, 128): 232, (224, 256): 233}[tile], splits)   # a split takes an even number of 64-channel blocks
    try:
        for tag, n, h, w, c, k, epi in (("st_a", 2, 13, 12, 128, 96, True), ("st_b", 1, 37, 40, 256, 264, True), ("st_c", 3, 5, 70, 128, 8, False),
                                        ("st_d", 5, 9, 3, 128, 64, True), ("st_e", 1, 1, 1, 128, 16, True), ("st_f", 7, 2, 2, 384, 40, False),
                                        ("st_g", 2, 11, 9, 512, 72, True)):
            case = U.ConvCase(tag, n, h, w, c, k, 3, 3, (1, 1), (1, 1), bf16=True, bias=epi, relu=epi)
            assert dp.dp_conv2d_kernel_info(case.desc, 0) == (f"k_conv_strip<false, {rows}, {chans}>", splits if (c // 64) % (2 * splits) == 0 else 1)
            y = case.run_fwd()
            torch.cuda.synchronize()
            U.assert_bf16_close(U.to_np(y), orc.conv2d_fwd(case.x, case.w, case.b if epi else None, relu=epi, stride=(1, 1), pad=(1, 1)), tag)
        # other shapes are not this kernel's: 64 input channels, no padding, stride 2, 5x5
        for tag, c, r, st, pd in (("st_c64", 64, 3, (1, 1), (1, 1)), ("st_p0", 128, 3, (1, 1), (0, 0)), ("st_s2", 128, 3, (2, 2), (1, 1)),
                                  ("st_5x5", 128, 5, (1, 1), (2, 2))):
            case = U.ConvCase(tag, 1, 12, 12, c, 32, r, r, st, pd, bf16=True, bias=True, relu=True)
            assert "k_conv_strip" not in dp.dp_conv2d_kernel_info(case.desc, 0)[0]
    finally:
        dp.dp_set_override(0, -1, 0)


@pytest.mark.parametrize("splits", [1, 2])
@pytest.mark.parametrize("tile", [(256, 256), (128, 256), (256, 128), (224, 256)])
def test_backward_data_pixel_strip_kernel(env, tile, splits):
    """The same kernel on the backward-data pass (c_out % 128 == 0): mirrored filter, weights through the LDS transpose
    read, with and without the fused backward of the input ReLU; fp32 gradients are not this kernel's."""
    dp, U, orc = env
    rows, chans = tile
    dp.dp_set_override(1, {(256, 256): 230, (128, 256): 231, (256, 128): 232, (224, 256): 233}[tile], splits)
    try:
        for tag, n, h, w, c, k in (("sd_a", 2, 13, 12, 96, 128), ("sd_b", 1, 37, 40, 264, 256), ("sd_c", 3, 5, 70, 8, 128),
                                   ("sd_d", 5, 9, 3, 64, 128), ("sd_e", 1, 1, 1, 16, 128), ("sd_f", 7, 2, 2, 40, 384), ("sd_g", 2, 11, 9, 72, 512)):
            case = U.ConvCase(tag, n, h, w, c, k, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True)
            assert dp.dp_conv2d_kernel_info(case.desc, 1) == (f"k_conv_strip<true, {rows}, {chans}>", splits if (k // 64) % (2 * splits) == 0 else 1)
            y = case.run_fwd()
            dx = case.run_dgrad(y)          # the incoming gradient is masked by the saved output first
            torch.cuda.synchronize()
            ref = orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=U.to_np(y), pad=(1, 1))
            U.assert_bf16_close(U.to_np(dx), ref, tag)
            dxm = case.run_dgrad_relu_in(y)      # the backward of the ReLU in front of the layer rides in the epilogue
            torch.cuda.synchronize()
            U.assert_bf16_close(U.to_np(dxm), orc.relu_in_backward(ref, case.x), tag + " masked")
        case = U.ConvCase("sd_f32", 2, 13, 12, 72, 128, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True, dx_f32=True)
        assert "k_conv_strip" not in dp.dp_conv2d_kernel_info(case.desc, 1)[0]
        dx = case.run_dgrad(None)
        torch.cuda.synchronize()
        assert dx.dtype == torch.float32
        U.assert_bf16_close(U.to_np(dx), orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=None, pad=(1, 1)), "sd_f32")
        case = U.ConvCase("sd_k64", 1, 12, 12, 32, 64, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True)
        assert "k_conv_strip" not in dp.dp_conv2d_kernel_info(case.desc, 1)[0]
    finally:
        dp.dp_set_override(1, -1, 0)


@pytest.mark.parametrize("variant", [300, 301, 302, 303, 304, 305, 306, 307, 308, 309, 310, 311, 312, 313, 314, 315])
@pytest.mark.parametrize("splits", [1, 3])
def test_pipelined_backward_filter_variants(env, variant, splits):
    """Backward-filter kernels with the direct-to-LDS pipeline and LDS transpose reads."""
    dp, U, orc = env
    dp.dp_set_override(2, variant, splits)
    try:
        for tag, n, h, w, c, k, r, s_, st, pd in (("pipew_a", 2, 13, 12, 64, 96, 3, 3, (1, 1), (1, 1)),
                                                  ("pipew_b", 3, 15, 14, 40, 72, 3, 3, (2, 2), (1, 1)),
                                                  ("pipew_c", 1, 9, 17, 136, 200, 1, 7, (1, 1), (0, 3))):
            case = U.ConvCase(tag, n, h, w, c, k, r, s_, st, pd, bf16=True, bias=True, relu=True)
            assert "wgrad_dma" in dp.dp_conv2d_kernel_info(case.desc, 2)[0]
            y = case.run_fwd()
            dw, db = case.run_wgrad(y)
            torch.cuda.synchronize()
            y_np = U.to_np(y)
            rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=y_np, stride=st, pad=pd, want_db=True)
            U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} variant {variant} splits {splits} dw")
            U.assert_bf16_close(U.to_np(db), rdb, f"{tag} variant {variant} splits {splits} db")
            # no saved output: the kernel itself sums the bias gradient (column sums on the matrix cores)
            dw, db = case.run_wgrad(None)
            db.fill_(7.0)
            dw, db = case.run_wgrad(None)
            torch.cuda.synchronize()
            rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=None, stride=st, pad=pd, want_db=True)
            U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} variant {variant} splits {splits} dw, unmasked")
            U.assert_bf16_close(U.to_np(db), rdb, f"{tag} variant {variant} splits {splits} db, fused")
    finally:
        dp.dp_set_override(2, -1, 0)


@pytest.mark.parametrize("splits", [1, 3])
def test_filter_gradient_pixel_strip_kernel(env, splits):
    """3x3, stride 1, pad 1, c_in % 64 == 0: the filter-gradient kernel that pads every image row to a power-of-two number
    of pixel slots and shares one strip of x between the three taps of a filter row.  Row widths that fill a segment
    exactly (14), almost (28, 56, 30) and to three quarters (12); one, two and four image rows per step; steps that
    straddle images and run past the last row; c_out below, at and above one tile; 3 to 24 tap-and-channel tiles; with
    the saved-output mask and the bias gradient (a separate pass here) and without."""
    dp, U, orc = env
    dp.dp_set_override(2, 316, splits)
    try:
        for tag, n, h, w, c, k in (("wsx_a", 2, 5, 28, 64, 256), ("wsx_b", 1, 9, 14, 128, 72), ("wsx_c", 3, 4, 56, 64, 264),
                                   ("wsx_d", 2, 7, 12, 192, 16), ("wsx_e", 1, 1, 14, 64, 8), ("wsx_f", 5, 3, 30, 64, 40),
                                   ("wsx_g", 2, 6, 14, 256, 40), ("wsx_h", 2, 14, 14, 512, 264), ("wsx_i", 1, 20, 28, 320, 24)):
            case = U.ConvCase(tag, n, h, w, c, k, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True)
            name, got_splits = dp.dp_conv2d_kernel_info(case.desc, 2)
            assert name == "k_wgrad_strip" and 1 <= got_splits <= splits
            y = case.run_fwd()
            dw, db = case.run_wgrad(y)
            torch.cuda.synchronize()
            rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=U.to_np(y), stride=(1, 1), pad=(1, 1), want_db=True)
            U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} splits {splits} dw")
            U.assert_bf16_close(U.to_np(db), rdb, f"{tag} splits {splits} db")
            dw, db = case.run_wgrad(None)
            torch.cuda.synchronize()
            rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=None, stride=(1, 1), pad=(1, 1), want_db=True)
            U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} splits {splits} dw, unmasked")
            U.assert_bf16_close(U.to_np(db), rdb, f"{tag} splits {splits} db, unmasked")
        # other shapes are not this kernel's: rows that would leave more than a quarter of their slots empty or are too long,
        # 48 input channels, other filters and strides
        for tag, w, c, r, st, pd in (("wsx_w40", 40, 64, 3, (1, 1), (1, 1)), ("wsx_w70", 70, 64, 3, (1, 1), (1, 1)), ("wsx_c48", 14, 48, 3, (1, 1), (1, 1)),
                                     ("wsx_1x1", 14, 64, 1, (1, 1), (0, 0)), ("wsx_s2", 14, 64, 3, (2, 2), (1, 1))):
            case = U.ConvCase(tag, 1, 6, w, c, 32, r, r, st, pd, bf16=True, bias=True, relu=True)
            assert dp.dp_conv2d_kernel_info(case.desc, 2)[0] != "k_wgrad_strip"
    finally:
        dp.dp_set_override(2, -1, 0)


def test_unfused_relu_gradient_flow(env):
    """dp_relu_bias_grad materialises the masked gradient once; both backward passes then take it
    with y_saved = NULL and must agree with the oracle's masked definitions."""
    dp, U, orc = env
    case = U.ConvCase("unfused", 2, 28, 28, 64, 128, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True)
    n, h, w, c, k, r, s = case.shape
    y = case.run_fwd()
    g = torch.empty_like(case.dyd)
    db = torch.empty((k,), dtype=torch.float32, device=U.DEV)
    rows = n * case.ho * case.wo
    ws = U.workspace(max(dp.dp_relu_bias_grad_workspace_bytes(rows, k), *(dp.dp_conv2d_workspace_bytes(case.desc, p) for p in range(3))))
    dp.dp_relu_bias_grad(rows, k, dp.DP_BF16, case.dyd, y, g, db, ws)
    dx = torch.empty((n, h, w, c), dtype=torch.bfloat16, device=U.DEV)
    dw = torch.empty((k, r, s, c), dtype=torch.float32, device=U.DEV)
    dp.dp_conv2d_bwd_data(case.desc, g, None, case.wd, dx, ws)
    dp.dp_conv2d_bwd_filter(case.desc, case.xd, g, None, dw, None, ws)
    torch.cuda.synchronize()
    y_np = U.to_np(y)
    U.assert_bf16_close(U.to_np(dx), orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=y_np, pad=(1, 1)), "unfused dx")
    rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=y_np, pad=(1, 1), want_db=True)
    U.assert_bf16_close(U.to_np(dw), rdw, "unfused dw")
    U.assert_bf16_close(U.to_np(db), rdb, "unfused db")


def test_bitwise_deterministic(env):
    dp, U, orc = env
    case = U.ConvCase("det", 2, 28, 28, 64, 128, 3, 3, (1, 1), (1, 1), bf16=True)
    y1 = case.run_fwd(); dw1, db1 = case.run_wgrad(y1); dx1 = case.run_dgrad(y1)
    y2 = case.run_fwd(); dw2, db2 = case.run_wgrad(y2); dx2 = case.run_dgrad(y2)
    torch.cuda.synchronize()
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))
    assert torch.equal(dx1.view(torch.int16), dx2.view(torch.int16))
    assert torch.equal(dw1, dw2) and torch.equal(db1, db2)


@pytest.mark.parametrize("mode", [1, 2], ids=["warm", "cold"])
def test_measured_kernel_choice(env, mode):
    """With the measured choice on (back-to-back launches, or the caches flushed before every timed launch), the first call
    of each pass times the candidates on the caller's buffers: results must match the oracle on that call and on the next
    (cached plan), the workspace the query asks for must suffice, and the choice must stay the same afterwards."""
    dp, U, orc = env
    dp.dp_set_autotune(mode)
    try:
        for tag, n, h, w, c, k, pd in ((f"tune_a{mode}", 2, 28 + mode, 28, 64, 128, (1, 1)), (f"tune_b{mode}", 1, 14, 14 + mode, 128, 192, (1, 1))):
            case = U.ConvCase(tag, n, h, w, c, k, 3, 3, (1, 1), pd, bf16=True, bias=True, relu=True)
            for rep in range(2):
                y = case.run_fwd()
                dw, db = case.run_wgrad(y)
                dx = case.run_dgrad(y)
                torch.cuda.synchronize()
                y_np = U.to_np(y)
                U.assert_bf16_close(y_np, orc.conv2d_fwd(case.x, case.w, case.b, relu=True, pad=pd), f"{tag} y rep {rep}")
                U.assert_bf16_close(U.to_np(dx), orc.conv2d_bwd_data(case.dy, case.w, case.x.shape, y_saved=y_np, pad=pd), f"{tag} dx rep {rep}")
                rdw, rdb = orc.conv2d_bwd_filter(case.x, case.dy, case.w.shape, y_saved=y_np, pad=pd, want_db=True)
                U.assert_bf16_close(U.to_np(dw), rdw, f"{tag} dw rep {rep}")
                U.assert_bf16_close(U.to_np(db), rdb, f"{tag} db rep {rep}")
                info = [dp.dp_conv2d_kernel_info(case.desc, p) for p in range(3)]
                if rep == 0:
                    first = info
                assert info == first
        # DP_DETERMINISTIC keeps a call on the analytic choice even while the measured choice is on
        d_det = dp.conv_desc(2, 28, 28, 64, 128, 3, 3, (1, 1), (1, 1), dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU | dp.DP_DETERMINISTIC)
        while_on = [dp.dp_conv2d_kernel_info(d_det, p) for p in range(3)]
        dp.dp_set_autotune(False)
        assert while_on == [dp.dp_conv2d_kernel_info(d_det, p) for p in range(3)]
    finally:
        dp.dp_set_autotune(False)


def test_dense_forward_kernel_names(env):
    """Which forward kernel a dense layer gets (names as the profiler shows them)."""
    dp, U, orc = env
    assert dp.dp_conv2d_kernel_info(dp.conv_desc(16, 1, 1, 4096, 1000, 1, 1, (1, 1), (0, 0), dp.DP_BF16, dp.DP_BIAS), 0)[0] == "k_dense_fwd<1>"
    assert dp.dp_conv2d_kernel_info(dp.conv_desc(17, 1, 1, 4096, 1000, 1, 1, (1, 1), (0, 0), dp.DP_BF16, dp.DP_BIAS), 0)[0] != "k_dense_fwd<1>"
    assert dp.dp_conv2d_kernel_info(dp.conv_desc(4, 1, 1, 448, 1000, 1, 1, (1, 1), (0, 0), dp.DP_BF16, dp.DP_BIAS), 0)[0] != "k_dense_fwd<1>"
    # backward-data: the streaming kernel takes the shapes whose output count is not a multiple of 64 (the cases (1, 4096, 1000) and
    # (5, 200, 136) of test_linear_parity run it, the second with a ragged last block of input features)
    assert dp.dp_conv2d_kernel_info(dp.conv_desc(32, 1, 1, 4096, 1000, 1, 1, (1, 1), (0, 0), dp.DP_BF16, 0), 1)[0] == "k_dense_dgrad"
    assert dp.dp_conv2d_kernel_info(dp.conv_desc(5, 1, 1, 200, 136, 1, 1, (1, 1), (0, 0), dp.DP_BF16, 0), 1)[0] == "k_dense_dgrad"
    assert dp.dp_conv2d_kernel_info(dp.conv_desc(32, 1, 1, 4096, 4096, 1, 1, (1, 1), (0, 0), dp.DP_BF16, 0), 1)[0] != "k_dense_dgrad"
    # filter gradient: gradients of 4 to 128 MB
    assert dp.dp_conv2d_kernel_info(dp.conv_desc(32, 1, 1, 4096, 1000, 1, 1, (1, 1), (0, 0), dp.DP_BF16, 0), 2)[0] == "k_dense_wgrad<false>"
    assert dp.dp_conv2d_kernel_info(dp.conv_desc(1, 1, 1, 25088, 4096, 1, 1, (1, 1), (0, 0), dp.DP_BF16, 0), 2)[0][:13] != "k_dense_wgrad"


# ---- dense layers ----------------------------------------------------------------------------
# up to 16 samples with at least 512 input features (a multiple of 64) take the streaming forward kernel: whole and ragged
# 16-row groups of outputs, an output count that is not a multiple of 4, features that do not divide evenly over the eight waves
@pytest.mark.parametrize("n,i,o,bf16", [(5, 200, 136, True), (32, 1024, 512, True), (1, 4096, 1000, True),
                                        (16, 512, 48, True), (7, 1600, 42, True), (2, 576, 200, True), (17, 512, 64, True),
                                        (9, 1032, 1016, True), (20, 2048, 520, True),   # streaming filter gradient, ragged tiles both ways
                                        (3, 50, 20, False)])
def test_linear_parity(env, n, i, o, bf16):
    dp, U, orc = env
    from paper_2112_10065_amd import synth
    x, W, b = synth.linear_tensors(f"lin{n}_{i}_{o}", n, i, o)
    dy = synth.upstream_grad(f"lin{n}_{i}_{o}", (n, o))
    if bf16:
        xb, Wb, dyb = (synth.f32_to_bf16_bits(a) for a in (x, W, dy))
        x, W, dy = (synth.bf16_bits_to_f32(a) for a in (xb, Wb, dyb))
        xd, Wd, dyd = U.bf16_dev(xb), U.bf16_dev(Wb), U.bf16_dev(dyb)
        tdt = torch.bfloat16
    else:
        xd, Wd, dyd = (torch.from_numpy(a).to(U.DEV) for a in (x, W, dy))
        tdt = torch.float32
    bd = torch.from_numpy(b).to(U.DEV)
    desc = dp.linear_desc(n, i, o, dp.DP_BF16 if bf16 else dp.DP_F32, dp.DP_BIAS | dp.DP_RELU)
    ws = U.workspace(dp.dp_linear_workspace_bytes(desc))
    y = torch.empty((n, o), dtype=tdt, device=U.DEV)
    dx = torch.empty((n, i), dtype=tdt, device=U.DEV)
    dW = torch.empty((o, i), dtype=torch.float32, device=U.DEV)
    db = torch.empty((o,), dtype=torch.float32, device=U.DEV)
    dp.dp_linear_fwd_bwd(desc, x=xd, W=Wd, bias=bd, y=y, ws=ws)                      # forward half
    dp.dp_linear_fwd_bwd(desc, x=xd, W=Wd, dy=dyd, y_saved=y, dx=dx, dW=dW, dbias=db, ws=ws)  # backward half
    torch.cuda.synchronize()
    y_np = U.to_np(y)
    chk = U.assert_bf16_close if bf16 else U.assert_f32_close
    chk(y_np, orc.linear_fwd(x, W, b, relu=True), "linear y")
    rdx, rdW, rdb = orc.linear_bwd(x, W, dy, y_np)
    chk(U.to_np(dx), rdx, "linear dx")
    chk(U.to_np(dW), rdW, "linear dW")
    chk(U.to_np(db), rdb, "linear db")


# ---- ReLU / bias gradient -----------------------------------------------------------------
@pytest.mark.parametrize("rows,k,bf16", [(1000, 64, True), (777, 512, True), (50, 4096, True), (33, 1000, True),
                                         (300, 24, True), (65, 12, True), (130, 16, False)])
def test_relu_bias_grad(env, rows, k, bf16):
    dp, U, orc = env
    from paper_2112_10065_amd import synth
    dy = synth.normal(f"rbg{rows}_{k}/dy", (rows, k))
    y = np.maximum(synth.normal(f"rbg{rows}_{k}/y", (rows, k)), 0).astype(np.float32)
    if bf16:
        dyb, yb = synth.f32_to_bf16_bits(dy), synth.f32_to_bf16_bits(y)
        dy, y = synth.bf16_bits_to_f32(dyb), synth.bf16_bits_to_f32(yb)
        dyd, yd = U.bf16_dev(dyb), U.bf16_dev(yb)
    else:
        dyd, yd = torch.from_numpy(dy).to(U.DEV), torch.from_numpy(y).to(U.DEV)
    g = torch.empty_like(dyd)
    db = torch.empty((k,), dtype=torch.float32, device=U.DEV)
    ws = U.workspace(dp.dp_relu_bias_grad_workspace_bytes(rows, k))
    dp.dp_relu_bias_grad(rows, k, dp.DP_BF16 if bf16 else dp.DP_F32, dyd, yd, g, db, ws)
    torch.cuda.synchronize()
    rg, rdb = orc.relu_bias_grad(dy, y)
    np.testing.assert_array_equal(U.to_np(g), rg.astype(np.float32))  # masking is exact
    rel, mx = U.errs(U.to_np(db), rdb)
    assert rel <= 1e-5, (rel, mx)


# Full-size layers of the benchmark workload at every per-GPU batch: tests/test_gpu_full_size.py; the chained step:
# tests/test_gpu_chain.py.


# ---- the planner's table --------------------------------------------------------------------
def test_profile_layer_rows(env):
    dp, U, orc = env
    d = dp.conv_desc(1, 28, 28, 256, 512, 3, 3, (1, 1), (1, 1), dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU)
    rows = dp.dp_profile_layer(conv=d, batches=(1, 2, 4), warmup=2, iters=5)
    assert [r["batch"] for r in rows] == [1, 2, 4]
    for r in rows:
        assert r["fwd_us"] > 0 and r["dgrad_us"] > 0 and r["wgrad_us"] > 0
        assert r["flops_per_pass"] == 2.0 * r["batch"] * 28 * 28 * 512 * 9 * 256
        assert r["min_bytes_fwd"] > 0
    ld = dp.linear_desc(1, 4096, 1000, dp.DP_BF16, dp.DP_BIAS)
    rows = dp.dp_profile_layer(linear=ld, batches=(1, 32), warmup=1, iters=3)
    assert rows[1]["flops_per_pass"] == 2.0 * 32 * 4096 * 1000 and rows[0]["wgrad_us"] > 0


def test_trace_rows_and_profile_table_agree(env):
    """dp_trace_begin / dp_trace_end: one row per pass in call order, naming the kernel dp_conv2d_kernel_info names; and
    the planner's table (dp_profile_layer: back-to-back launches between two events) agrees with those per-call event
    timings within a band of 0.5x .. 1.6x on a layer whose kernels take tens of microseconds (the trace's events sit
    between dependent launches, so its figures run a few microseconds higher)."""
    dp, U, orc = env
    flags = dp.DP_BIAS | dp.DP_RELU | dp.DP_RELU_IN
    n, hw, c, k = 8, 28, 512, 512
    case = U.ConvCase("trace", n, hw, hw, c, k, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True)
    d = dp.conv_desc(n, hw, hw, c, k, 3, 3, (1, 1), (1, 1), dp.DP_BF16, flags)
    ws = U.workspace(max(dp.dp_conv2d_workspace_bytes(d, p) for p in range(3)))
    y = torch.empty((n, hw, hw, k), dtype=torch.bfloat16, device=U.DEV)
    dx = torch.empty((n, hw, hw, c), dtype=torch.bfloat16, device=U.DEV)
    dw = torch.empty((k, 3, 3, c), dtype=torch.float32, device=U.DEV)
    db = torch.empty((k,), dtype=torch.float32, device=U.DEV)

    def three_passes():
        dp.dp_conv2d_fwd(d, case.xd, case.wd, case.bd, y, ws)
        dp.dp_conv2d_bwd_data_relu(d, case.dyd, None, case.wd, case.xd, dx, ws)
        dp.dp_conv2d_bwd_filter(d, case.xd, case.dyd, None, dw, db, ws)

    three_passes()
    torch.cuda.synchronize()
    runs = []
    for _ in range(7):
        dp.dp_trace_begin()
        three_passes()
        rows = dp.dp_trace_end()
        assert [r["pass"] for r in rows] == [0, 1, 2]
        for p, r in enumerate(rows):
            name, splits = dp.dp_conv2d_kernel_info(d, p)
            assert r["kernel"] == name and r["splits"] == splits
            assert 0.0 < r["main_us"] <= r["total_us"] * 1.001
        runs.append(rows)
    with pytest.raises(dp.DpError):
        dp.dp_trace_end()          # nothing is being recorded any more
    # results are not disturbed by the events
    torch.cuda.synchronize()
    U.assert_bf16_close(U.to_np(y), orc.conv2d_fwd(case.x, case.w, case.b, relu=True, pad=(1, 1)), "traced forward")
    traced = [sorted(r[p]["total_us"] for r in runs)[len(runs) // 2] for p in range(3)]
    prof = dp.dp_profile_layer(conv=d, batches=(n,), warmup=0, iters=20)[0]
    for p, key in enumerate(("fwd_us", "dgrad_us", "wgrad_us")):
        ratio = prof[key] / traced[p]
        assert 0.5 <= ratio <= 1.6, (key, prof[key], traced[p])
    # a dense call yields one row per half it ran
    ld = dp.linear_desc(4, 512, 256, dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU)
    x, W, b = U.synth.linear_tensors("trace/fc", 4, 512, 256)
    xd, Wd = (U.bf16_dev(U.synth.f32_to_bf16_bits(a)) for a in (x, W))
    dyd = U.bf16_dev(U.synth.f32_to_bf16_bits(U.synth.upstream_grad("trace/fc", (4, 256))))
    yl = torch.empty((4, 256), dtype=torch.bfloat16, device=U.DEV)
    dxl = torch.empty((4, 512), dtype=torch.bfloat16, device=U.DEV)
    dWl = torch.empty((256, 512), dtype=torch.float32, device=U.DEV)
    wsl = U.workspace(dp.dp_linear_workspace_bytes(ld))
    dp.dp_trace_begin()
    dp.dp_linear_fwd_bwd(ld, x=xd, W=Wd, bias=torch.from_numpy(b).to(U.DEV), y=yl, ws=wsl)
    dp.dp_linear_fwd_bwd(ld, x=xd, W=Wd, dy=dyd, dx=dxl, dW=dWl, ws=wsl)
    assert [r["pass"] for r in dp.dp_trace_end()] == [0, 1, 2]


def test_profile_layer_with_measured_choice_and_no_warmup(env):
    """With the measured kernel choice on and warmup = 0 the candidates of a new shape are timed in the untimed call that
    precedes the window: the reported time is a layer time (well under a millisecond here), not the tuning time."""
    dp, U, orc = env
    dp.dp_set_autotune(True)
    try:
        d = dp.conv_desc(1, 20, 20, 192, 320, 3, 3, (1, 1), (1, 1), dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU)   # a shape no other test uses
        r = dp.dp_profile_layer(conv=d, batches=(3,), warmup=0, iters=3)[0]
        assert 0 < r["fwd_us"] < 300 and 0 < r["dgrad_us"] < 300 and 0 < r["wgrad_us"] < 300, r
    finally:
        dp.dp_set_autotune(False)


# ---- ResNet-50 and Inception-v3-style layer lists (configurations 3 and 4), full size, spot-checked --------
def _sampled_layer_check(dp, U, orc, l, n, tag):
    st, pd = (l.sh, l.sw), (l.ph, l.pw)
    dxf = l.c < 8
    case = U.ConvCase(f"{tag}/{l.name}", n, l.h, l.w, l.c, l.k, l.r, l.s, st, pd, bf16=True, bias=l.bias, relu=True, dx_f32=dxf)
    y = case.run_fwd()
    dx = case.run_dgrad(y)
    dw, db = case.run_wgrad(y)
    torch.cuda.synchronize()
    rng = np.random.default_rng(abs(hash(l.name)) % (1 << 31))
    y_np = U.to_np(y)
    idx = rng.integers(0, y_np.size, 1500)
    idx[:16] = np.arange(16)
    idx[16:32] = y_np.size - 1 - np.arange(16)
    U.assert_bf16_close(y_np.ravel()[idx], orc.conv2d_fwd_at(case.x, case.w, case.b, True, st, pd, idx), f"{l.name} y")
    dx_np = U.to_np(dx)
    idx = rng.integers(0, dx_np.size, 1500)
    idx[:16] = np.arange(16)
    idx[16:32] = dx_np.size - 1 - np.arange(16)
    U.assert_bf16_close(dx_np.ravel()[idx], orc.conv2d_bwd_data_at(case.dy, case.w, case.x.shape, y_np, st, pd, idx), f"{l.name} dx")
    dw_np = U.to_np(dw)
    idx = rng.integers(0, dw_np.size, 400)
    idx[:8] = np.arange(8)
    idx[8:16] = dw_np.size - 1 - np.arange(8)
    U.assert_bf16_close(dw_np.ravel()[idx], orc.conv2d_bwd_filter_at(case.x, case.dy, case.w.shape, y_np, st, pd, idx), f"{l.name} dw")
    _, rdb = orc.relu_bias_grad(case.dy, y_np)
    U.assert_bf16_close(U.to_np(db), rdb, f"{l.name} db")


def _resnet_layers():
    from paper_2112_10065_amd import workloads
    return workloads.resnet50_convs()


def _inception_layers():
    from paper_2112_10065_amd import workloads
    return workloads.inception_convs()


@pytest.mark.parametrize("li", range(23))
def test_resnet50_layers_sampled(env, li):
    dp, U, orc = env
    l = _resnet_layers()[li]
    _sampled_layer_check(dp, U, orc, l, 2 if l.h > 56 else 3, "resnet50")


@pytest.mark.parametrize("li", range(18))
def test_inception_layers_sampled(env, li):
    dp, U, orc = env
    l = _inception_layers()[li]
    _sampled_layer_check(dp, U, orc, l, 1 if l.h > 100 else 4, "inception")


@pytest.mark.parametrize("li", range(24))
def test_wrn101_2_layers_sampled(env, li):
    """Wide ResNet-101-2 at 400x400 (the paper's second image model): every unique conv shape, sampled."""
    dp, U, orc = env
    from paper_2112_10065_amd import workloads
    l = workloads.wrn101_2_convs()[li]
    _sampled_layer_check(dp, U, orc, l, 1 if l.h > 100 else 2, "wrn101_2")
