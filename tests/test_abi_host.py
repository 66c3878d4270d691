"""Host-side checks of the C ABI: the library loads, exports every declared symbol, and every
argument error is reported before any launch (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dp():
    from paper_2112_10065_amd import binding
    return binding


def test_exports_every_declared_symbol(dp):
    hdr = open(os.path.join(ROOT, "include", "dp.h")).read()
    declared = set(re.findall(r"\b(dp_[a-z0-9_]+)\s*\(", hdr))
    assert {"dp_conv2d_fwd", "dp_conv2d_bwd_data", "dp_conv2d_bwd_filter", "dp_linear_fwd_bwd",
            "dp_profile_layer"} <= declared
    for name in declared:
        assert hasattr(dp.lib, name), name
    assert declared == set(dp.EXPORTS)
    assert "gfx950" in dp.dp_version()


def test_struct_sizes_match_header(dp):
    assert C.sizeof(dp.dp_conv_desc) == 13 * 4
    assert C.sizeof(dp.dp_linear_desc) == 5 * 4
    assert C.sizeof(dp.dp_profile_row) == 48


A = 0x1000  # fake, 16-byte aligned, never dereferenced: validation fails first


def test_conv_argument_errors(dp):
    lib = dp.lib
    good = dp.conv_desc(2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1), dp.DP_BF16, dp.DP_BIAS)
    assert lib.dp_conv2d_fwd(None, A, A, A, A, None, 0, None) == dp.DP_ERR_NULL
    assert lib.dp_conv2d_fwd(C.byref(good), None, A, A, A, None, 0, None) == dp.DP_ERR_NULL
    assert b"x is NULL" in lib.dp_last_error()
    assert lib.dp_conv2d_fwd(C.byref(good), A, A, None, A, None, 0, None) == dp.DP_ERR_NULL  # DP_BIAS without bias
    assert lib.dp_conv2d_fwd(C.byref(good), A + 2, A, A, A, None, 0, None) == dp.DP_ERR_BAD_DESC  # misaligned
    bad = dp.conv_desc(0, 16, 16, 16, 16, 3, 3)
    assert lib.dp_conv2d_fwd(C.byref(bad), A, A, A, A, None, 0, None) == dp.DP_ERR_BAD_DESC
    bad = dp.conv_desc(1, 2, 2, 4, 4, 3, 3)  # filter larger than the unpadded image
    assert lib.dp_conv2d_bwd_data(C.byref(bad), A, None, A, A, None, 0, None) == dp.DP_ERR_BAD_DESC
    bad = dp.conv_desc(1, 8, 8, 4, 4, 3, 3, io_dtype=7)
    assert lib.dp_conv2d_bwd_filter(C.byref(bad), A, A, None, A, None, None, 0, None) == dp.DP_ERR_UNSUPPORTED
    bad = dp.conv_desc(1, 8, 8, 4, 4, 3, 3, flags=1 << 20)
    assert lib.dp_conv2d_fwd(C.byref(bad), A, A, A, A, None, 0, None) == dp.DP_ERR_UNSUPPORTED
    bad = dp.conv_desc(1, 8, 8, 4, 4, 3, 3, io_dtype=dp.DP_F32, flags=dp.DP_DX_F32)
    assert lib.dp_conv2d_fwd(C.byref(bad), A, A, A, A, None, 0, None) == dp.DP_ERR_UNSUPPORTED
    huge = dp.conv_desc(1 << 12, 1 << 10, 1 << 10, 8, 8, 1, 1)
    assert lib.dp_conv2d_fwd(C.byref(huge), A, A, A, A, None, 0, None) == dp.DP_ERR_BAD_DESC
    assert dp.dp_conv2d_workspace_bytes(bad, 0) == 0
    assert dp.dp_conv2d_workspace_bytes(good, 9) == 0


def test_workspace_errors(dp):
    lib = dp.lib
    # backward-filter always splits its long reduction here -> needs scratch
    d = dp.conv_desc(2, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1), dp.DP_BF16, 0)
    need = dp.dp_conv2d_workspace_bytes(d, dp.DP_PASS_WGRAD)
    assert need > 0
    assert lib.dp_conv2d_bwd_filter(C.byref(d), A, A, None, A, A, None, 0, None) == dp.DP_ERR_WORKSPACE
    assert lib.dp_conv2d_bwd_filter(C.byref(d), A, A, None, A, A, A, 16, None) == dp.DP_ERR_WORKSPACE
    ld = dp.linear_desc(4, 4096, 4096, dp.DP_BF16, 0)
    assert dp.dp_linear_workspace_bytes(ld) > 0
    assert lib.dp_linear_fwd_bwd(C.byref(ld), A, A, None, None, None, A, None, None, None, None, 0, None) == dp.DP_ERR_WORKSPACE
    assert lib.dp_relu_bias_grad(100, 64, dp.DP_BF16, A, A, None, A, None, 0, None) == dp.DP_ERR_WORKSPACE
    assert dp.dp_relu_bias_grad_workspace_bytes(100, 64) > 0


def test_noalloc_backward_filter_argument_errors(dp):
    """The allocation-free form validates like dp_conv2d_bwd_filter and rejects layers beyond its built-in scratch
    before any HIP call."""
    lib = dp.lib
    d = dp.conv_desc(2, 28, 28, 64, 64, 3, 3, (1, 1), (1, 1), dp.DP_BF16, 0)
    assert lib.dp_conv2d_bwd_filter_noalloc(None, A, A, None, A, A, None) == dp.DP_ERR_NULL
    assert lib.dp_conv2d_bwd_filter_noalloc(C.byref(d), None, A, None, A, A, None) == dp.DP_ERR_NULL
    assert lib.dp_conv2d_bwd_filter_noalloc(C.byref(d), A, A, None, None, A, None) == dp.DP_ERR_NULL
    assert lib.dp_conv2d_bwd_filter_noalloc(C.byref(d), A, A + 4, None, A, A, None) == dp.DP_ERR_BAD_DESC
    big = dp.conv_desc(32, 224, 224, 64, 64, 3, 3, (1, 1), (1, 1), dp.DP_BF16, 0)
    assert dp.dp_conv2d_workspace_bytes(big, dp.DP_PASS_WGRAD) > dp.DP_NOALLOC_SCRATCH_BYTES
    assert lib.dp_conv2d_bwd_filter_noalloc(C.byref(big), A, A, None, A, A, None) == dp.DP_ERR_WORKSPACE
    assert b"built-in scratch" in lib.dp_last_error()
    hdr = open(os.path.join(ROOT, "include", "dp.h")).read()
    assert "#define DP_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)" in hdr and dp.DP_NOALLOC_SCRATCH_BYTES == 32 << 20


def test_linear_and_pointwise_argument_errors(dp):
    lib = dp.lib
    ld = dp.linear_desc(4, 64, 32, dp.DP_BF16, dp.DP_BIAS)
    N = None
    assert lib.dp_linear_fwd_bwd(C.byref(ld), A, A, A, N, N, N, N, N, N, N, 0, N) == dp.DP_ERR_NULL  # nothing requested
    assert lib.dp_linear_fwd_bwd(C.byref(ld), N, A, A, N, N, A, N, N, N, N, 0, N) == dp.DP_ERR_NULL  # y needs x
    assert lib.dp_linear_fwd_bwd(C.byref(ld), A, A, A, N, N, N, A, N, N, N, 0, N) == dp.DP_ERR_NULL  # dx needs dy
    assert lib.dp_linear_fwd_bwd(C.byref(dp.linear_desc(0, 64, 32)), A, A, A, N, N, A, N, N, N, N, 0, N) == dp.DP_ERR_BAD_DESC
    assert lib.dp_relu_bias_grad(0, 64, dp.DP_BF16, A, A, A, N, N, 0, N) == dp.DP_ERR_BAD_DESC
    assert lib.dp_relu_bias_grad(10, 64, dp.DP_BF16, A, A, N, N, N, 0, N) == dp.DP_ERR_NULL
    assert lib.dp_relu_bias_grad(10, 64, 5, A, A, A, N, N, 0, N) == dp.DP_ERR_UNSUPPORTED


def test_profile_and_override_argument_errors(dp):
    lib = dp.lib
    cd = dp.conv_desc(1, 8, 8, 8, 8, 3, 3, (1, 1), (1, 1))
    ld = dp.linear_desc(1, 8, 8)
    rows = (dp.dp_profile_row * 1)()
    b = (C.c_int32 * 1)(1)
    assert lib.dp_profile_layer(None, None, b, 1, 1, 1, rows, None) == dp.DP_ERR_NULL
    assert lib.dp_profile_layer(C.byref(cd), C.byref(ld), b, 1, 1, 1, rows, None) == dp.DP_ERR_NULL
    assert lib.dp_profile_layer(C.byref(cd), None, None, 1, 1, 1, rows, None) == dp.DP_ERR_NULL
    assert lib.dp_profile_layer(C.byref(cd), None, b, 1, 1, 0, rows, None) == dp.DP_ERR_BAD_DESC
    bneg = (C.c_int32 * 1)(-3)
    assert lib.dp_profile_layer(C.byref(cd), None, bneg, 1, 1, 1, rows, None) == dp.DP_ERR_BAD_DESC
    assert lib.dp_set_override(5, 0, 0) == dp.DP_ERR_UNSUPPORTED
    assert lib.dp_set_override(0, -1, 0) == dp.DP_OK
    assert lib.dp_set_autotune(1) == dp.DP_OK and lib.dp_set_autotune(0) == dp.DP_OK
    # the trace hook: end without begin, begin twice, missing output arguments; an empty trace has no rows
    n = C.c_int32(7)
    trows = (dp.dp_trace_row * 2)()
    assert lib.dp_trace_end(trows, 2, C.byref(n)) == dp.DP_ERR_UNSUPPORTED
    assert lib.dp_trace_begin() == dp.DP_OK and lib.dp_trace_begin() == dp.DP_ERR_UNSUPPORTED
    assert lib.dp_trace_end(trows, 2, None) == dp.DP_ERR_NULL
    assert lib.dp_trace_begin() == dp.DP_OK
    assert lib.dp_trace_end(trows, 2, C.byref(n)) == dp.DP_OK and n.value == 0
    assert C.sizeof(dp.dp_trace_row) == 96 + 16


def test_no_gpu_fails_loudly(dp):
    """On a host without a GPU a valid call must return DP_ERR_HIP, never succeed or fall back."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    d = dp.conv_desc(1, 8, 8, 8, 8, 3, 3, (1, 1), (1, 1), dp.DP_BF16, 0)
    assert dp.lib.dp_conv2d_fwd(C.byref(d), A, A, None, A, None, 0, None) == dp.DP_ERR_HIP
    assert dp.lib.dp_last_error() != b""


def test_glue_argument_errors(dp):
    lib = dp.lib
    assert lib.dp_maxpool2x2_fwd(1, 4, 4, 8, dp.DP_BF16, None, A, None) == dp.DP_ERR_NULL
    assert lib.dp_maxpool2x2_fwd(1, 4, 4, 8, dp.DP_BF16, A, None, None) == dp.DP_ERR_NULL
    assert lib.dp_maxpool2x2_fwd(1, 4, 4, 8, 5, A, A, None) == dp.DP_ERR_UNSUPPORTED
    assert lib.dp_maxpool2x2_fwd(0, 4, 4, 8, dp.DP_BF16, A, A, None) == dp.DP_ERR_BAD_DESC
    assert lib.dp_maxpool2x2_fwd(1, 4, 4, 8, dp.DP_BF16, A + 2, A, None) == dp.DP_ERR_BAD_DESC
    assert lib.dp_maxpool2x2_bwd(1, 4, 4, 8, dp.DP_BF16, A, None, A, None) == dp.DP_ERR_NULL
    assert lib.dp_maxpool2x2_bwd(1, 4, 4, 8, dp.DP_BF16, A, A, None, None) == dp.DP_ERR_NULL
    assert lib.dp_softmax_xent(4, 10, dp.DP_F32, A, None, A, None, None) == dp.DP_ERR_NULL
    assert lib.dp_softmax_xent(4, 0, dp.DP_F32, A, A, A, None, None) == dp.DP_ERR_BAD_DESC
    assert lib.dp_softmax_xent(4, 10, 9, A, A, A, None, None) == dp.DP_ERR_UNSUPPORTED
    assert lib.dp_sgd_update(16, 0.1, 0.9, None, A, A, None, None) == dp.DP_ERR_NULL
    assert lib.dp_sgd_update(-1, 0.1, 0.9, A, A, A, None, None) == dp.DP_ERR_BAD_DESC
    assert lib.dp_sgd_update(16, 0.1, 0.9, A, A + 4, A, None, None) == dp.DP_ERR_BAD_DESC
    assert lib.dp_sgd_update(0, 0.1, 0.9, A, A, A, None, None) == dp.DP_OK   # nothing to do, nothing launched


def test_fused_input_relu_argument_errors(dp):
    lib = dp.lib
    d = dp.conv_desc(2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1), dp.DP_BF16, dp.DP_RELU_IN)
    assert lib.dp_conv2d_bwd_data(C.byref(d), A, None, A, A, None, 0, None) == dp.DP_ERR_NULL        # no saved input to mask with
    assert b"x_saved" in lib.dp_last_error()
    assert lib.dp_conv2d_bwd_data_relu(C.byref(d), A, None, A, None, A, None, 0, None) == dp.DP_ERR_NULL
    assert lib.dp_conv2d_bwd_data_relu(C.byref(d), A, None, A, A + 8, A, None, 0, None) == dp.DP_ERR_BAD_DESC  # misaligned
    ld = dp.linear_desc(4, 64, 32, dp.DP_BF16, dp.DP_RELU_IN)
    assert lib.dp_linear_fwd_bwd(C.byref(ld), None, A, None, A, None, None, A, None, None, None, 0, None) == dp.DP_ERR_NULL  # dx needs x
    # the flag changes which kernels a call may use, so the workspace query takes it into account without failing
    assert dp.dp_conv2d_workspace_bytes(d, 1) >= 0


def test_pixel_strip_plan_rules(dp):
    """Host logic of the kernel choice (no GPU call): the pixel-strip kernels are planned for the 3x3 / stride 1 / pad 1
    layers with 128 or more reduction channels on grids of 160 or more blocks, never for fp32 input gradients, other
    filters, strides or paddings, and a reduction split takes an even number of 64-channel blocks."""
    def info(n, h, c, k, pass_, r=3, stride=(1, 1), pad=(1, 1), extra=0):
        d = dp.conv_desc(n, h, h, c, k, r, r, stride, pad, dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU | extra)
        return dp.dp_conv2d_kernel_info(d, pass_)
    assert info(32, 56, 256, 256, 0) == ("k_conv_strip<false, 224, 256>", 1)        # conv3_2: 448 tiles of 224 pixels fill two rounds of
    assert info(32, 56, 256, 256, 1) == ("k_conv_strip<true, 224, 256>", 1)         # 256 blocks better than 392 tiles of 256
    assert info(32, 28, 512, 512, 0) == ("k_conv_strip<false, 224, 256>", 1)        # conv4_2: 224 blocks instead of 196
    assert info(32, 14, 512, 512, 0) == ("k_conv_strip<false, 128, 256>", 2)        # conv5_x: 98 tiles, two splits of four blocks
    assert "k_conv_strip" not in info(32, 56, 256, 256, 1, extra=dp.DP_DX_F32)[0]   # bf16 staged epilogue only
    assert "k_conv_strip" not in info(4, 14, 512, 512, 0)[0]                         # too few blocks
    assert "k_conv_strip" not in info(32, 56, 64, 256, 0)[0]                         # 64 reduction channels
    assert "k_conv_strip" not in info(32, 56, 256, 256, 0, r=1, pad=(0, 0))[0]
    assert "k_conv_strip" not in info(32, 56, 256, 256, 0, stride=(2, 2))[0]
    assert "k_conv_strip" not in info(32, 56, 256, 256, 2)[0]                        # not a filter-gradient kernel
    for code, splits, want in ((230, 2, 2), (230, 3, 2), (230, 4, 2), (231, 4, 2), (232, 8, 2)):   # 256 channels: four blocks
        dp.dp_set_override(0, code, splits)
        try:
            assert info(8, 28, 256, 256, 0)[1] == want
        finally:
            dp.dp_set_override(0, -1, 0)
    dp.dp_set_override(1, 230, 4)
    try:
        assert info(8, 14, 512, 512, 1) == ("k_conv_strip<true, 256, 256>", 4)      # 512 channels: eight blocks, four splits of two
    finally:
        dp.dp_set_override(1, -1, 0)

