"""The allocation-free backward-filter entry point against dp_conv2d_bwd_filter (which takes a caller workspace):
same kernels, built-in scratch.  Two calls in a row share the scratch, the second on a smaller layer, so stale
contents of the first must not leak into the second; each is compared with the workspace form to the bf16 bar
(and must in fact be identical: the kernels are deterministic and both calls use the analytic kernel choice)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_noalloc_backward_filter_twice_then_smaller():
    from paper_2112_10065_amd import binding as dp
    import gpu_util as U
    dp.dp_set_autotune(False)
    # (n, h, w, c, k): split partials + bias-gradient sums in scratch; then a smaller layer; then the first-layer kernels
    cases = [("na_big", 4, 28, 28, 128, 256, True), ("na_small", 2, 14, 14, 64, 96, True), ("na_small_nomask", 1, 9, 10, 24, 40, False),
             ("na_rgb", 2, 20, 22, 3, 64, True)]
    for tag, n, h, w, c, k, masked in cases:
        case = U.ConvCase(tag, n, h, w, c, k, 3, 3, (1, 1), (1, 1), bf16=True, bias=True, relu=True, dx_f32=c < 8)
        need = dp.dp_conv2d_workspace_bytes(case.desc, dp.DP_PASS_WGRAD)
        assert 0 < need <= dp.DP_NOALLOC_SCRATCH_BYTES, need
        y = case.run_fwd()
        ys = y if masked else None
        want_dw, want_db = case.run_wgrad(ys)
        dw = torch.full((k, 3, 3, c), 7.0, dtype=torch.float32, device=U.DEV)
        db = torch.full((k,), 7.0, dtype=torch.float32, device=U.DEV)
        dp.dp_conv2d_bwd_filter_noalloc(case.desc, case.xd, case.dyd, ys, dw, db)
        torch.cuda.synchronize()
        U.assert_bf16_close(U.to_np(dw), U.to_np(want_dw), f"{tag} dw")
        U.assert_bf16_close(U.to_np(db), U.to_np(want_db), f"{tag} db")
        assert torch.equal(dw, want_dw) and torch.equal(db, want_db), tag
        # without the bias gradient
        dw.fill_(7.0)
        dp.dp_conv2d_bwd_filter_noalloc(case.desc, case.xd, case.dyd, ys, dw, None)
        torch.cuda.synchronize()
        assert torch.equal(dw, want_dw), tag + " (no db)"


def test_noalloc_rejects_what_does_not_fit():
    from paper_2112_10065_amd import binding as dp
    import gpu_util as U
    dp.dp_set_autotune(False)
    d = dp.conv_desc(32, 224, 224, 64, 64, 3, 3, (1, 1), (1, 1), dp.DP_BF16, dp.DP_BIAS | dp.DP_RELU)
    assert dp.dp_conv2d_workspace_bytes(d, dp.DP_PASS_WGRAD) > dp.DP_NOALLOC_SCRATCH_BYTES
    a = torch.empty(64, dtype=torch.float32, device=U.DEV)   # never touched: the call fails before any launch
    with pytest.raises(dp.DpError) as ei:
        dp.dp_conv2d_bwd_filter_noalloc(d, a, a, None, a, a)
    assert ei.value.status == dp.DP_ERR_WORKSPACE
