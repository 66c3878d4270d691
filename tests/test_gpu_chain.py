"""One small network run end to end the way bench.py's step issues the calls, against the oracle chain.

conv a (3 -> 64) - ReLU - conv b (64 -> 64) - ReLU - pool - conv c (64 -> 128) - ReLU - conv d (128 -> 128) - ReLU
- pool - dense 1 (ReLU) - dense 2 - softmax cross-entropy, on a 3 x 18 x 14 x 3 input.

GPU side (the fused formulation of the benchmark's step): forward calls with bias + ReLU in the epilogue; backward
from the loss, each layer's backward-data applying the backward of the ReLU IN FRONT of it (DP_RELU_IN with the
layer's saved input), so that every incoming gradient is already masked and all backward calls pass
y_saved = NULL; pooled gradients go through dp_maxpool2x2_bwd after that masking.

Oracle side (the textbook formulation, wired independently): every layer masks its incoming gradient with its OWN
saved output (the y_saved arguments of the oracle's backward functions), pooling backward comes before the
mask of the ReLU under it.  Saved activations are the GPU forward's stored tensors on both sides (the ReLU masks
and pooling routes then never differ), while the gradient chain itself runs in fp64 on the oracle side and through
bf16 tensors on the GPU side.  Forward is checked layer by layer on the GPU's own inputs.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_chained_step_matches_oracle_chain(orc):
    from paper_2112_10065_amd import binding as dp, synth
    from oracle import glue
    import gpu_util as U

    n, h, w, classes = 3, 18, 14, 10
    convs = [("a", 3, 64), ("b", 64, 64), ("c", 64, 128), ("d", 128, 128)]
    pool_after = {"b", "d"}
    bf = torch.bfloat16

    def dev_bf16(a):
        bits = synth.f32_to_bf16_bits(a)
        return synth.bf16_bits_to_f32(bits), U.bf16_dev(bits)

    # parameters and input
    P = {}
    for name, c, k in convs:
        x_, wt, b = synth.conv_tensors(f"chain/{name}", 1, 1, 1, c, k, 3, 3)
        P[name] = (*dev_bf16(wt), b, torch.from_numpy(b).to(U.DEV))
    x0, x0d = dev_bf16(synth.normal("chain/input", (n, h, w, 3)))
    hp, wp = h // 4, w // 4
    feat = hp * wp * 128
    dense = [("fc1", feat, 96, True), ("fc2", 96, classes, False)]
    for name, i, o, _ in dense:
        _, W, b = synth.linear_tensors(f"chain/{name}", 1, i, o)
        P[name] = (*dev_bf16(W), b, torch.from_numpy(b).to(U.DEV))
    labels = np.array([3, 0, 7], dtype=np.int32)
    labels_d = torch.from_numpy(labels).to(U.DEV)

    def conv_desc(hh, ww, c, k, first):
        flags = dp.DP_BIAS | dp.DP_RELU | (0 if first else dp.DP_RELU_IN)
        return dp.conv_desc(n, hh, ww, c, k, 3, 3, (1, 1), (1, 1), dp.DP_BF16, flags)

    # ---- forward on the GPU, every activation kept (as a training step keeps them) ----
    acts = {}          # name -> (input tensor, output tensor, desc, spatial size)
    cur, hh, ww = x0d, h, w
    pools = {}         # name of the conv before the pool -> (pool input, pool output, h, w, c)
    for name, c, k in convs:
        d = conv_desc(hh, ww, c, k, name == "a")
        y = torch.empty((n, hh, ww, k), dtype=bf, device=U.DEV)
        ws = U.workspace(max(dp.dp_conv2d_workspace_bytes(d, p) for p in range(3)))
        dp.dp_conv2d_fwd(d, cur, P[name][1], P[name][3], y, ws)
        acts[name] = (cur, y, d, (hh, ww, c, k))
        cur = y
        if name in pool_after:
            p = torch.empty((n, hh // 2, ww // 2, k), dtype=bf, device=U.DEV)
            dp.dp_maxpool2x2_fwd(n, hh, ww, k, dp.DP_BF16, cur, p)
            pools[name] = (cur, p, hh, ww, k)
            cur, hh, ww = p, hh // 2, ww // 2
    cur = cur.reshape(n, feat)
    for name, i, o, relu in dense:
        d = dp.linear_desc(n, i, o, dp.DP_BF16, dp.DP_BIAS | (dp.DP_RELU if relu else 0) | dp.DP_RELU_IN)
        y = torch.empty((n, o), dtype=bf, device=U.DEV)
        ws = U.workspace(dp.dp_linear_workspace_bytes(d))
        dp.dp_linear_fwd_bwd(d, x=cur, W=P[name][1], bias=P[name][3], y=y, ws=ws)
        acts[name] = (cur, y, d, (i, o))
        cur = y
    z = cur
    loss = torch.zeros(4, dtype=torch.float32, device=U.DEV)
    dz = torch.empty_like(z)
    dp.dp_softmax_xent(n, classes, dp.DP_BF16, z, labels_d, loss, dz)

    # ---- backward on the GPU, exactly the calls of the benchmark's step ----
    grads = {}
    g = dz
    for name, i, o, relu in reversed(dense):
        xin, y, d, _ = acts[name]
        ws = U.workspace(dp.dp_linear_workspace_bytes(d))
        dW = torch.empty((o, i), dtype=torch.float32, device=U.DEV)
        db = torch.empty((o,), dtype=torch.float32, device=U.DEV)
        dx = torch.empty((n, i), dtype=bf, device=U.DEV)
        dp.dp_linear_fwd_bwd(d, x=xin, dy=g, dW=dW, dbias=db, ws=ws)
        dp.dp_linear_fwd_bwd(d, x=xin, W=P[name][1], dy=g, dx=dx, ws=ws)   # dx *= [x > 0]: the ReLU (or pooled ReLU) in front
        grads[name] = (dW, db, dx)
        g = dx
    g = g.reshape(n, hp, wp, 128)
    for name, c, k in reversed(convs):
        xin, y, d, (hh, ww, _, _) = acts[name]
        if name in pool_after:
            pin, pout, ph_, pw_, pc = pools[name]
            gp = torch.empty((n, ph_, pw_, pc), dtype=bf, device=U.DEV)
            dp.dp_maxpool2x2_bwd(n, ph_, pw_, pc, dp.DP_BF16, pin, g, gp)
            g = gp
        ws = U.workspace(max(dp.dp_conv2d_workspace_bytes(d, p) for p in range(3)))
        dw = torch.empty((k, 3, 3, c), dtype=torch.float32, device=U.DEV)
        db = torch.empty((k,), dtype=torch.float32, device=U.DEV)
        dp.dp_conv2d_bwd_filter(d, xin, g, None, dw, db, ws)
        dx = None
        if name != "a":
            dx = torch.empty((n, hh, ww, c), dtype=bf, device=U.DEV)
            dp.dp_conv2d_bwd_data_relu(d, g, None, P[name][1], xin, dx, ws)
        grads[name] = (dw, db, dx)
        g = dx
    torch.cuda.synchronize()

    # ---- forward parity, layer by layer on the GPU's own inputs ----
    for name, c, k in convs:
        xin, y, _, _ = acts[name]
        ref = orc.conv2d_fwd(U.to_np(xin), P[name][0], P[name][2], relu=True, pad=(1, 1))
        U.assert_bf16_close(U.to_np(y), ref, f"forward conv {name}")
        if name in pool_after:
            pin, pout, *_ = pools[name]
            np.testing.assert_array_equal(U.to_np(pout), glue.maxpool2x2_fwd(U.to_np(pin)).astype(np.float32))
    for name, i, o, relu in dense:
        xin, y, _, _ = acts[name]
        U.assert_bf16_close(U.to_np(y), orc.linear_fwd(U.to_np(xin), P[name][0], P[name][2], relu=relu), f"forward {name}")
    z_np = U.to_np(z)
    ref_loss, ref_dz = glue.softmax_xent(z_np, labels)
    assert abs(float(loss[0].item()) - ref_loss) <= 1e-5 * max(1.0, abs(ref_loss))

    # ---- backward: the oracle's own chain in fp64, textbook wiring ----
    def close(got, ref, what):
        rel, mx = U.errs(got, ref)
        assert rel <= U.BF16_REL and mx <= U.BF16_ABS, f"{what}: rel_l2={rel:.3e} max_abs={mx:.3e}"
        assert np.linalg.norm(ref) > 0, what

    close(U.to_np(dz), ref_dz, "dz")
    g = ref_dz                                   # gradient w.r.t. the output of the layer being processed
    for li, (name, i, o, relu) in enumerate(reversed(dense)):
        xin, y, _, _ = acts[name]
        dx, dW, db = orc.linear_bwd(U.to_np(xin), P[name][0], g, U.to_np(y) if relu else None)   # masks by its own output
        close(U.to_np(grads[name][0]), dW, f"{name} dW")
        close(U.to_np(grads[name][1]), db, f"{name} db")
        close(U.to_np(grads[name][2]), dx * (U.to_np(xin) > 0), f"{name} dx")
        g = dx                                   # unmasked here; the GPU's dx already carries the next mask
    g = g.reshape(n, hp, wp, 128)
    for name, c, k in reversed(convs):
        xin, y, _, (hh, ww, _, _) = acts[name]
        if name in pool_after:
            pin, pout, *_ = pools[name]
            g = glue.maxpool2x2_bwd(U.to_np(pin), g)
        y_np, x_np = U.to_np(y), U.to_np(xin)
        dw, db = orc.conv2d_bwd_filter(x_np, g, P[name][0].shape, y_saved=y_np, pad=(1, 1), want_db=True)
        close(U.to_np(grads[name][0]), dw, f"conv {name} dw")
        close(U.to_np(grads[name][1]), db, f"conv {name} db")
        if name != "a":
            g = orc.conv2d_bwd_data(g, P[name][0], x_np.shape, y_saved=y_np, pad=(1, 1))
            # the GPU's dx is this times the mask of the ReLU below, which the oracle applies in its next step
            close(U.to_np(grads[name][2]), g * (x_np > 0), f"conv {name} dx")
