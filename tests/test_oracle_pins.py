"""Pins of the fp64 CPU oracle against facts that do not depend on it.

The paper prints no numeric worked example of a layer, so the oracle is pinned
by mathematics: an explicit dense-operator construction written from the index
rule (independent loop structure), adjoint identities, finite differences,
closed forms and structural properties (superposition, batch independence --
the property data-parallel sharding rests on, paper section 2).
"""
import itertools

import numpy as np
import pytest

rng = np.random.default_rng(1234)

GEOMS = [  # (H, W, C, K, R, S, sh, sw, ph, pw)
    (5, 6, 2, 3, 1, 1, 1, 1, 0, 0),
    (5, 6, 2, 3, 3, 3, 1, 1, 1, 1),
    (6, 5, 3, 2, 3, 3, 2, 2, 1, 1),
    (6, 6, 2, 2, 3, 3, 2, 2, 0, 0),
    (4, 7, 2, 2, 1, 7, 1, 1, 0, 3),
    (7, 4, 2, 2, 7, 1, 1, 1, 3, 0),
    (6, 6, 1, 2, 7, 7, 2, 2, 3, 3),
    (5, 5, 2, 2, 1, 1, 2, 2, 0, 0),
    (6, 5, 2, 3, 3, 1, 1, 2, 1, 0),
    (5, 7, 3, 2, 1, 3, 2, 1, 0, 1),
]


def explicit_operator(n, h, w, c, k, r, s, sh, sw, ph, pw, wt):
    """Dense A with vec(y) = A vec(x), built by testing the tap relation for every
    (output element, input element) pair."""
    ho = (h + 2 * ph - r) // sh + 1
    wo = (w + 2 * pw - s) // sw + 1
    A = np.zeros((n * ho * wo * k, n * h * w * c))
    for (no, p, q, ko) in itertools.product(range(n), range(ho), range(wo), range(k)):
        row = ((no * ho + p) * wo + q) * k + ko
        for (ni, ih, iw, ci) in itertools.product(range(n), range(h), range(w), range(c)):
            if ni != no:
                continue
            rr = ih - (p * sh - ph)
            ss = iw - (q * sw - pw)
            if 0 <= rr < r and 0 <= ss < s:
                A[row, ((ni * h + ih) * w + iw) * c + ci] = wt[ko, rr, ss, ci]
    return A, ho, wo


@pytest.mark.parametrize("geom", GEOMS)
def test_explicit_operator_fwd_dgrad_wgrad(orc, geom):
    h, w, c, k, r, s, sh, sw, ph, pw = geom
    n = 2
    x = rng.standard_normal((n, h, w, c))
    wt = rng.standard_normal((k, r, s, c))
    A, ho, wo = explicit_operator(n, h, w, c, k, r, s, sh, sw, ph, pw, wt)
    assert (ho, wo) == orc.out_hw(h, w, r, s, sh, sw, ph, pw)
    y = orc.conv2d_fwd(x, wt, stride=(sh, sw), pad=(ph, pw))
    assert y.shape == (n, ho, wo, k)
    np.testing.assert_allclose(y.ravel(), A @ x.ravel(), rtol=0, atol=1e-12)
    g = rng.standard_normal(y.shape)
    dx = orc.conv2d_bwd_data(g, wt, x.shape, stride=(sh, sw), pad=(ph, pw))
    np.testing.assert_allclose(dx.ravel(), A.T @ g.ravel(), rtol=0, atol=1e-12)
    # operator in w: y is linear in w; column e of B is the response to the unit filter e
    B = np.zeros((y.size, wt.size))
    for e in range(wt.size):
        unit = np.zeros(wt.size)
        unit[e] = 1.0
        Ae, _, _ = explicit_operator(n, h, w, c, k, r, s, sh, sw, ph, pw, unit.reshape(wt.shape))
        B[:, e] = Ae @ x.ravel()
    dw = orc.conv2d_bwd_filter(x, g, wt.shape, stride=(sh, sw), pad=(ph, pw))
    np.testing.assert_allclose(dw.ravel(), B.T @ g.ravel(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("geom", [(16, 16, 16, 16, 3, 3, 1, 1, 1, 1), (13, 11, 5, 7, 3, 3, 2, 2, 1, 1),
                                  (17, 17, 6, 5, 1, 7, 1, 1, 0, 3), (12, 9, 4, 6, 7, 7, 2, 2, 3, 3)])
def test_adjoint_identities(orc, geom):
    h, w, c, k, r, s, sh, sw, ph, pw = geom
    x = rng.standard_normal((3, h, w, c))
    wt = rng.standard_normal((k, r, s, c))
    y = orc.conv2d_fwd(x, wt, stride=(sh, sw), pad=(ph, pw))
    g = rng.standard_normal(y.shape)
    lhs = np.vdot(y, g)
    dx = orc.conv2d_bwd_data(g, wt, x.shape, stride=(sh, sw), pad=(ph, pw))
    dw = orc.conv2d_bwd_filter(x, g, wt.shape, stride=(sh, sw), pad=(ph, pw))
    assert abs(np.vdot(x, dx) - lhs) <= 1e-12 * abs(lhs) + 1e-10
    assert abs(np.vdot(wt, dw) - lhs) <= 1e-12 * abs(lhs) + 1e-10


def test_linear_adjoints_and_matmul(orc):
    x = rng.standard_normal((5, 37))
    W = rng.standard_normal((11, 37))
    b = rng.standard_normal(11)
    g = rng.standard_normal((5, 11))
    y = orc.linear_fwd(x, W, b)
    np.testing.assert_allclose(y, x @ W.T + b, atol=1e-12)
    dx, dW, db = orc.linear_bwd(x, W, g)
    np.testing.assert_allclose(dx, g @ W, atol=1e-12)
    np.testing.assert_allclose(dW, g.T @ x, atol=1e-12)
    np.testing.assert_allclose(db, g.sum(0), atol=1e-12)
    # masked by a saved post-ReLU output
    yr = orc.linear_fwd(x, W, b, relu=True)
    np.testing.assert_allclose(yr, np.maximum(x @ W.T + b, 0), atol=1e-12)
    gm = g * (yr > 0)
    dx2, dW2, db2 = orc.linear_bwd(x, W, g, yr)
    np.testing.assert_allclose(dx2, gm @ W, atol=1e-12)
    np.testing.assert_allclose(dW2, gm.T @ x, atol=1e-12)
    np.testing.assert_allclose(db2, gm.sum(0), atol=1e-12)


def test_finite_differences_with_bias_and_relu(orc):
    n, h, w, c, k = 2, 7, 6, 3, 4
    st, pd = (2, 1), (1, 1)
    x = rng.standard_normal((n, h, w, c))
    wt = rng.standard_normal((k, 3, 3, c))
    b = rng.standard_normal(k)
    y = orc.conv2d_fwd(x, wt, b, relu=True, stride=st, pad=pd)
    pre = orc.conv2d_fwd(x, wt, b, relu=False, stride=st, pad=pd)
    assert np.abs(pre).min() > 1e-4  # stay off the ReLU kink
    g = rng.standard_normal(y.shape)

    def loss(x_, w_, b_):
        return np.vdot(orc.conv2d_fwd(x_, w_, b_, relu=True, stride=st, pad=pd), g)

    dx = orc.conv2d_bwd_data(g, wt, x.shape, y_saved=y, stride=st, pad=pd)
    dw, db = orc.conv2d_bwd_filter(x, g, wt.shape, y_saved=y, stride=st, pad=pd, want_db=True)
    eps = 1e-6
    for arr, grad, which in ((x, dx, 0), (wt, dw, 1), (b, db, 2)):
        flat = arr.ravel()
        for i in rng.choice(flat.size, size=min(12, flat.size), replace=False):
            old = flat[i]
            flat[i] = old + eps
            lp = loss(x, wt, b)
            flat[i] = old - eps
            lm = loss(x, wt, b)
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.ravel()[i]) <= 1e-7 * max(1.0, abs(fd)), (which, i)


def test_relu_in_backward_by_finite_differences(orc):
    """relu_in_backward (the backward of the ReLU that produced a layer's input, reading "derivative 0 at 0") against
    finite differences of L(u) = <conv(relu(u), w), g> in the pre-activation u: central differences where u != 0,
    and, at entries that are exactly 0, the one-sided difference from below (0: the reading taken) next to the one
    from above (the unmasked gradient).  A mask of x >= 0 instead of x > 0 fails at every u <= 0."""
    n, h, w, c, k = 2, 6, 5, 3, 4
    st, pd = (1, 2), (1, 1)
    u = rng.standard_normal((n, h, w, c))
    zeros = rng.choice(u.size, size=9, replace=False)
    u.ravel()[zeros] = 0.0
    wt = rng.standard_normal((k, 3, 3, c))
    x_in = np.maximum(u, 0.0)
    g = rng.standard_normal(orc.conv2d_fwd(x_in, wt, None, stride=st, pad=pd).shape)

    def loss(u_):
        return np.vdot(orc.conv2d_fwd(np.maximum(u_, 0.0), wt, None, stride=st, pad=pd), g)

    plain = orc.conv2d_bwd_data(g, wt, u.shape, stride=st, pad=pd)
    got = orc.relu_in_backward(plain, x_in)
    assert got.shape == u.shape and not got.ravel()[zeros].any() and not got[u < 0].any()
    np.testing.assert_array_equal(got[u > 0], plain[u > 0])
    assert (np.abs(plain[u <= 0]) > 1e-3).any()   # the mask matters: unmasked gradients there are not small
    eps = 1e-6
    flat = u.ravel()
    picks = np.concatenate([rng.choice(np.flatnonzero(flat > 1e-3), 10, replace=False),
                            rng.choice(np.flatnonzero(flat < -1e-3), 10, replace=False)])
    for i in picks:
        old = flat[i]
        flat[i] = old + eps
        lp = loss(u)
        flat[i] = old - eps
        lm = loss(u)
        flat[i] = old
        fd = (lp - lm) / (2 * eps)
        assert abs(fd - got.ravel()[i]) <= 1e-7 * max(1.0, abs(fd)), i
    l0 = loss(u)
    for i in zeros:
        flat[i] = -eps
        below = (l0 - loss(u)) / eps
        flat[i] = eps
        above = (loss(u) - l0) / eps
        flat[i] = 0.0
        assert below == 0.0 and got.ravel()[i] == 0.0
        assert abs(above - plain.ravel()[i]) <= 1e-6 * max(1.0, abs(above))


def test_delta_and_shifted_delta_kernels(orc):
    n, h, w, c = 2, 6, 7, 3
    x = rng.standard_normal((n, h, w, c))
    ident = np.zeros((c, 3, 3, c))
    for i in range(c):
        ident[i, 1, 1, i] = 1.0
    np.testing.assert_array_equal(orc.conv2d_fwd(x, ident, pad=(1, 1)), x)
    # tap (r=0, s=2): y[p,q] = x[p-1, q+1] (cross-correlation, zero fill)
    sh_k = np.zeros((c, 3, 3, c))
    for i in range(c):
        sh_k[i, 0, 2, i] = 1.0
    y = orc.conv2d_fwd(x, sh_k, pad=(1, 1))
    exp = np.zeros_like(x)
    exp[:, 1:, :-1, :] = x[:, :-1, 1:, :]
    np.testing.assert_array_equal(y, exp)


def test_all_ones_tap_counts(orc):
    c = 5
    x = np.ones((1, 6, 8, c))
    wt = np.ones((2, 3, 3, c))
    y = orc.conv2d_fwd(x, wt, pad=(1, 1))
    assert y[0, 0, 0, 0] == 4 * c and y[0, 0, 3, 1] == 6 * c and y[0, 2, 0, 0] == 6 * c
    assert y[0, 2, 3, 1] == 9 * c and y[0, 5, 7, 0] == 4 * c
    # wgrad of all-ones x and dy: centre tap sees every pixel, corner tap loses a row and a column
    dw = orc.conv2d_bwd_filter(x, np.ones_like(y), wt.shape, pad=(1, 1))
    assert dw[0, 1, 1, 0] == 6 * 8 and dw[1, 0, 0, 2] == 5 * 7 and dw[0, 1, 2, 1] == 6 * 7


def test_1x1_conv_is_matmul(orc):
    x = rng.standard_normal((2, 5, 4, 6))
    wt = rng.standard_normal((7, 1, 1, 6))
    y = orc.conv2d_fwd(x, wt)
    np.testing.assert_allclose(y.reshape(-1, 7), x.reshape(-1, 6) @ wt.reshape(7, 6).T, atol=1e-12)


def test_output_shapes_of_the_workloads(orc):
    assert orc.out_hw(224, 224, 7, 7, 2, 2, 3, 3) == (112, 112)
    assert orc.out_hw(299, 299, 3, 3, 2, 2, 0, 0) == (149, 149)
    assert orc.out_hw(149, 149, 3, 3, 1, 1, 0, 0) == (147, 147)
    assert orc.out_hw(73, 73, 3, 3, 1, 1, 0, 0) == (71, 71)
    assert orc.out_hw(35, 35, 3, 3, 2, 2, 0, 0) == (17, 17)
    assert orc.out_hw(17, 17, 1, 7, 1, 1, 0, 3) == (17, 17)


def test_superposition_and_batch_independence(orc):
    st, pd = (1, 1), (1, 1)
    x1 = rng.standard_normal((3, 6, 6, 4)); x2 = rng.standard_normal((3, 6, 6, 4))
    wt = rng.standard_normal((5, 3, 3, 4))
    f = lambda a: orc.conv2d_fwd(a, wt, stride=st, pad=pd)
    np.testing.assert_allclose(f(2 * x1 - 3 * x2), 2 * f(x1) - 3 * f(x2), atol=1e-12)
    # forward / dgrad per sample do not depend on the other samples
    y = f(x1)
    for i in range(3):
        np.testing.assert_array_equal(f(x1[i:i + 1])[0], y[i])
    g = rng.standard_normal(y.shape)
    dx = orc.conv2d_bwd_data(g, wt, x1.shape, stride=st, pad=pd)
    np.testing.assert_array_equal(
        orc.conv2d_bwd_data(g[1:2], wt, (1, 6, 6, 4), stride=st, pad=pd)[0], dx[1])
    # wgrad is additive over samples (what gradient synchronisation sums)
    dw = orc.conv2d_bwd_filter(x1, g, wt.shape, stride=st, pad=pd)
    parts = sum(orc.conv2d_bwd_filter(x1[i:i + 1], g[i:i + 1], wt.shape, stride=st, pad=pd)
                for i in range(3))
    np.testing.assert_allclose(dw, parts, atol=1e-12)


def test_relu_bias_grad(orc):
    dy = rng.standard_normal((2, 3, 4, 5))
    y = np.maximum(rng.standard_normal(dy.shape), 0)
    y.ravel()[3] = 0.0
    g, db = orc.relu_bias_grad(dy, y)
    np.testing.assert_array_equal(g, np.where(y > 0, dy, 0.0))
    np.testing.assert_allclose(db, np.where(y > 0, dy, 0.0).reshape(-1, 5).sum(0), atol=1e-13)


def test_spot_evaluation_matches_full(orc):
    st, pd = (2, 1), (1, 3)
    x = rng.standard_normal((2, 9, 10, 4)).astype(np.float32)
    wt = rng.standard_normal((6, 3, 7, 4)).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    y = orc.conv2d_fwd(x, wt, b, relu=True, stride=st, pad=pd)
    g = rng.standard_normal(y.shape).astype(np.float32)
    idx = rng.choice(y.size, 50, replace=False)
    np.testing.assert_allclose(orc.conv2d_fwd_at(x, wt, b, True, st, pd, idx), y.ravel()[idx], atol=1e-13)
    ys = y.astype(np.float32)
    dx = orc.conv2d_bwd_data(g, wt, x.shape, y_saved=ys, stride=st, pad=pd)
    idx = rng.choice(dx.size, 50, replace=False)
    np.testing.assert_allclose(orc.conv2d_bwd_data_at(g, wt, x.shape, ys, st, pd, idx), dx.ravel()[idx], atol=1e-13)
    dw = orc.conv2d_bwd_filter(x, g, wt.shape, y_saved=ys, stride=st, pad=pd)
    idx = rng.choice(dw.size, 50, replace=False)
    np.testing.assert_allclose(orc.conv2d_bwd_filter_at(x, g, wt.shape, ys, st, pd, idx), dw.ravel()[idx], atol=1e-12)
    # dense
    xl = rng.standard_normal((4, 33)).astype(np.float32); W = rng.standard_normal((9, 33)).astype(np.float32)
    bl = rng.standard_normal(9).astype(np.float32); gl = rng.standard_normal((4, 9)).astype(np.float32)
    yl = orc.linear_fwd(xl, W, bl, relu=True)
    dxl, dWl, _ = orc.linear_bwd(xl, W, gl, yl.astype(np.float32))
    np.testing.assert_allclose(orc.linear_fwd_at(xl, W, bl, True, np.arange(36)), yl.ravel(), atol=1e-13)
    np.testing.assert_allclose(orc.linear_dx_at(W, gl, yl.astype(np.float32), np.arange(132)), dxl.ravel(), atol=1e-13)
    np.testing.assert_allclose(orc.linear_dw_at(xl, gl, yl.astype(np.float32), np.arange(297)), dWl.ravel(), atol=1e-13)


def test_vgg16_parameter_count():
    from paper_2112_10065_amd import workloads
    assert workloads.vgg16_param_count() == 138357544
    assert len(workloads.vgg16_convs()) + len(workloads.vgg16_linears()) + 5 == 21  # paper Table 1: 21 layers
