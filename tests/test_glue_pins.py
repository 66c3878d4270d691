"""Pins of oracle/glue.py (pooling, loss, update) against loops, identities and closed forms."""
import math

import numpy as np
import pytest

from oracle import glue

rng = np.random.default_rng(4321)


def pool_loops(x, dy=None):
    """Definition written as scalar loops: first strict maximum in row-major window order."""
    n, h, w, c = x.shape
    ho, wo = h // 2, w // 2
    y = np.zeros((n, ho, wo, c))
    dx = np.zeros_like(x)
    for ni in range(n):
        for p in range(ho):
            for q in range(wo):
                for ci in range(c):
                    best, bh, bw = x[ni, 2 * p, 2 * q, ci], 0, 0
                    for dh in range(2):
                        for dw in range(2):
                            v = x[ni, 2 * p + dh, 2 * q + dw, ci]
                            if v > best:
                                best, bh, bw = v, dh, dw
                    y[ni, p, q, ci] = best
                    if dy is not None:
                        dx[ni, 2 * p + bh, 2 * q + bw, ci] = dy[ni, p, q, ci]
    return y, dx


@pytest.mark.parametrize("shape", [(2, 4, 6, 3), (1, 5, 7, 2), (3, 2, 2, 1), (1, 1, 4, 2)])
def test_pool_matches_loops_with_ties(shape):
    x = np.maximum(rng.integers(-3, 3, shape).astype(np.float64), 0.0)   # many equal values, as after ReLU
    dy = rng.normal(size=(shape[0], shape[1] // 2, shape[2] // 2, shape[3]))
    y, dx = pool_loops(x, dy)
    assert np.array_equal(glue.maxpool2x2_fwd(x), y)
    assert np.array_equal(glue.maxpool2x2_bwd(x, dy), dx)


def test_pool_adjoint_mass_and_ties():
    x = rng.normal(size=(2, 6, 8, 3))
    dy = rng.normal(size=(2, 3, 4, 3))
    dx = glue.maxpool2x2_bwd(x, dy)
    # y = P(x) x with a selection matrix P, backward = P^T dy
    assert math.isclose(float((dx * x).sum()), float((dy * glue.maxpool2x2_fwd(x)).sum()), rel_tol=1e-12)
    assert math.isclose(float(dx.sum()), float(dy.sum()), rel_tol=1e-12)
    assert int((dx != 0).sum()) == dy.size                      # one receiver per window and channel
    # an all-equal window sends its gradient to position (0, 0) only
    dx = glue.maxpool2x2_bwd(np.zeros((1, 2, 2, 1)), np.full((1, 1, 1, 1), 5.0))
    assert dx.ravel().tolist() == [5.0, 0.0, 0.0, 0.0]
    # odd sizes: the last row and column belong to no window
    dx = glue.maxpool2x2_bwd(rng.normal(size=(1, 5, 3, 2)), rng.normal(size=(1, 2, 1, 2)))
    assert not dx[:, 4].any() and not dx[:, :, 2].any()


def test_pool_finite_difference():
    x = rng.permutation(48).astype(np.float64).reshape(1, 4, 6, 2)   # distinct values: differentiable
    dy = rng.normal(size=(1, 2, 3, 2))
    dx = glue.maxpool2x2_bwd(x, dy)
    for idx in [(0, 0, 0, 0), (0, 1, 3, 1), (0, 3, 5, 0), (0, 2, 2, 1)]:
        e = np.zeros_like(x); e[idx] = 1e-3
        fd = float((dy * (glue.maxpool2x2_fwd(x + e) - glue.maxpool2x2_fwd(x - e))).sum()) / 2e-3
        assert math.isclose(fd, dx[idx], abs_tol=1e-9)


def test_softmax_xent_closed_forms():
    n, c = 4, 10
    labels = np.array([0, 3, 9, 3])
    loss, dz = glue.softmax_xent(np.full((n, c), 2.5), labels)
    assert math.isclose(loss, math.log(c), rel_tol=1e-14)
    want = np.full((n, c), 1.0 / c); want[np.arange(n), labels] -= 1.0
    assert np.allclose(dz, want / n, rtol=1e-14)
    z = rng.normal(size=(n, c)) * 3
    loss, dz = glue.softmax_xent(z, labels)
    assert np.allclose(dz.sum(axis=1), 0.0, atol=1e-15)
    loss2, dz2 = glue.softmax_xent(z + 1000.0, labels)            # shift invariance, no overflow
    assert math.isclose(loss, loss2, rel_tol=1e-12) and np.allclose(dz, dz2, atol=1e-12)
    # two classes: loss = log(1 + exp(-(z_label - z_other)))
    l2, _ = glue.softmax_xent(np.array([[1.0, 3.0]]), np.array([1]))
    assert math.isclose(l2, math.log1p(math.exp(-2.0)), rel_tol=1e-14)
    # a dominant correct logit: loss -> 0
    big = np.zeros((1, 5)); big[0, 2] = 60.0
    assert glue.softmax_xent(big, np.array([2]))[0] < 1e-20 + 5 * math.exp(-60.0)


def test_softmax_xent_finite_difference():
    n, c = 3, 7
    z = rng.normal(size=(n, c))
    labels = np.array([6, 0, 2])
    _, dz = glue.softmax_xent(z, labels)
    for idx in [(0, 0), (0, 6), (1, 3), (2, 2)]:
        e = np.zeros_like(z); e[idx] = 1e-5
        fd = (glue.softmax_xent(z + e, labels)[0] - glue.softmax_xent(z - e, labels)[0]) / 2e-5
        assert math.isclose(fd, dz[idx], rel_tol=1e-6, abs_tol=1e-10)


def test_sgd_momentum_closed_form():
    w0, g = rng.normal(size=17), rng.normal(size=17)
    lr, mu, k = 0.05, 0.9, 6
    w, m = w0.copy(), np.zeros(17)
    for _ in range(k):
        w, m = glue.sgd_momentum(w, m, g, lr, mu)
    # constant gradient: m_j = g (1 - mu^j) / (1 - mu); w_k = w_0 - lr * sum_j m_j
    mk = g * (1 - mu ** k) / (1 - mu)
    sum_m = g * (k - mu * (1 - mu ** k) / (1 - mu)) / (1 - mu)
    assert np.allclose(m, mk, rtol=1e-12) and np.allclose(w, w0 - lr * sum_m, rtol=1e-12)
    w1, m1 = glue.sgd_momentum(w0, rng.normal(size=17), g, lr, 0.0)   # no momentum: plain gradient step
    assert np.allclose(w1, w0 - lr * g, rtol=1e-15) and np.array_equal(m1, g)
