"""Oracle of the layers that turn the per-layer compute into a whole VGG-16 training step:
2x2 max pooling (forward / backward), softmax cross-entropy, SGD with momentum.

TEST INFRASTRUCTURE ONLY (see the package docstring).  numpy, fp64, each function the plain definition.
The paper lists these layers (Table 1 counts VGG-16's five pooling layers among its 21) but gives no
arithmetic for them; the readings are the usual ones and are listed in the design notes:
  * pooling windows are 2x2 at stride 2 without padding; a trailing odd row / column is dropped;
  * the gradient of a window goes to its FIRST maximum in row-major order ((0,0), (0,1), (1,0), (1,1)),
    which decides the many ties that post-ReLU zeros produce;
  * the loss is the mean over the batch of -log softmax(z)[label];
  * the update is SGD with momentum, m <- mu*m + g, w <- w - lr*m (no dampening, no Nesterov term,
    no weight decay).

Pins (tests/test_glue_pins.py): loop-written brute force, the adjoint identity of pooling, gradient mass
conservation, tie routing, finite differences, log(C) at uniform logits, shift invariance, the closed form
of k momentum steps under a constant gradient.
Layouts: x [N,H,W,C]; z [N,classes]; labels [N] integers.
"""
import numpy as np


def _windows(x):
    """The four window positions in scan order, each [N, H//2, W//2, C]."""
    n, h, w, c = x.shape
    ho, wo = h // 2, w // 2
    return np.stack([x[:, 0:2 * ho:2, 0:2 * wo:2], x[:, 0:2 * ho:2, 1:2 * wo:2],
                     x[:, 1:2 * ho:2, 0:2 * wo:2], x[:, 1:2 * ho:2, 1:2 * wo:2]])


def maxpool2x2_fwd(x):
    x = np.asarray(x, dtype=np.float64)
    return _windows(x).max(axis=0)


def maxpool2x2_bwd(x, dy):
    x, dy = np.asarray(x, dtype=np.float64), np.asarray(dy, dtype=np.float64)
    n, h, w, c = x.shape
    ho, wo = h // 2, w // 2
    first = _windows(x).argmax(axis=0)          # numpy returns the first maximum
    dx = np.zeros_like(x)
    for pos, (dh, dw_) in enumerate(((0, 0), (0, 1), (1, 0), (1, 1))):
        dx[:, dh:2 * ho:2, dw_:2 * wo:2] = np.where(first == pos, dy, 0.0)
    return dx


def softmax_xent(z, labels):
    """(loss, dz): loss = mean_n(logsumexp(z_n) - z_n[label_n]); dz = (softmax(z) - onehot) / N."""
    z = np.asarray(z, dtype=np.float64)
    n = z.shape[0]
    zs = z - z.max(axis=1, keepdims=True)
    lse = np.log(np.exp(zs).sum(axis=1))
    rows = np.arange(n)
    loss = float((lse - zs[rows, labels]).mean())
    dz = np.exp(zs - lse[:, None])
    dz[rows, labels] -= 1.0
    return loss, dz / n


def sgd_momentum(w, m, g, lr, mu):
    """(w', m'): m' = mu*m + g; w' = w - lr*m'."""
    w, m, g = (np.asarray(a, dtype=np.float64) for a in (w, m, g))
    m2 = mu * m + g
    return w - lr * m2, m2
