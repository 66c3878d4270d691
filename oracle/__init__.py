"""fp64 CPU oracle (numpy front end of dp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never calls into this package and
this package never imports the GPU library.

Every function is the plain definition of the layer operation (see the header
of dp_oracle.c; paper section 4.1 "Computation cost" names the operations whose
forward+backward time the planner consumes, Table 1 the layer kinds).

Pins (tests/test_oracle_pins.py): explicit-operator brute force, adjoint
identities, finite differences, closed forms (delta / shifted-delta kernels,
all-ones tap counts, 1x1 conv == matmul), superposition, batch independence;
relu_in_backward by finite differences through relu(u) including entries that
are exactly zero.  No function here is "parity unpinned"; timings have no paper
value to pin to.

Layouts: x [N,H,W,C], w [K,R,S,C], y/dy [N,Ho,Wo,K], dense, C order.
"""
import ctypes as C
import numpy as np

from .build import build as _build

_lib = None


class _Conv(C.Structure):
    _fields_ = [(f, C.c_int) for f in ("n", "h", "w", "c", "k", "r", "s", "sh", "sw", "ph", "pw")]


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build())
        _lib.orc_max_threads.restype = C.c_int
    return _lib


def max_threads() -> int:
    return int(lib().orc_max_threads())


def out_hw(h, w, r, s, sh, sw, ph, pw):
    return (h + 2 * ph - r) // sh + 1, (w + 2 * pw - s) // sw + 1


def _desc(xshape, wshape, stride, pad):
    n, h, w, c = xshape
    k, r, s, c2 = wshape
    assert c == c2, "channel mismatch"
    return _Conv(n, h, w, c, k, r, s, stride[0], stride[1], pad[0], pad[1])


def _d(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _f(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def conv2d_fwd(x, w, bias=None, relu=False, stride=(1, 1), pad=(0, 0)):
    x, w, bias = _d(x), _d(w), _d(bias)
    d = _desc(x.shape, w.shape, stride, pad)
    ho, wo = out_hw(d.h, d.w, d.r, d.s, d.sh, d.sw, d.ph, d.pw)
    y = np.empty((d.n, ho, wo, d.k), dtype=np.float64)
    lib().orc_conv2d_fwd(C.byref(d), _p(x), _p(w), _p(bias), C.c_int(int(relu)), _p(y))
    return y


def conv2d_bwd_data(dy, w, xshape, y_saved=None, stride=(1, 1), pad=(0, 0)):
    dy, w, y_saved = _d(dy), _d(w), _d(y_saved)
    d = _desc(xshape, w.shape, stride, pad)
    dx = np.empty(tuple(xshape), dtype=np.float64)
    lib().orc_conv2d_bwd_data(C.byref(d), _p(dy), _p(y_saved), _p(w), _p(dx))
    return dx


def relu_in_backward(dx, x_in):
    """Backward of the ReLU that produced a layer's input, applied to that layer's data gradient:
    dx * [x_in > 0] (derivative 0 at 0, as for the output-side mask).  Pinned by
    test_relu_in_backward_by_finite_differences."""
    return _d(dx) * (_d(x_in) > 0)


def conv2d_bwd_filter(x, dy, wshape, y_saved=None, stride=(1, 1), pad=(0, 0), want_db=False):
    x, dy, y_saved = _d(x), _d(dy), _d(y_saved)
    d = _desc(x.shape, wshape, stride, pad)
    dw = np.empty(tuple(wshape), dtype=np.float64)
    db = np.empty((d.k,), dtype=np.float64) if want_db else None
    lib().orc_conv2d_bwd_filter(C.byref(d), _p(x), _p(dy), _p(y_saved), _p(dw), _p(db))
    return (dw, db) if want_db else dw


def relu_bias_grad(dy, y_saved):
    dy, y_saved = _d(dy), _d(y_saved)
    k = dy.shape[-1]
    rows = dy.size // k
    g = np.empty_like(dy)
    db = np.empty((k,), dtype=np.float64)
    lib().orc_relu_bias_grad(C.c_longlong(rows), C.c_int(k), _p(dy), _p(y_saved), _p(g), _p(db))
    return g, db


def linear_fwd(x, W, bias=None, relu=False):
    x, W, bias = _d(x), _d(W), _d(bias)
    n, i = x.shape
    o = W.shape[0]
    assert W.shape[1] == i
    y = np.empty((n, o), dtype=np.float64)
    lib().orc_linear_fwd(n, i, o, _p(x), _p(W), _p(bias), int(relu), _p(y))
    return y


def linear_bwd(x, W, dy, y_saved=None):
    x, W, dy, y_saved = _d(x), _d(W), _d(dy), _d(y_saved)
    n, i = x.shape
    o = W.shape[0]
    dx = np.empty((n, i)); dW = np.empty((o, i)); db = np.empty((o,))
    lib().orc_linear_bwd(n, i, o, _p(x), _p(W), _p(dy), _p(y_saved), _p(dx), _p(dW), _p(db))
    return dx, dW, db


# ---- spot evaluation at flat output indices (fp32 inputs widened to fp64) ----
def _idx(idx):
    return np.ascontiguousarray(idx, dtype=np.int64)


def conv2d_fwd_at(x, w, bias, relu, stride, pad, idx):
    x, w, bias, idx = _f(x), _f(w), _f(bias), _idx(idx)
    d = _desc(x.shape, w.shape, stride, pad)
    out = np.empty(idx.shape, dtype=np.float64)
    lib().orc_conv2d_fwd_at(C.byref(d), _p(x), _p(w), _p(bias), int(relu), _p(idx),
                            C.c_longlong(idx.size), _p(out))
    return out


def conv2d_bwd_data_at(dy, w, xshape, y_saved, stride, pad, idx):
    dy, w, y_saved, idx = _f(dy), _f(w), _f(y_saved), _idx(idx)
    d = _desc(xshape, w.shape, stride, pad)
    out = np.empty(idx.shape, dtype=np.float64)
    lib().orc_conv2d_bwd_data_at(C.byref(d), _p(dy), _p(y_saved), _p(w), _p(idx),
                                 C.c_longlong(idx.size), _p(out))
    return out


def conv2d_bwd_filter_at(x, dy, wshape, y_saved, stride, pad, idx):
    x, dy, y_saved, idx = _f(x), _f(dy), _f(y_saved), _idx(idx)
    d = _desc(x.shape, wshape, stride, pad)
    out = np.empty(idx.shape, dtype=np.float64)
    lib().orc_conv2d_bwd_filter_at(C.byref(d), _p(x), _p(dy), _p(y_saved), _p(idx),
                                   C.c_longlong(idx.size), _p(out))
    return out


def linear_fwd_at(x, W, bias, relu, idx):
    x, W, bias, idx = _f(x), _f(W), _f(bias), _idx(idx)
    n, i = x.shape
    out = np.empty(idx.shape, dtype=np.float64)
    lib().orc_linear_fwd_at(n, i, W.shape[0], _p(x), _p(W), _p(bias), int(relu), _p(idx),
                            C.c_longlong(idx.size), _p(out))
    return out


def linear_dx_at(W, dy, y_saved, idx):
    W, dy, y_saved, idx = _f(W), _f(dy), _f(y_saved), _idx(idx)
    n, o = dy.shape
    out = np.empty(idx.shape, dtype=np.float64)
    lib().orc_linear_dx_at(n, W.shape[1], o, _p(W), _p(dy), _p(y_saved), _p(idx),
                           C.c_longlong(idx.size), _p(out))
    return out


def linear_dw_at(x, dy, y_saved, idx):
    x, dy, y_saved, idx = _f(x), _f(dy), _f(y_saved), _idx(idx)
    n, i = x.shape
    out = np.empty(idx.shape, dtype=np.float64)
    lib().orc_linear_dw_at(n, i, dy.shape[1], _p(x), _p(dy), _p(y_saved), _p(idx),
                           C.c_longlong(idx.size), _p(out))
    return out
