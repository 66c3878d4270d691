"""ctypes binding of libdp_mi355x.so: same names as the C ABI (include/dp.h), argument
marshalling only.  PyTorch supplies device memory and streams; every computation runs in
the library's HIP kernels.  Importing this module fails loudly if the library is missing.
"""
import ctypes as C
import os

import torch  # noqa: F401  (first: the library must bind to the HIP runtime that PyTorch loads)

from . import build as _build

DP_OK, DP_ERR_NULL, DP_ERR_BAD_DESC, DP_ERR_UNSUPPORTED, DP_ERR_WORKSPACE, DP_ERR_HIP = range(6)
DP_F32, DP_BF16 = 0, 1
DP_BIAS, DP_RELU, DP_DETERMINISTIC, DP_DX_F32, DP_RELU_IN = 1, 2, 4, 8, 16
DP_PASS_FWD, DP_PASS_DGRAD, DP_PASS_WGRAD = 0, 1, 2

EXPORTS = ["dp_conv2d_workspace_bytes", "dp_linear_workspace_bytes", "dp_conv2d_fwd", "dp_conv2d_bwd_data", "dp_conv2d_bwd_data_relu",
           "dp_conv2d_bwd_filter", "dp_conv2d_bwd_filter_noalloc", "dp_linear_fwd_bwd", "dp_relu_bias_grad_workspace_bytes", "dp_relu_bias_grad",
           "dp_profile_layer", "dp_trace_begin", "dp_trace_end", "dp_conv2d_kernel_info", "dp_set_override", "dp_set_autotune", "dp_plan_chain",
           "dp_plan_cost_tables", "dp_plan_graph", "dp_maxpool2x2_fwd", "dp_maxpool2x2_bwd", "dp_softmax_xent", "dp_sgd_update",
           "dp_last_error", "dp_version"]


class dp_conv_desc(C.Structure):
    _fields_ = [(f, C.c_int32) for f in ("n", "h", "w", "c_in", "c_out", "r", "s", "stride_h", "stride_w",
                                         "pad_h", "pad_w", "io_dtype")] + [("flags", C.c_uint32)]


class dp_linear_desc(C.Structure):
    _fields_ = [("n", C.c_int32), ("in_features", C.c_int32), ("out_features", C.c_int32),
                ("io_dtype", C.c_int32), ("flags", C.c_uint32)]


class dp_profile_row(C.Structure):
    _fields_ = [("batch", C.c_int32), ("fwd_us", C.c_float), ("dgrad_us", C.c_float), ("wgrad_us", C.c_float),
                ("flops_per_pass", C.c_double), ("min_bytes_fwd", C.c_double), ("min_bytes_dgrad", C.c_double),
                ("min_bytes_wgrad", C.c_double)]


class dp_trace_row(C.Structure):
    _fields_ = [("kernel", C.c_char * 96), ("pass_", C.c_int32), ("splits", C.c_int32), ("main_us", C.c_float),
                ("total_us", C.c_float)]


class dp_plan_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_gpu_counts", C.c_int32), ("gpu_counts", C.POINTER(C.c_int32)),
                ("comp", C.POINTER(C.c_double)), ("comm", C.POINTER(C.c_double)), ("sync", C.POINTER(C.c_double)),
                ("amp_limit", C.c_double)]


class dp_plan_branch(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("comp", C.POINTER(C.c_double)), ("comm", C.POINTER(C.c_double)),
                ("sync", C.POINTER(C.c_double)), ("join", C.POINTER(C.c_double)), ("move", C.POINTER(C.c_double))]


class dp_plan_graph_desc(C.Structure):
    _fields_ = [("chain", dp_plan_desc), ("n_branches", C.POINTER(C.c_int32)), ("branches", C.POINTER(dp_plan_branch))]


class DpError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"dp status {status}: {msg}")
        self.status = status


def _load():
    path = _build.LIB
    if not os.path.exists(path):
        path = _build.build(force=True)   # nothing built yet: compile once
    lib = C.CDLL(path)
    vp, sz, i32, i64, u32 = C.c_void_p, C.c_size_t, C.c_int32, C.c_int64, C.c_uint32
    P = C.POINTER
    lib.dp_conv2d_workspace_bytes.restype = sz
    lib.dp_conv2d_workspace_bytes.argtypes = [P(dp_conv_desc), C.c_int]
    lib.dp_linear_workspace_bytes.restype = sz
    lib.dp_linear_workspace_bytes.argtypes = [P(dp_linear_desc)]
    lib.dp_conv2d_fwd.argtypes = [P(dp_conv_desc), vp, vp, vp, vp, vp, sz, vp]
    lib.dp_conv2d_bwd_data.argtypes = [P(dp_conv_desc), vp, vp, vp, vp, vp, sz, vp]
    lib.dp_conv2d_bwd_data_relu.argtypes = [P(dp_conv_desc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dp_conv2d_bwd_data_relu.restype = C.c_int
    lib.dp_conv2d_bwd_filter.argtypes = [P(dp_conv_desc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dp_conv2d_bwd_filter_noalloc.argtypes = [P(dp_conv_desc), vp, vp, vp, vp, vp, vp]
    lib.dp_linear_fwd_bwd.argtypes = [P(dp_linear_desc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dp_relu_bias_grad_workspace_bytes.restype = sz
    lib.dp_relu_bias_grad_workspace_bytes.argtypes = [i64, i32]
    lib.dp_relu_bias_grad.argtypes = [i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.dp_profile_layer.argtypes = [P(dp_conv_desc), P(dp_linear_desc), P(i32), i32, i32, i32, P(dp_profile_row), vp]
    lib.dp_trace_begin.argtypes = []
    lib.dp_trace_end.argtypes = [P(dp_trace_row), i32, P(i32)]
    lib.dp_set_override.argtypes = [C.c_int, C.c_int, C.c_int]
    lib.dp_set_autotune.argtypes = [C.c_int]
    lib.dp_conv2d_kernel_info.argtypes = [P(dp_conv_desc), C.c_int, C.c_char_p, sz, P(i32)]
    lib.dp_conv2d_kernel_info.restype = C.c_int
    pd = P(C.c_double)
    lib.dp_plan_chain.argtypes = [P(dp_plan_desc), P(i32), pd, pd, pd]
    lib.dp_plan_cost_tables.argtypes = [i32, i32, P(i32), pd, pd, C.c_double, C.c_double, pd, pd]
    lib.dp_plan_graph.argtypes = [P(dp_plan_graph_desc), P(i32), P(i32), P(C.c_uint8), P(i32), pd, pd, pd]
    lib.dp_maxpool2x2_fwd.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp]
    lib.dp_maxpool2x2_bwd.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.dp_softmax_xent.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp]
    lib.dp_sgd_update.argtypes = [i64, C.c_float, C.c_float, vp, vp, vp, vp, vp]
    for name in ("dp_conv2d_fwd", "dp_conv2d_bwd_data", "dp_conv2d_bwd_filter", "dp_conv2d_bwd_filter_noalloc", "dp_linear_fwd_bwd",
                 "dp_relu_bias_grad", "dp_profile_layer", "dp_trace_begin", "dp_trace_end", "dp_set_override", "dp_set_autotune", "dp_plan_chain",
                 "dp_plan_cost_tables", "dp_plan_graph", "dp_maxpool2x2_fwd", "dp_maxpool2x2_bwd", "dp_softmax_xent", "dp_sgd_update"):
        getattr(lib, name).restype = C.c_int
    lib.dp_last_error.restype = C.c_char_p
    lib.dp_version.restype = C.c_char_p
    return lib


lib = _load()


def _check(st):
    if st != DP_OK:
        raise DpError(st, lib.dp_last_error().decode())


def _ptr(t):
    """Device (or raw integer) address of a torch tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def conv_desc(n, h, w, c_in, c_out, r, s, stride=(1, 1), pad=(0, 0), io_dtype=DP_BF16, flags=0):
    return dp_conv_desc(n, h, w, c_in, c_out, r, s, stride[0], stride[1], pad[0], pad[1], io_dtype, flags)


def linear_desc(n, in_features, out_features, io_dtype=DP_BF16, flags=0):
    return dp_linear_desc(n, in_features, out_features, io_dtype, flags)


def dp_version():
    return lib.dp_version().decode()


def dp_last_error():
    return lib.dp_last_error().decode()


def dp_set_override(pass_, tile_variant=-1, splits=0):
    _check(lib.dp_set_override(pass_, tile_variant, splits))


def dp_set_autotune(enabled):
    """0 / False: analytic choice; 1 / True: measured warm; 2: measured with the caches flushed before each timed launch."""
    _check(lib.dp_set_autotune(int(enabled)))


def dp_maxpool2x2_fwd(n, h, w, c, io_dtype, x, y, stream=None):
    _check(lib.dp_maxpool2x2_fwd(n, h, w, c, io_dtype, _ptr(x), _ptr(y), _stream(stream)))


def dp_maxpool2x2_bwd(n, h, w, c, io_dtype, x, dy, dx, stream=None):
    _check(lib.dp_maxpool2x2_bwd(n, h, w, c, io_dtype, _ptr(x), _ptr(dy), _ptr(dx), _stream(stream)))


def dp_softmax_xent(n, classes, io_dtype, z, labels, loss, dz=None, stream=None):
    _check(lib.dp_softmax_xent(n, classes, io_dtype, _ptr(z), _ptr(labels), _ptr(loss), _ptr(dz), _stream(stream)))


def dp_sgd_update(count, lr, momentum, grad, mom, w32, w_bf16=None, stream=None):
    _check(lib.dp_sgd_update(count, lr, momentum, _ptr(grad), _ptr(mom), _ptr(w32), _ptr(w_bf16), _stream(stream)))


def _doubles(rows, n):
    """Flat C array of n doubles from a (nested) Python sequence, or None."""
    if rows is None:
        return None
    flat = []

    def walk(v):
        if isinstance(v, (list, tuple)):
            for e in v:
                walk(e)
        else:
            flat.append(float(v))
    walk(rows)
    if len(flat) != n:
        raise ValueError(f"expected {n} values, got {len(flat)}")
    return (C.c_double * n)(*flat)


def dp_plan_chain(gpu_counts, comp, comm=None, sync=None, amp_limit=float("inf")):
    """Host-only.  comp [L][G], comm [L][G][G] or None, sync [L][G] or None (nested sequences).
    Returns {"gpus": [L], "time": float, "S": [L+1][G], "T": [L+1][G]}."""
    L, G = len(comp), len(gpu_counts)
    gc = (C.c_int32 * G)(*gpu_counts)
    d = dp_plan_desc(L, G, gc, _doubles(comp, L * G), _doubles(comm, L * G * G), _doubles(sync, L * G), float(amp_limit))
    out = (C.c_int32 * L)()
    t = C.c_double(0.0)
    S = (C.c_double * ((L + 1) * G))()
    T = (C.c_double * ((L + 1) * G))()
    _check(lib.dp_plan_chain(C.byref(d), out, C.byref(t), S, T))
    rows = lambda a: [[a[i * G + j] for j in range(G)] for i in range(L + 1)]
    return {"gpus": list(out), "time": t.value, "S": rows(S), "T": rows(T)}


def dp_plan_cost_tables(gpu_counts, act_bytes, param_bytes, bandwidth, delay):
    """Host-only.  Returns (comm [L][G][G], sync [L][G]) as nested lists."""
    L, G = len(param_bytes), len(gpu_counts)
    gc = (C.c_int32 * G)(*gpu_counts)
    comm = (C.c_double * (L * G * G))()
    sync = (C.c_double * (L * G))()
    _check(lib.dp_plan_cost_tables(L, G, gc, _doubles(act_bytes, L), _doubles(param_bytes, L), float(bandwidth), float(delay), comm, sync))
    return ([[[comm[(i * G + b) * G + a] for a in range(G)] for b in range(G)] for i in range(L)],
            [[sync[i * G + a] for a in range(G)] for i in range(L)])


def dp_plan_graph(gpu_counts, layers, amp_limit=float("inf")):
    """Host-only.  layers[i] = {"comp": [G], "sync": [G] or None, "comm": [G][G] or None, "branches": [...]}; a layer
    with branches is the joining layer of a block that leaves layer i-1; a branch = {"comp": [Lb][G], "comm":
    [Lb][G][G] or None, "sync": [Lb][G] or None, "join": [G][G] or None, "move": [G][G] or None}.
    Returns {"gpus", "time", "S", "T", "blocks": per layer None or {"critical", "parallel": [..], "gpus": [[..], ..]}}."""
    L, G = len(layers), len(gpu_counts)
    gc = (C.c_int32 * G)(*gpu_counts)
    keep = []                     # the C arrays must outlive the call

    def arr(rows, n):
        a = _doubles(rows, n)
        keep.append(a)
        return C.cast(a, C.POINTER(C.c_double)) if a is not None else None

    no_sync = all(l.get("sync") is None for l in layers)
    sync = None if no_sync else [l.get("sync") or [0.0] * G for l in layers]
    comm = [l.get("comm") if l.get("comm") is not None else [[0.0] * G] * G for l in layers]
    flat = [br for l in layers for br in (l.get("branches") or [])]
    brs = (dp_plan_branch * max(1, len(flat)))()
    for k, br in enumerate(flat):
        Lb = len(br["comp"])
        brs[k] = dp_plan_branch(Lb, arr(br["comp"], Lb * G) if Lb else None, arr(br.get("comm"), Lb * G * G) if Lb else None,
                                arr(br.get("sync"), Lb * G) if Lb else None, arr(br.get("join"), G * G), arr(br.get("move"), G * G))
    nbr = (C.c_int32 * L)(*[len(l.get("branches") or []) for l in layers])
    d = dp_plan_graph_desc(dp_plan_desc(L, G, gc, arr([l["comp"] for l in layers], L * G), arr(comm, L * G * G), arr(sync, L * G),
                                        float(amp_limit)), nbr, brs)
    out = (C.c_int32 * L)()
    n_bl = sum(len(br["comp"]) for br in flat)
    bg = (C.c_int32 * max(1, n_bl))()
    par = (C.c_uint8 * max(1, len(flat)))()
    crit = (C.c_int32 * L)()
    t = C.c_double(0.0)
    S = (C.c_double * ((L + 1) * G))()
    T = (C.c_double * ((L + 1) * G))()
    _check(lib.dp_plan_graph(C.byref(d), out, bg, par, crit, C.byref(t), S, T))
    rows = lambda a: [[a[i * G + j] for j in range(G)] for i in range(L + 1)]
    blocks, kb, kl = [], 0, 0
    for l in layers:
        bl = l.get("branches") or []
        if not bl:
            blocks.append(None)
            continue
        plans = []
        for br in bl:
            plans.append([bg[kl + j] for j in range(len(br["comp"]))])
            kl += len(br["comp"])
        blocks.append({"critical": crit[len(blocks)], "parallel": [bool(par[kb + j]) for j in range(len(bl))], "gpus": plans})
        kb += len(bl)
    return {"gpus": list(out), "time": t.value, "S": rows(S), "T": rows(T), "blocks": blocks}


def dp_conv2d_kernel_info(desc, pass_):
    buf = C.create_string_buffer(128)
    splits = C.c_int32(0)
    _check(lib.dp_conv2d_kernel_info(C.byref(desc), pass_, buf, 128, C.byref(splits)))
    return buf.value.decode(), int(splits.value)


def dp_conv2d_workspace_bytes(desc, pass_):
    return int(lib.dp_conv2d_workspace_bytes(C.byref(desc), pass_))


def dp_linear_workspace_bytes(desc):
    return int(lib.dp_linear_workspace_bytes(C.byref(desc)))


def dp_relu_bias_grad_workspace_bytes(rows, k):
    return int(lib.dp_relu_bias_grad_workspace_bytes(rows, k))


def dp_conv2d_fwd(desc, x, w, bias, y, ws=None, stream=None):
    p, b = _ws(ws)
    _check(lib.dp_conv2d_fwd(C.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), p, b, _stream(stream)))


def dp_conv2d_bwd_data(desc, dy, y_saved, w, dx, ws=None, stream=None):
    p, b = _ws(ws)
    _check(lib.dp_conv2d_bwd_data(C.byref(desc), _ptr(dy), _ptr(y_saved), _ptr(w), _ptr(dx), p, b, _stream(stream)))


def dp_conv2d_bwd_data_relu(desc, dy, y_saved, w, x_saved, dx, ws=None, stream=None):
    p, b = _ws(ws)
    _check(lib.dp_conv2d_bwd_data_relu(C.byref(desc), _ptr(dy), _ptr(y_saved), _ptr(w), _ptr(x_saved), _ptr(dx), p, b,
                                       _stream(stream)))


def dp_conv2d_bwd_filter(desc, x, dy, y_saved, dw, dbias=None, ws=None, stream=None):
    p, b = _ws(ws)
    _check(lib.dp_conv2d_bwd_filter(C.byref(desc), _ptr(x), _ptr(dy), _ptr(y_saved), _ptr(dw), _ptr(dbias), p, b,
                                    _stream(stream)))


DP_NOALLOC_SCRATCH_BYTES = 32 << 20


def dp_conv2d_bwd_filter_noalloc(desc, x, dy, y_saved, dw, dbias=None, stream=None):
    _check(lib.dp_conv2d_bwd_filter_noalloc(C.byref(desc), _ptr(x), _ptr(dy), _ptr(y_saved), _ptr(dw), _ptr(dbias),
                                            _stream(stream)))


def dp_linear_fwd_bwd(desc, x=None, W=None, bias=None, dy=None, y_saved=None, y=None, dx=None, dW=None, dbias=None,
                      ws=None, stream=None):
    p, b = _ws(ws)
    _check(lib.dp_linear_fwd_bwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(bias), _ptr(dy), _ptr(y_saved), _ptr(y),
                                 _ptr(dx), _ptr(dW), _ptr(dbias), p, b, _stream(stream)))


def dp_relu_bias_grad(rows, k, io_dtype, dy, y_saved, g_out=None, dbias=None, ws=None, stream=None):
    p, b = _ws(ws)
    _check(lib.dp_relu_bias_grad(rows, k, io_dtype, _ptr(dy), _ptr(y_saved), _ptr(g_out), _ptr(dbias), p, b,
                                 _stream(stream)))


def dp_profile_layer(conv=None, linear=None, batches=(1,), warmup=3, iters=10, stream=None):
    n = len(batches)
    arr = (C.c_int32 * n)(*batches)
    rows = (dp_profile_row * n)()
    _check(lib.dp_profile_layer(C.byref(conv) if conv is not None else None,
                                C.byref(linear) if linear is not None else None, arr, n, warmup, iters, rows,
                                _stream(stream)))
    return [dict((f, getattr(r, f)) for f, _ in dp_profile_row._fields_) for r in rows]


def dp_trace_begin():
    _check(lib.dp_trace_begin())


def dp_trace_end(max_rows=8192):
    """Rows of the trace started by dp_trace_begin, in call order: dicts with kernel, pass, splits, main_us, total_us."""
    rows = (dp_trace_row * max_rows)()
    n = C.c_int32(0)
    _check(lib.dp_trace_end(rows, max_rows, C.byref(n)))
    return [{"kernel": rows[i].kernel.decode(), "pass": rows[i].pass_, "splits": rows[i].splits,
             "main_us": rows[i].main_us, "total_us": rows[i].total_us} for i in range(n.value)]


def bind(fn_name, *args):
    """Pre-marshalled call: `fn_name` is an entry point of this module (e.g. "dp_conv2d_fwd"), `args` its
    arguments in the order of the wrapper above.  Returns a zero-argument callable that issues exactly
    that C call (descriptor, pointers, sizes and stream are resolved once), for launch-bound loops."""
    cap = {}
    g = globals()
    saved = g["lib"]

    class _Recorder:
        def __getattr__(self, name):
            def rec(*cargs):
                cap["fn"], cap["args"] = getattr(saved, name), cargs
                return DP_OK
            return rec

    g["lib"] = _Recorder()
    try:
        g[fn_name](*args)
    finally:
        g["lib"] = saved
    fn, cargs = cap["fn"], cap["args"]
    keep = args   # keeps descriptors / tensors alive as long as the callable

    def call(_fn=fn, _a=cargs, _keep=keep):
        st = _fn(*_a)
        if st != DP_OK:
            raise DpError(st, lib.dp_last_error().decode())
    return call
