"""ctypes front end of the C oracle (TEST INFRASTRUCTURE, not product code).

Every function takes NumPy arrays holding the exact fp32 / bf16 input values (any float dtype, any
strides, broadcast views allowed), widens them to float64 without changing layout, calls the plain C
definition in ``chn_oracle.c`` and returns float64 results.  Nothing here touches the GPU library.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_MAX_NDIM = 8


class _View(C.Structure):
    _fields_ = [("data", C.c_void_p), ("ndim", C.c_int32),
                ("shape", C.c_int64 * _MAX_NDIM), ("strides", C.c_int64 * _MAX_NDIM)]


_OPS = ["copy", "add", "sub", "mul", "mad", "mad_relu", "relu", "relu_bwd", "gelu", "gelu_bwd",
        "scale", "axpy", "add_relu", "add_gelu", "fill", "sigmoid", "tanh", "sqrt", "exp", "gelu_bwd2"]
_OP_CODE = {name: i for i, name in enumerate(_OPS)}

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        L = C.CDLL(path)
        VP = C.POINTER(_View)
        L.orc_elementwise.argtypes = [C.c_int, C.c_int, C.POINTER(VP), VP, C.POINTER(C.c_double)]
        L.orc_elementwise.restype = C.c_int
        L.orc_reduce_axis.argtypes = [C.c_int, VP, C.c_int, C.c_int, VP]
        L.orc_reduce_axis.restype = C.c_int
        L.orc_gemm.argtypes = [VP, VP, VP, C.c_double, C.c_double, VP]
        L.orc_gemm.restype = C.c_int
        L.orc_gemm_entry.argtypes = [VP, VP, C.c_int64, C.c_int64]
        L.orc_gemm_entry.restype = C.c_double
        dp, ip = C.POINTER(C.c_double), C.POINTER(C.c_int64)
        L.orc_lstm_fwd.argtypes = [dp, dp, dp, C.c_int64, C.c_int64, dp, dp, dp]
        L.orc_lstm_fwd.restype = None
        L.orc_lstm_bwd.argtypes = [dp, dp, dp, dp, dp, C.c_int64, C.c_int64, dp, dp]
        L.orc_lstm_bwd.restype = None
        L.orc_softmax_ce_fwd.argtypes = [dp, ip, C.c_int64, C.c_int64, C.c_int64, dp, dp, dp]
        L.orc_softmax_ce_fwd.restype = C.c_int64
        L.orc_softmax_ce_bwd.argtypes = [dp, ip, C.c_int64, C.c_int64, C.c_int64, C.c_double, dp]
        L.orc_softmax_ce_bwd.restype = None
        L.orc_softmax_ce_bwd2.argtypes = [dp, ip, C.c_int64, C.c_int64, C.c_int64, C.c_double, dp, dp, dp]
        L.orc_softmax_ce_bwd2.restype = None
        L.orc_sgd_update.argtypes = [dp, dp, C.c_int64, C.c_double]
        L.orc_sgd_update.restype = None
        L.orc_embed_fwd.argtypes = [dp, ip, C.c_int64, C.c_int64, C.c_int64, dp]
        L.orc_embed_fwd.restype = None
        L.orc_embed_bwd.argtypes = [ip, dp, C.c_int64, C.c_int64, C.c_int64, C.c_int, dp]
        L.orc_embed_bwd.restype = None
        L.orc_round_bf16.argtypes = [dp, C.c_int64]
        L.orc_round_bf16.restype = None
        L.orc_num_threads.argtypes = []
        L.orc_num_threads.restype = C.c_int
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _f64(a):
    """Widen to float64 keeping the view's layout (strides scale with the item size)."""
    a = np.asarray(a)
    if a.dtype == np.float64:
        return a
    if a.size == 0:
        return np.zeros(a.shape)
    if any(s < 0 for s in a.strides):
        return a.astype(np.float64)
    es = [s // a.itemsize for s in a.strides]
    span = 1 + sum((n - 1) * e for n, e in zip(a.shape, es))
    flat = np.lib.stride_tricks.as_strided(a, shape=(span,), strides=(a.itemsize,),
                                           writeable=False)
    base = flat.astype(np.float64)
    return np.lib.stride_tricks.as_strided(base, shape=a.shape,
                                           strides=tuple(e * 8 for e in es), writeable=False)


def _view(a):
    v = _View()
    v.data = a.ctypes.data
    v.ndim = a.ndim
    for d in range(a.ndim):
        v.shape[d] = a.shape[d]
        v.strides[d] = a.strides[d]
    return v


def _dptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _iptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_int64))


def _c64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


def elementwise(op, inputs, out_shape=None, scalars=()):
    """NumPy-broadcast element-wise map; ``op`` is a name from ``_OPS``."""
    ins = [_f64(x) for x in inputs]
    if out_shape is None:
        out_shape = np.broadcast_shapes(*[x.shape for x in ins])
    out = np.empty(tuple(out_shape), dtype=np.float64)
    views = [_view(x) for x in ins]
    arr = (C.POINTER(_View) * max(1, len(views)))(*[C.pointer(v) for v in views])
    sc = (C.c_double * max(1, len(scalars)))(*[float(s) for s in scalars])
    rc = lib().orc_elementwise(_OP_CODE[op], len(views), arr, C.byref(_view(out)), sc)
    if rc != 0:
        raise ValueError("oracle: operands do not broadcast to the output shape")
    return out


def reduce_axis(op, x, axis, keepdims=False):
    """Fold ``+`` (op 'sum') or ``max`` over one axis."""
    x = _f64(x)
    ax = axis + x.ndim if axis < 0 else axis
    if not 0 <= ax < x.ndim:
        raise ValueError("oracle: axis out of range")
    shp = list(x.shape)
    if keepdims:
        shp[ax] = 1
    else:
        del shp[ax]
    out = np.empty(tuple(shp), dtype=np.float64)
    rc = lib().orc_reduce_axis({"sum": 0, "max": 1}[op], C.byref(_view(x)), axis, int(keepdims),
                               C.byref(_view(out)))
    if rc != 0:
        raise ValueError("oracle: bad reduce arguments")
    return out


def argmax_axis(x, axis, keepdims=False):
    """Index of the largest element along `axis`, the smallest such index among equals: written as
    the definition (first position where the slice equals its maximum)."""
    x = _f64(x)
    m = x.max(axis=axis, keepdims=True)
    idx = np.arange(x.shape[axis]).reshape([-1 if d == axis % x.ndim else 1 for d in range(x.ndim)])
    first = np.where(x == m, idx, x.shape[axis]).min(axis=axis, keepdims=keepdims)
    return first.astype(np.int64)


def gemm(A, B, Cin=None, alpha=1.0, beta=0.0):
    """alpha * A @ B + beta * Cin for 2-d views (transposition is expressed by strides)."""
    A, B = _f64(A), _f64(B)
    out = np.empty((A.shape[0], B.shape[1]), dtype=np.float64)
    cv = None
    if Cin is not None:
        Cin = _f64(Cin)
        cv = C.byref(_view(Cin))
    rc = lib().orc_gemm(C.byref(_view(A)), C.byref(_view(B)), cv, float(alpha), float(beta),
                        C.byref(_view(out)))
    if rc != 0:
        raise ValueError("oracle: gemm shapes do not agree")
    return out


def gemm_entries(A, B, ms, ns):
    """Selected entries (A @ B)[m, n] for spot checks at sizes the full product cannot afford."""
    A, B = _f64(A), _f64(B)
    va, vb = _view(A), _view(B)
    return np.array([lib().orc_gemm_entry(C.byref(va), C.byref(vb), int(m), int(n))
                     for m, n in zip(ms, ns)], dtype=np.float64)


def lstm_fwd(z, bias, c_prev):
    """Returns (c, h, gates) for pre-activations z (B,4H), gate order i,f,g,o."""
    z, c_prev = _c64(z), _c64(c_prev)
    B, H = c_prev.shape
    assert z.shape == (B, 4 * H)
    b = None if bias is None else _c64(bias)
    c, h, gates = np.empty((B, H)), np.empty((B, H)), np.empty((B, 4 * H))
    lib().orc_lstm_fwd(_dptr(z), None if b is None else _dptr(b), _dptr(c_prev), B, H,
                       _dptr(c), _dptr(h), _dptr(gates))
    return c, h, gates


def lstm_bwd(gates, c_prev, c, dh, dc_next=None):
    """Returns (dz, dc_prev) from retained outputs (activated gates, c) and c_prev."""
    gates, c_prev, c, dh = _c64(gates), _c64(c_prev), _c64(c), _c64(dh)
    B, H = c.shape
    dcn = None if dc_next is None else _c64(dc_next)
    dz, dcp = np.empty((B, 4 * H)), np.empty((B, H))
    lib().orc_lstm_bwd(_dptr(gates), _dptr(c_prev), _dptr(c), _dptr(dh),
                       None if dcn is None else _dptr(dcn), B, H, _dptr(dz), _dptr(dcp))
    return dz, dcp


def softmax_ce_fwd(logits, labels, ignore_label=-1):
    """Returns (loss_mean, loss_rows, lse, n_valid)."""
    z, t = _c64(logits), _i64(labels)
    N, Cn = z.shape
    loss = C.c_double(0.0)
    rows, lse = np.empty(N), np.empty(N)
    nv = lib().orc_softmax_ce_fwd(_dptr(z), _iptr(t), N, Cn, int(ignore_label), C.byref(loss),
                                  _dptr(rows), _dptr(lse))
    return float(loss.value), rows, lse, int(nv)


def softmax_ce_bwd(logits, labels, ignore_label=-1, upstream=1.0):
    z, t = _c64(logits), _i64(labels)
    N, Cn = z.shape
    dz = np.empty((N, Cn))
    lib().orc_softmax_ce_bwd(_dptr(z), _iptr(t), N, Cn, int(ignore_label), float(upstream), _dptr(dz))
    return dz


def softmax_ce_bwd2(logits, labels, gg, ignore_label=-1, upstream=1.0):
    """Derivative of softmax_ce_bwd: returns (dlogits, dupstream) for the gradient gg reaching its result."""
    z, t, u = _c64(logits), _i64(labels), _c64(gg)
    N, Cn = z.shape
    dz = np.empty((N, Cn))
    du = C.c_double(0.0)
    lib().orc_softmax_ce_bwd2(_dptr(z), _iptr(t), N, Cn, int(ignore_label), float(upstream), _dptr(u), _dptr(dz), C.byref(du))
    return dz, float(du.value)


def sgd_update(p, g, lr):
    """Returns the updated parameter (the input is not modified)."""
    out = _c64(p).copy()
    g = _c64(g)
    assert out.shape == g.shape
    lib().orc_sgd_update(_dptr(out), _dptr(g), out.size, float(lr))
    return out


def adam_update(p, g, m, v, lr, step, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam step (Kingma & Ba, Algorithm 1), written out: returns (p', m', v').  `step` counts from 1."""
    p, g, m, v = (np.asarray(a, dtype=np.float64) for a in (p, g, m, v))
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    return p - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def embed_fwd(table, ids):
    table, ids = _c64(table), _i64(ids).reshape(-1)
    out = np.empty((ids.size, table.shape[1]))
    lib().orc_embed_fwd(_dptr(table), _iptr(ids), ids.size, table.shape[1], table.shape[0], _dptr(out))
    return out


def embed_bwd(ids, dout, V, dtable=None):
    """dtable (V,D): zero (or the given array, accumulated into a copy) plus the scattered rows."""
    ids, dout = _i64(ids).reshape(-1), _c64(dout)
    D = dout.shape[1]
    acc = dtable is not None
    out = _c64(dtable).copy() if acc else np.empty((V, D))
    lib().orc_embed_bwd(_iptr(ids), _dptr(dout), ids.size, D, V, int(acc), _dptr(out))
    return out


def round_bf16(x):
    """Nearest-even rounding of each value to bfloat16, returned as float64."""
    out = _c64(x).copy()
    lib().orc_round_bf16(_dptr(out), out.size)
    return out
