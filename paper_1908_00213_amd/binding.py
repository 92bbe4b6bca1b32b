"""Thin ctypes binding of libchn (argument marshalling only; every step runs in the HIP kernels).

Functions carry the names of the C entry points in ``include/chn.h`` without the ``chn_`` prefix.
Arrays are ``torch.Tensor`` objects on the GPU: PyTorch supplies device memory and the stream, nothing
else.  Each call turns its tensors into ``chn_array`` descriptors (data pointer, shape, BYTE strides,
dtype), passes ``torch.cuda.current_stream()`` and raises :class:`ChnError` on a non-zero status.
The library must have been built (``python -m paper_1908_00213_amd.build``); there is no fallback.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libchn.so")
MAX_NDIM = 8

F32, BF16, I32, I64 = 0, 1, 2, 3
_DTYPES = {torch.float32: F32, torch.bfloat16: BF16, torch.int32: I32, torch.int64: I64}

OPS = ["copy", "add", "sub", "mul", "mad", "mad_relu", "relu", "relu_bwd", "gelu", "gelu_bwd",
       "scale", "axpy", "add_relu", "add_gelu", "fill", "sigmoid", "tanh", "sqrt"]
OP = {n: i for i, n in enumerate(OPS)}
REDUCE = {"sum": 0, "max": 1}
EPILOGUES = ["none", "bias", "bias_relu", "bias_gelu", "relu_bwd", "gelu_bwd", "bf16_copy"]
EPI = {n: i for i, n in enumerate(EPILOGUES)}

EXPORTS = ["chn_elementwise_broadcast", "chn_reduce_axis_workspace_bytes", "chn_reduce_axis",
           "chn_gemm_workspace_bytes", "chn_gemm", "chn_lstm_fwd", "chn_lstm_bwd",
           "chn_softmax_ce_workspace_bytes", "chn_softmax_ce_fwd", "chn_softmax_ce_bwd",
           "chn_sgd_update", "chn_sgd_update_multi", "chn_embed_fwd", "chn_embed_bwd",
           "chn_status_string", "chn_last_error", "chn_version", "chn_elementwise_plan", "chn_gemm_plan"]


class ChnArray(C.Structure):
    _fields_ = [("data", C.c_void_p), ("ndim", C.c_int32), ("shape", C.c_int64 * MAX_NDIM),
                ("strides", C.c_int64 * MAX_NDIM), ("dtype", C.c_int32)]


class ChnError(RuntimeError):
    def __init__(self, status, detail):
        super().__init__("chn status %d: %s" % (status, detail))
        self.status = status


_lib = None


def lib():
    """Load libchn.so; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libchn.so is missing: run `python -m paper_1908_00213_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    AP = C.POINTER(ChnArray)
    APP = C.POINTER(AP)
    vp, st = C.c_void_p, C.c_void_p
    L.chn_elementwise_broadcast.argtypes = [C.c_int, C.c_int, APP, AP, C.POINTER(C.c_float), C.c_int, st]
    L.chn_elementwise_plan.argtypes = [C.c_int, C.c_int, APP, AP]
    L.chn_reduce_axis_workspace_bytes.argtypes = [AP, C.c_int]
    L.chn_reduce_axis_workspace_bytes.restype = C.c_size_t
    L.chn_reduce_axis.argtypes = [C.c_int, AP, C.c_int, C.c_int, AP, vp, C.c_size_t, st]
    L.chn_gemm_workspace_bytes.argtypes = [AP, AP, AP]
    L.chn_gemm_workspace_bytes.restype = C.c_size_t
    L.chn_gemm_plan.argtypes = [AP, AP, AP, C.c_int]
    L.chn_gemm.argtypes = [AP, AP, AP, C.c_float, C.c_float, C.c_int, AP, AP, AP, vp, C.c_size_t, st]
    L.chn_lstm_fwd.argtypes = [AP, AP, AP, AP, AP, AP, st]
    L.chn_lstm_bwd.argtypes = [AP, AP, AP, AP, AP, AP, AP, st]
    L.chn_softmax_ce_workspace_bytes.argtypes = [C.c_int64]
    L.chn_softmax_ce_workspace_bytes.restype = C.c_size_t
    L.chn_softmax_ce_fwd.argtypes = [AP, AP, C.c_int64, AP, AP, AP, vp, C.c_size_t, st]
    L.chn_softmax_ce_bwd.argtypes = [AP, AP, C.c_int64, AP, C.c_float, AP, vp, C.c_size_t, st]
    L.chn_sgd_update.argtypes = [AP, AP, C.c_float, AP, st]
    L.chn_sgd_update_multi.argtypes = [C.c_int, APP, APP, C.c_float, APP, st]
    L.chn_embed_fwd.argtypes = [AP, AP, AP, st]
    L.chn_embed_bwd.argtypes = [AP, AP, AP, C.c_int, st]
    L.chn_status_string.argtypes = [C.c_int32]
    L.chn_status_string.restype = C.c_char_p
    L.chn_last_error.argtypes = []
    L.chn_last_error.restype = C.c_char_p
    L.chn_version.argtypes = []
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is C.c_int and name not in ("chn_version", "chn_elementwise_plan", "chn_gemm_plan"):
            fn.restype = C.c_int32
    _lib = L
    return L


def desc(t):
    """chn_array descriptor of a tensor (or None)."""
    if t is None:
        return None
    if isinstance(t, ChnArray):
        return t
    a = ChnArray()
    n = t.dim()
    isz = t.element_size()
    a.data = t.data_ptr()
    a.ndim = n
    a.shape[:n] = t.shape
    a.strides[:n] = [s * isz for s in t.stride()]
    a.dtype = _DTYPES[t.dtype]
    return a


def raw_desc(ptr, shape, strides_bytes, dtype):
    """Descriptor from raw fields (used by tests of the validation paths)."""
    a = ChnArray()
    a.data = ptr
    a.ndim = len(shape)
    for d, (n, s) in enumerate(zip(shape, strides_bytes)):
        if d < MAX_NDIM:
            a.shape[d] = n
            a.strides[d] = s
    a.dtype = dtype
    return a


def _ref(a):
    return None if a is None else C.byref(a)


def _ptrs(descs):
    AP = C.POINTER(ChnArray)
    arr = (AP * max(1, len(descs)))()
    for i, d in enumerate(descs):
        arr[i] = C.pointer(d) if d is not None else AP()
    return arr


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status):
    if status != 0:
        L = lib()
        raise ChnError(status, "%s: %s" % (L.chn_status_string(status).decode(), L.chn_last_error().decode()))


def _ws(t):
    if t is None:
        return None, 0
    return C.c_void_p(t.data_ptr()), t.numel() * t.element_size()


def version():
    return lib().chn_version()


def elementwise_plan(op, inputs, out):
    ds = [desc(x) for x in inputs]
    return lib().chn_elementwise_plan(OP[op] if isinstance(op, str) else op, len(ds), _ptrs(ds), _ref(desc(out)))


def elementwise_broadcast(op, inputs, out, scalars=(), stream=None):
    ds = [desc(x) for x in inputs]
    sc = (C.c_float * max(1, len(scalars)))(*[float(s) for s in scalars])
    _check(lib().chn_elementwise_broadcast(OP[op] if isinstance(op, str) else op, len(ds), _ptrs(ds),
                                           _ref(desc(out)), sc, len(scalars),
                                           _stream() if stream is None else stream))
    return out


def reduce_axis_workspace_bytes(x, axis):
    return lib().chn_reduce_axis_workspace_bytes(_ref(desc(x)), axis)


def reduce_axis(op, x, axis, out, keepdims=False, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().chn_reduce_axis(REDUCE[op] if isinstance(op, str) else op, _ref(desc(x)), axis,
                                 int(keepdims), _ref(desc(out)), p, n,
                                 _stream() if stream is None else stream))
    return out


def gemm_workspace_bytes(A, B, Cm):
    return lib().chn_gemm_workspace_bytes(_ref(desc(A)), _ref(desc(B)), _ref(desc(Cm)))


def gemm_plan(A, B, Cm, have_workspace=False):
    """(tile, direct_copy, splits) chn_gemm would use: tile 0/1/2 = 64/128/256 square."""
    code = lib().chn_gemm_plan(_ref(desc(A)), _ref(desc(B)), _ref(desc(Cm)), 1 if have_workspace else 0)
    if code < 0:
        _check(code)
    return code & 3, bool(code & 4), code >> 4


def gemm(A, B, Cm, alpha=1.0, beta=0.0, epilogue="none", bias=None, aux=None, preact_out=None,
         ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().chn_gemm(_ref(desc(A)), _ref(desc(B)), _ref(desc(Cm)), float(alpha), float(beta),
                          EPI[epilogue] if isinstance(epilogue, str) else epilogue,
                          _ref(desc(bias)), _ref(desc(aux)), _ref(desc(preact_out)), p, n,
                          _stream() if stream is None else stream))
    return Cm


def lstm_fwd(z, bias, c_prev, c, h, gates=None, stream=None):
    _check(lib().chn_lstm_fwd(_ref(desc(z)), _ref(desc(bias)), _ref(desc(c_prev)), _ref(desc(c)),
                              _ref(desc(h)), _ref(desc(gates)), _stream() if stream is None else stream))


def lstm_bwd(gates, c_prev, c, dh, dc_next, dz, dc_prev, stream=None):
    _check(lib().chn_lstm_bwd(_ref(desc(gates)), _ref(desc(c_prev)), _ref(desc(c)), _ref(desc(dh)),
                              _ref(desc(dc_next)), _ref(desc(dz)), _ref(desc(dc_prev)),
                              _stream() if stream is None else stream))


def softmax_ce_workspace_bytes(n_rows):
    return lib().chn_softmax_ce_workspace_bytes(int(n_rows))


def softmax_ce_fwd(logits, labels, loss_mean, loss_rows=None, lse=None, ignore_label=-1, ws=None,
                   stream=None):
    p, n = _ws(ws)
    _check(lib().chn_softmax_ce_fwd(_ref(desc(logits)), _ref(desc(labels)), int(ignore_label),
                                    _ref(desc(loss_mean)), _ref(desc(loss_rows)), _ref(desc(lse)), p, n,
                                    _stream() if stream is None else stream))
    return loss_mean


def softmax_ce_bwd(logits, labels, dlogits, lse=None, upstream=1.0, ignore_label=-1, ws=None,
                   stream=None):
    p, n = _ws(ws)
    _check(lib().chn_softmax_ce_bwd(_ref(desc(logits)), _ref(desc(labels)), int(ignore_label),
                                    _ref(desc(lse)), float(upstream), _ref(desc(dlogits)), p, n,
                                    _stream() if stream is None else stream))
    return dlogits


def sgd_update(param, grad, lr, lowp_copy=None, stream=None):
    _check(lib().chn_sgd_update(_ref(desc(param)), _ref(desc(grad)), float(lr), _ref(desc(lowp_copy)),
                                _stream() if stream is None else stream))


def sgd_update_multi(params, grads, lr, lowp_copies=None, stream=None):
    ps, gs = [desc(p) for p in params], [desc(g) for g in grads]
    ls = None if lowp_copies is None else [desc(l) for l in lowp_copies]
    _check(lib().chn_sgd_update_multi(len(ps), _ptrs(ps), _ptrs(gs), float(lr),
                                      None if ls is None else _ptrs(ls),
                                      _stream() if stream is None else stream))


def embed_fwd(table, ids, out, stream=None):
    _check(lib().chn_embed_fwd(_ref(desc(table)), _ref(desc(ids)), _ref(desc(out)),
                               _stream() if stream is None else stream))
    return out


def embed_bwd(ids, dout, dtable, accumulate=False, stream=None):
    _check(lib().chn_embed_bwd(_ref(desc(ids)), _ref(desc(dout)), _ref(desc(dtable)), int(accumulate),
                               _stream() if stream is None else stream))
    return dtable
