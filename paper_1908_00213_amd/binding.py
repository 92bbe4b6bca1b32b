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
       "scale", "axpy", "add_relu", "add_gelu", "fill", "sigmoid", "tanh", "sqrt", "exp", "gelu_bwd2"]
OP = {n: i for i, n in enumerate(OPS)}
REDUCE = {"sum": 0, "max": 1}
EPILOGUES = ["none", "bias", "bias_relu", "bias_gelu", "relu_bwd", "gelu_bwd", "bf16_copy"]
EPI = {n: i for i, n in enumerate(EPILOGUES)}

EXPORTS = ["chn_elementwise_broadcast", "chn_reduce_axis_workspace_bytes", "chn_reduce_axis", "chn_reduce_axis_static", "chn_argmax_axis",
           "chn_gemm_workspace_bytes", "chn_gemm", "chn_lstm_fwd", "chn_lstm_bwd", "chn_lstm_step_fwd", "chn_lstm_step_bwd",
           "chn_lstm_seq_workspace_bytes", "chn_lstm_seq_supported", "chn_lstm_seq_fwd",
           "chn_lstm_seq_bwd_supported", "chn_lstm_seq_bwd_workspace_bytes", "chn_lstm_seq_bwd", "chn_lstm_seq_spin_limit",
           "chn_softmax_ce_workspace_bytes", "chn_softmax_ce_fwd", "chn_softmax_ce_bwd", "chn_softmax_ce_bwd2", "chn_softmax_ce_fwd_bwd",
           "chn_sgd_update", "chn_sgd_update_multi", "chn_adam_update_multi", "chn_embed_fwd", "chn_embed_bwd",
           "chn_status_string", "chn_last_error", "chn_version", "chn_elementwise_plan", "chn_gemm_plan", "chn_gemm_plan_override",
           "chn_user_kernel_config", "chn_user_kernel_stats", "chn_user_kernel_destroy",
           "chn_elementwise_kernel_create", "chn_elementwise_kernel_prepare", "chn_elementwise_kernel_launch",
           "chn_reduction_kernel_create", "chn_reduction_kernel_workspace_bytes", "chn_reduction_kernel_prepare",
           "chn_reduction_kernel_launch", "chn_user_kernel_source"]
AXIS_ALL = -1000


def _axis_code(axis, ndim):
    """The C ABI's axis argument: one axis, CHN_AXIS_ALL for None, CHN_AXES(mask) for a tuple."""
    if axis is None:
        return AXIS_ALL
    if isinstance(axis, (tuple, list)):
        mask = 0
        for a in axis:
            mask |= 1 << (a % ndim)
        return 0x40000000 + mask
    return int(axis)


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
    L.chn_reduce_axis_static.argtypes = [C.c_int, AP, C.c_int, C.c_int, AP, st]
    L.chn_argmax_axis.argtypes = [AP, C.c_int, C.c_int, AP, st]
    L.chn_gemm_workspace_bytes.argtypes = [AP, AP, AP]
    L.chn_gemm_workspace_bytes.restype = C.c_size_t
    L.chn_gemm_plan.argtypes = [AP, AP, AP, C.c_int]
    L.chn_gemm_plan_override.argtypes = [C.c_int, C.c_int, C.c_int]
    L.chn_gemm_plan_override.restype = None
    L.chn_gemm.argtypes = [AP, AP, AP, C.c_float, C.c_float, C.c_int, AP, AP, AP, vp, C.c_size_t, st]
    L.chn_lstm_fwd.argtypes = [AP, AP, AP, AP, AP, AP, st]
    L.chn_lstm_bwd.argtypes = [AP, AP, AP, AP, AP, AP, AP, st]
    L.chn_lstm_step_fwd.argtypes = [AP, AP, AP, AP, AP, AP, AP, AP, st]
    L.chn_lstm_step_bwd.argtypes = [AP, AP, AP, AP, AP, AP, AP, AP, AP, st]
    L.chn_lstm_seq_workspace_bytes.argtypes = [C.c_int64]
    L.chn_lstm_seq_workspace_bytes.restype = C.c_size_t
    L.chn_lstm_seq_supported.argtypes = [C.c_int64, C.c_int64, C.c_int]
    L.chn_lstm_seq_fwd.argtypes = [AP, AP, AP, AP, AP, AP, C.c_int64, C.c_void_p, C.c_size_t, st]
    L.chn_lstm_seq_bwd_supported.argtypes = [C.c_int64, C.c_int64, C.c_int]
    L.chn_lstm_seq_bwd_workspace_bytes.argtypes = [C.c_int64, C.c_int64]
    L.chn_lstm_seq_bwd_workspace_bytes.restype = C.c_size_t
    L.chn_lstm_seq_bwd.argtypes = [AP, AP, AP, AP, AP, AP, AP, C.c_int64, C.c_void_p, C.c_size_t, st]
    L.chn_lstm_seq_spin_limit.argtypes = [C.c_int64]
    L.chn_lstm_seq_spin_limit.restype = None
    L.chn_softmax_ce_workspace_bytes.argtypes = [C.c_int64]
    L.chn_softmax_ce_workspace_bytes.restype = C.c_size_t
    L.chn_softmax_ce_fwd.argtypes = [AP, AP, C.c_int64, AP, AP, AP, vp, C.c_size_t, st]
    L.chn_softmax_ce_bwd.argtypes = [AP, AP, C.c_int64, AP, C.c_float, AP, vp, C.c_size_t, st]
    L.chn_softmax_ce_fwd_bwd.argtypes = [AP, AP, C.c_int64, AP, AP, C.c_float, AP, vp, C.c_size_t, st]
    L.chn_softmax_ce_bwd2.argtypes = [AP, AP, C.c_int64, AP, C.c_float, AP, AP, AP, vp, C.c_size_t, st]
    L.chn_sgd_update.argtypes = [AP, AP, C.c_float, AP, st]
    L.chn_sgd_update_multi.argtypes = [C.c_int, APP, APP, C.c_float, APP, st]
    L.chn_adam_update_multi.argtypes = [C.c_int, APP, APP, APP, APP, C.c_double, C.c_double, C.c_double, C.c_double, C.c_int64, APP, st]
    L.chn_embed_fwd.argtypes = [AP, AP, AP, st]
    L.chn_embed_bwd.argtypes = [AP, AP, AP, C.c_int, st]
    L.chn_status_string.argtypes = [C.c_int32]
    L.chn_status_string.restype = C.c_char_p
    L.chn_last_error.argtypes = []
    L.chn_last_error.restype = C.c_char_p
    L.chn_version.argtypes = []
    cs, KP, dp = C.c_char_p, C.c_void_p, C.POINTER(C.c_double)
    L.chn_user_kernel_config.argtypes = [cs, cs]
    L.chn_user_kernel_stats.argtypes = [C.POINTER(C.c_longlong)] * 3
    L.chn_user_kernel_stats.restype = None
    L.chn_user_kernel_destroy.argtypes = [KP]
    L.chn_user_kernel_destroy.restype = None
    L.chn_elementwise_kernel_create.argtypes = [cs, cs, cs, cs, cs, C.POINTER(KP)]
    L.chn_elementwise_kernel_prepare.argtypes = [KP, C.c_int, APP, C.c_int, APP]
    L.chn_elementwise_kernel_launch.argtypes = [KP, C.c_int, APP, C.c_int, APP, dp, st]
    L.chn_reduction_kernel_create.argtypes = [cs, cs, cs, cs, cs, cs, cs, cs, C.POINTER(KP)]
    L.chn_reduction_kernel_workspace_bytes.argtypes = [KP, C.c_int, APP, C.c_int, APP, C.c_int, C.c_int]
    L.chn_reduction_kernel_workspace_bytes.restype = C.c_size_t
    L.chn_reduction_kernel_prepare.argtypes = [KP, C.c_int, APP, C.c_int, APP, C.c_int, C.c_int]
    L.chn_reduction_kernel_launch.argtypes = [KP, C.c_int, APP, C.c_int, APP, dp, C.c_int, C.c_int, vp, C.c_size_t, st]
    L.chn_user_kernel_source.argtypes = [KP, C.c_int, APP, C.c_int, APP, C.c_int, C.c_int, C.c_char_p, C.c_size_t,
                                         C.POINTER(C.c_size_t)]
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is C.c_int and name not in ("chn_version", "chn_elementwise_plan", "chn_gemm_plan"):  # i.e. not set above
            fn.restype = C.c_int32
    _lib = L
    return L


def desc(t):
    """chn_array descriptor of a tensor (or None).  The descriptor is kept on the tensor object: a
    tensor's storage pointer, shape and strides do not change for the life of the object (this
    package never calls the in-place re-shaping methods that could), and parameters, inputs and
    gradients are described thousands of times."""
    if t is None:
        return None
    if isinstance(t, ChnArray):
        return t
    try:
        return t._chn_desc
    except AttributeError:
        pass
    a = ChnArray()
    n = t.dim()
    isz = t.element_size()
    a.data = t.data_ptr()
    a.ndim = n
    a.shape[:n] = t.shape
    a.strides[:n] = [s * isz for s in t.stride()]
    a.dtype = _DTYPES[t.dtype]
    t._chn_desc = a
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


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
_raw_device = getattr(torch._C, "_cuda_getDevice", None)


def _stream():
    """hipStream_t of torch's current stream (the raw-handle query costs a fraction of a microsecond,
    the Stream object several)."""
    if _raw_stream is not None and _raw_device is not None:
        return C.c_void_p(_raw_stream(_raw_device()))
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


def cast(x, dtype):
    """A copy of `x` in another storage type through the library's own kernel (CHN_OP_COPY: fp32 values
    round to nearest even on their way to bfloat16); torch only allocates the result."""
    if x.dtype == dtype:
        return x
    return elementwise_broadcast("copy", [x], torch.empty(x.shape, dtype=dtype, device=x.device))


def reduce_axis_workspace_bytes(x, axis):
    d = desc(x)
    return lib().chn_reduce_axis_workspace_bytes(_ref(d), _axis_code(axis, d.ndim))


def reduce_axis(op, x, axis, out, keepdims=False, ws=None, stream=None):
    """axis: an int, a tuple of ints (several axes at once) or None (all of them)."""
    p, n = _ws(ws)
    axis = _axis_code(axis, desc(x).ndim)
    _check(lib().chn_reduce_axis(REDUCE[op] if isinstance(op, str) else op, _ref(desc(x)), axis,
                                 int(keepdims), _ref(desc(out)), p, n,
                                 _stream() if stream is None else stream))
    return out


def reduce_axis_static(op, x, axis, out, keepdims=False, stream=None):
    """reduce_axis without a workspace argument and without any allocation (partial sums in the
    library's built-in per-device array)."""
    axis = _axis_code(axis, desc(x).ndim)
    _check(lib().chn_reduce_axis_static(REDUCE[op] if isinstance(op, str) else op, _ref(desc(x)), axis,
                                        int(keepdims), _ref(desc(out)), _stream() if stream is None else stream))
    return out


def argmax_axis(x, axis, out, keepdims=False, stream=None):
    _check(lib().chn_argmax_axis(_ref(desc(x)), int(axis), int(keepdims), _ref(desc(out)),
                                 _stream() if stream is None else stream))
    return out


def gemm_workspace_bytes(A, B, Cm):
    return lib().chn_gemm_workspace_bytes(_ref(desc(A)), _ref(desc(B)), _ref(desc(Cm)))


def gemm_plan(A, B, Cm, have_workspace=False):
    """(tile, direct_copy, splits) chn_gemm would use: tile 0/1/2 = 64/128/256 square, 3 = 256 x 128."""
    code = lib().chn_gemm_plan(_ref(desc(A)), _ref(desc(B)), _ref(desc(Cm)), 1 if have_workspace else 0)
    if code < 0:
        _check(code)
    return code & 3, bool(code & 4), code >> 4


def gemm_plan_eight_waves(A, B, Cm, have_workspace=False):
    """Whether the plain product would run on the eight-wave form of the direct-copy kernel."""
    code = lib().chn_gemm_plan(_ref(desc(A)), _ref(desc(B)), _ref(desc(Cm)), 1 if have_workspace else 0)
    if code < 0:
        _check(code)
    return bool(code & 8)


def gemm_plan_override(tile=-1, splits=-1, direct_copy=-1):
    """Test hook: force the macro tile / K splits / keep products off the direct-copy kernel (-1: planner's choice)."""
    lib().chn_gemm_plan_override(int(tile), int(splits), int(direct_copy))


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


def lstm_step_fwd(zx, h_prev, Ut, bias, c_prev, c, h, gates=None, stream=None):
    _check(lib().chn_lstm_step_fwd(_ref(desc(zx)), _ref(desc(h_prev)), _ref(desc(Ut)), _ref(desc(bias)), _ref(desc(c_prev)),
                                   _ref(desc(c)), _ref(desc(h)), _ref(desc(gates)), _stream() if stream is None else stream))


def lstm_step_bwd(dz_next, U, dh, gates, c_prev, c, dc_next, dz, dc_prev, stream=None):
    _check(lib().chn_lstm_step_bwd(_ref(desc(dz_next)), _ref(desc(U)), _ref(desc(dh)), _ref(desc(gates)), _ref(desc(c_prev)),
                                   _ref(desc(c)), _ref(desc(dc_next)), _ref(desc(dz)), _ref(desc(dc_prev)),
                                   _stream() if stream is None else stream))


def lstm_seq_workspace_bytes(batch):
    return lib().chn_lstm_seq_workspace_bytes(int(batch))


def lstm_seq_supported(batch, hidden, dtype):
    """Whether lstm_seq_fwd takes this batch and hidden width (torch dtype) on the current device."""
    return lib().chn_lstm_seq_supported(int(batch), int(hidden), _DTYPES[dtype]) == 0


def lstm_seq_status(ws):
    """The status word lstm_seq_fwd left in its workspace (synchronises): 0 = complete, 1 = a wait ran out."""
    return int(ws[:4].view(torch.int32).item())


def lstm_seq_fwd(zx, Ut, bias, Hs, Cs, gates, n_steps, ws, stream=None):
    """All n_steps forward steps in one launch.  ws[0:4] reads 1 after synchronisation if a wait ran out."""
    p, n = _ws(ws)
    _check(lib().chn_lstm_seq_fwd(_ref(desc(zx)), _ref(desc(Ut)), _ref(desc(bias)), _ref(desc(Hs)), _ref(desc(Cs)),
                                  _ref(desc(gates)), int(n_steps), p, n, _stream() if stream is None else stream))


def lstm_seq_bwd_supported(batch, hidden, dtype):
    return lib().chn_lstm_seq_bwd_supported(int(batch), int(hidden), _DTYPES[dtype]) == 0


def lstm_seq_bwd_workspace_bytes(batch, hidden):
    return lib().chn_lstm_seq_bwd_workspace_bytes(int(batch), int(hidden))


def lstm_seq_bwd(U, dHs, gates, Cs, dc_last, dZ, dc0, n_steps, ws, stream=None):
    """Back-propagation through all n_steps steps in one launch; status word in ws as for lstm_seq_fwd."""
    p, n = _ws(ws)
    _check(lib().chn_lstm_seq_bwd(_ref(desc(U)), _ref(desc(dHs)), _ref(desc(gates)), _ref(desc(Cs)), _ref(desc(dc_last)),
                                  _ref(desc(dZ)), _ref(desc(dc0)), int(n_steps), p, n, _stream() if stream is None else stream))


def lstm_seq_spin_limit(polls):
    lib().chn_lstm_seq_spin_limit(int(polls))


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


def softmax_ce_bwd2(logits, labels, gg, dlogits, dupstream=None, lse=None, upstream=1.0, ignore_label=-1, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().chn_softmax_ce_bwd2(_ref(desc(logits)), _ref(desc(labels)), int(ignore_label), _ref(desc(lse)), float(upstream),
                                     _ref(desc(gg)), _ref(desc(dlogits)), _ref(desc(dupstream)), p, n,
                                     _stream() if stream is None else stream))
    return dlogits


def softmax_ce_fwd_bwd(logits, labels, loss_mean, dlogits, lse=None, upstream=1.0, ignore_label=-1, ws=None,
                       stream=None):
    p, n = _ws(ws)
    _check(lib().chn_softmax_ce_fwd_bwd(_ref(desc(logits)), _ref(desc(labels)), int(ignore_label), _ref(desc(loss_mean)),
                                        _ref(desc(lse)), float(upstream), _ref(desc(dlogits)), p, n,
                                        _stream() if stream is None else stream))
    return loss_mean


def sgd_update(param, grad, lr, lowp_copy=None, stream=None):
    _check(lib().chn_sgd_update(_ref(desc(param)), _ref(desc(grad)), float(lr), _ref(desc(lowp_copy)),
                                _stream() if stream is None else stream))


def sgd_update_multi(params, grads, lr, lowp_copies=None, stream=None):
    ps, gs = [desc(p) for p in params], [desc(g) for g in grads]
    ls = None if lowp_copies is None else [desc(l) for l in lowp_copies]
    _check(lib().chn_sgd_update_multi(len(ps), _ptrs(ps), _ptrs(gs), float(lr),
                                      None if ls is None else _ptrs(ls),
                                      _stream() if stream is None else stream))


def _row_block(t, rows):
    """Descriptor of the first `rows` rows of a 2-d tensor and the byte distance to the next such block:
    a sequence of calls over consecutive row blocks moves the data pointer instead of slicing."""
    isz = t.element_size()
    return raw_desc(t.data_ptr(), (rows, t.shape[1]), (t.stride(0) * isz, t.stride(1) * isz), _DTYPES[t.dtype]), rows * t.stride(0) * isz


def lstm_step_fwd_seq(zx, Hs, Ut, bias, Cs, gates, n_steps, stream=None):
    """n_steps calls of lstm_step_fwd over time-major buffers: step t reads rows t*B.. of zx, block t of
    Hs and Cs ((n_steps+1)*B rows, block 0 = initial state) and writes block t+1 of Hs and Cs and block t
    of gates.  Same calls as the loop over slices; only the marshalling is done once."""
    L, st = lib(), (_stream() if stream is None else stream)
    Bn = zx.shape[0] // n_steps
    if zx.shape[0] != n_steps * Bn or Hs.shape[0] != (n_steps + 1) * Bn or Cs.shape[0] != (n_steps + 1) * Bn or gates.shape[0] != n_steps * Bn:
        raise ValueError("lstm_step_fwd_seq: buffers do not hold %d steps" % n_steps)
    (zd, zs), (hp, hs), (cp, cs), (gd, gs) = _row_block(zx, Bn), _row_block(Hs, Bn), _row_block(Cs, Bn), _row_block(gates, Bn)
    (hn, _), (cn, _) = _row_block(Hs, Bn), _row_block(Cs, Bn)
    hn.data += hs
    cn.data += cs
    ut, bd = _ref(desc(Ut)), _ref(desc(bias))
    for _ in range(n_steps):
        _check(L.chn_lstm_step_fwd(C.byref(zd), C.byref(hp), ut, bd, C.byref(cp), C.byref(cn), C.byref(hn), C.byref(gd), st))
        zd.data += zs; hp.data += hs; hn.data += hs; cp.data += cs; cn.data += cs; gd.data += gs


def lstm_step_bwd_seq(dZ, U, dHs, gates, Cs, dc_last, dc, n_steps, stream=None):
    """The n_steps calls of lstm_step_bwd of one back-propagation through time, last step first: dZ, dHs
    and gates hold n_steps row blocks, Cs n_steps + 1; dc_last (or None) is the gradient reaching the
    final cell state; dc = two (B, H) buffers that take turns (the one of step 0 holds the gradient
    of the initial cell state afterwards)."""
    L, st = lib(), (_stream() if stream is None else stream)
    Bn = dZ.shape[0] // n_steps
    if dZ.shape[0] != n_steps * Bn or dHs.shape[0] != n_steps * Bn or gates.shape[0] != n_steps * Bn or Cs.shape[0] != (n_steps + 1) * Bn:
        raise ValueError("lstm_step_bwd_seq: buffers do not hold %d steps" % n_steps)
    (zd, zs), (zn, _), (hd, hs), (gd, gs), (cp, cs), (cn, _) = (_row_block(dZ, Bn), _row_block(dZ, Bn), _row_block(dHs, Bn),
                                                             _row_block(gates, Bn), _row_block(Cs, Bn), _row_block(Cs, Bn))
    last = n_steps - 1
    zd.data += last * zs; zn.data += (last + 1) * zs; hd.data += last * hs; gd.data += last * gs; cp.data += last * cs; cn.data += (last + 1) * cs
    ud = _ref(desc(U))
    dcd = [C.byref(desc(dc[0])), C.byref(desc(dc[1]))]
    dc_next = _ref(desc(dc_last))
    for t in range(last, -1, -1):
        _check(L.chn_lstm_step_bwd(None if t == last else C.byref(zn), ud, C.byref(hd), C.byref(gd), C.byref(cp), C.byref(cn),
                                   dc_next, C.byref(zd), dcd[t & 1], st))
        dc_next = dcd[t & 1]
        zd.data -= zs; zn.data -= zs; hd.data -= hs; gd.data -= gs; cp.data -= cs; cn.data -= cs


def adam_update_multi(params, grads, ms, vs, lr, step, beta1=0.9, beta2=0.999, eps=1e-8, lowp_copies=None, stream=None):
    ps, gs, m_, v_ = ([desc(t) for t in ts] for ts in (params, grads, ms, vs))
    ls = None if lowp_copies is None else [desc(l) for l in lowp_copies]
    _check(lib().chn_adam_update_multi(len(ps), _ptrs(ps), _ptrs(gs), _ptrs(m_), _ptrs(v_), float(lr), float(beta1),
                                       float(beta2), float(eps), int(step), None if ls is None else _ptrs(ls),
                                       _stream() if stream is None else stream))


def embed_fwd(table, ids, out, stream=None):
    _check(lib().chn_embed_fwd(_ref(desc(table)), _ref(desc(ids)), _ref(desc(out)),
                               _stream() if stream is None else stream))
    return out


def embed_bwd(ids, dout, dtable, accumulate=False, stream=None):
    _check(lib().chn_embed_bwd(_ref(desc(ids)), _ref(desc(dout)), _ref(desc(dtable)), int(accumulate),
                               _stream() if stream is None else stream))
    return dtable


# ---- user-defined kernels ---------------------------------------------------------------------------------
def user_kernel_config(cache_dir=None, arch=None):
    enc = lambda v: None if v is None else str(v).encode()
    _check(lib().chn_user_kernel_config(enc(cache_dir), enc(arch)))


def user_kernel_stats():
    """(compiler runs, code objects found on disk, found in memory) since the library was loaded."""
    v = [C.c_longlong(0) for _ in range(3)]
    lib().chn_user_kernel_stats(*[C.byref(x) for x in v])
    return tuple(int(x.value) for x in v)


_TORCH_OF = {F32: torch.float32, BF16: torch.bfloat16, I32: torch.int32, I64: torch.int64}
_CONCRETE = {"float32": F32, "bfloat16": BF16, "int32": I32, "int64": I64}


class _UserKernel:
    """Owner of a chn_user_kernel handle.  Arguments of a call: arrays (tensors or descriptors) and
    Python numbers for scalar parameters, inputs first, then optionally the outputs; outputs that
    are left out are allocated (shape from broadcasting, dtype from the declaration or from the
    arrays that bind the output's type parameter)."""

    def __init__(self, handle, in_params, out_params, name):
        self._h = handle
        self.name = name
        split = lambda text: [tuple(item.split()) for item in text.split(",") if item.strip()]
        self.in_params, self.out_params = split(in_params), split(out_params)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h is not None and _lib is not None:
            _lib.chn_user_kernel_destroy(h)

    def _split(self, args):
        n_in, n_out = len(self.in_params), len(self.out_params)
        if len(args) not in (n_in, n_in + n_out):
            raise TypeError("%s takes %d inputs (and optionally %d outputs), got %d arguments"
                            % (self.name, n_in, n_out, len(args)))
        ins = list(args[:n_in])
        scalars = [float(a) for a in ins if isinstance(a, (int, float))]
        arrays = [None if isinstance(a, (int, float)) else a for a in ins]
        return arrays, scalars, list(args[n_in:])

    def _out_dtype(self, j, arrays):
        t = self.out_params[j][0]
        if t in _CONCRETE:
            return _TORCH_OF[_CONCRETE[t]]
        for (pt, _), a in zip(self.in_params, arrays):
            if pt == t and a is not None:
                return a.dtype
        raise TypeError("%s: no input binds the type parameter %s of output %s" % (self.name, t, self.out_params[j][1]))

    @staticmethod
    def _marshal(arrays, scalars):
        ds = [desc(a) for a in arrays]
        sc = (C.c_double * max(1, len(scalars)))(*scalars)
        return ds, sc

    def source(self, *args, axis=None, keepdims=False):
        """Generated source of the specialisation this call would use (outputs must be given)."""
        arrays, scalars, outs = self._split(args)
        ds, _ = self._marshal(arrays, scalars)
        os_ = [desc(o) for o in outs]
        need = C.c_size_t(0)
        ax = _axis_code(axis, max((a.ndim if isinstance(a, ChnArray) else a.dim()) for a in arrays if a is not None))
        _check(lib().chn_user_kernel_source(self._h, len(ds), _ptrs(ds), len(os_), _ptrs(os_), ax, int(keepdims), None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value)
        _check(lib().chn_user_kernel_source(self._h, len(ds), _ptrs(ds), len(os_), _ptrs(os_), ax, int(keepdims), buf, need.value, None))
        return buf.value.decode()


class ElementwiseKernel(_UserKernel):
    """``kernel = ElementwiseKernel('float32 x, float32 y, float32 z', 'float32 w', 'w = x * y + z',
    'my_mad'); w = kernel(x, y, z)`` -- the figure "Example of a user-defined kernel"."""

    def __init__(self, in_params, out_params, operation, name="kernel", preamble=""):
        h = C.c_void_p(None)
        _check(lib().chn_elementwise_kernel_create(in_params.encode(), out_params.encode(), operation.encode(),
                                                   name.encode(), preamble.encode(), C.byref(h)))
        super().__init__(h, in_params, out_params, name)

    def _outputs(self, arrays, outs):
        if outs:
            return outs
        shape = torch.broadcast_shapes(*[tuple(a.shape) for a in arrays if a is not None])
        dev = next(a.device for a in arrays if a is not None)
        return [torch.empty(shape, dtype=self._out_dtype(j, arrays), device=dev) for j in range(len(self.out_params))]

    def prepare(self, *args):
        arrays, scalars, outs = self._split(args)
        ds, _ = self._marshal(arrays, scalars)
        os_ = [desc(o) for o in self._outputs(arrays, outs)]
        _check(lib().chn_elementwise_kernel_prepare(self._h, len(ds), _ptrs(ds), len(os_), _ptrs(os_)))

    def __call__(self, *args, stream=None):
        arrays, scalars, outs = self._split(args)
        outs = self._outputs(arrays, outs)
        ds, sc = self._marshal(arrays, scalars)
        os_ = [desc(o) for o in outs]
        _check(lib().chn_elementwise_kernel_launch(self._h, len(ds), _ptrs(ds), len(os_), _ptrs(os_), sc,
                                                   _stream() if stream is None else stream))
        return outs[0] if len(outs) == 1 else tuple(outs)


class ReductionKernel(_UserKernel):
    """``ReductionKernel('T x', 'T y', 'x * x', 'a + b', 'y = sqrt(a)', '0', 'l2norm')(x, axis=1)``:
    fold map_expr of every element by reduce_expr from `identity`, then post_map_expr."""

    def __init__(self, in_params, out_params, map_expr, reduce_expr, post_map_expr, identity, name="reduce", preamble=""):
        h = C.c_void_p(None)
        _check(lib().chn_reduction_kernel_create(in_params.encode(), out_params.encode(), map_expr.encode(),
                                                 reduce_expr.encode(), post_map_expr.encode(), str(identity).encode(),
                                                 name.encode(), preamble.encode(), C.byref(h)))
        super().__init__(h, in_params, out_params, name)

    def _outputs(self, arrays, outs, axis, keepdims):
        if outs:
            return outs
        shape = list(torch.broadcast_shapes(*[tuple(a.shape) for a in arrays if a is not None]))
        axes = range(len(shape)) if axis is None else [a % len(shape) for a in (axis if isinstance(axis, (tuple, list)) else [axis])]
        oshape = [1 if d in axes else n for d, n in enumerate(shape)] if keepdims else [n for d, n in enumerate(shape) if d not in axes]
        dev = next(a.device for a in arrays if a is not None)
        return [torch.empty(oshape, dtype=self._out_dtype(j, arrays), device=dev) for j in range(len(self.out_params))]

    @staticmethod
    def _ndim(arrays):
        return max((a.ndim if isinstance(a, ChnArray) else a.dim()) for a in arrays if a is not None)

    def prepare(self, *args, axis=None, keepdims=False):
        arrays, scalars, outs = self._split(args)
        ds, _ = self._marshal(arrays, scalars)
        os_ = [desc(o) for o in self._outputs(arrays, outs, axis, keepdims)]
        _check(lib().chn_reduction_kernel_prepare(self._h, len(ds), _ptrs(ds), len(os_), _ptrs(os_),
                                                  _axis_code(axis, self._ndim(arrays)), int(keepdims)))

    def __call__(self, *args, axis=None, keepdims=False, ws=None, stream=None):
        arrays, scalars, outs = self._split(args)
        outs = self._outputs(arrays, outs, axis, keepdims)
        ds, sc = self._marshal(arrays, scalars)
        os_ = [desc(o) for o in outs]
        ax = _axis_code(axis, self._ndim(arrays))
        if ws is None:
            need = lib().chn_reduction_kernel_workspace_bytes(self._h, len(ds), _ptrs(ds), len(os_), _ptrs(os_), ax, int(keepdims))
            if need:
                ws = torch.empty(need, dtype=torch.uint8, device=outs[0].device)
        p, n = _ws(ws)
        _check(lib().chn_reduction_kernel_launch(self._h, len(ds), _ptrs(ds), len(os_), _ptrs(os_), sc, ax, int(keepdims),
                                                 p, n, _stream() if stream is None else stream))
        return outs[0] if len(outs) == 1 else tuple(outs)
