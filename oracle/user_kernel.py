"""CPU oracle for user-defined kernels (TEST INFRASTRUCTURE, not product code).

Section "Custom CUDA Kernels": an element-wise kernel applies a user's snippet to every element; a
reduction kernel folds the mapped elements by a binary operator; a parameter whose type is a type
parameter takes whatever dtype the call's arrays have.  Here the definition is written out as the
plainest possible program: the snippet is pasted into a sequential C++ loop over the broadcast
operands, compiled with g++ and run on the host.  Floating-point parameters are ``double`` (the
oracle computes in float64), int32 is ``int`` and int64 is ``long long`` (integer results must
agree bit for bit, so the integer types are the declared ones).  The reduction folds the elements
of each result strictly in index order, starting from the identity.

Nothing here shares code with the GPU library or its Python binding.  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import this module.
"""
import ctypes as C
import hashlib
import os
import subprocess
import tempfile

import numpy as np

_FLOAT_NAMES = ("float32", "bfloat16")
_INT_NAMES = {"int32": ("int", np.int32), "int64": ("long long", np.int64)}
_dir = None
_libs = {}

_HEADER = """
#include <cmath>
#include <algorithm>
#include <cstdint>
using namespace std;
#define __device__
#define __forceinline__ inline
"""


def _parse(text):
    out = []
    for item in text.split(","):
        if item.strip():
            t, n = item.split()
            out.append((t, n))
    return out


def _compile(src):
    global _dir
    key = hashlib.sha1(src.encode()).hexdigest()
    if key in _libs:
        return _libs[key]
    if _dir is None:
        _dir = tempfile.mkdtemp(prefix="chn_oracle_uk_")
    cpp, so = os.path.join(_dir, key + ".cpp"), os.path.join(_dir, key + ".so")
    with open(cpp, "w") as f:
        f.write(src)
    r = subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-o", so, cpp], capture_output=True, text=True)
    if r.returncode != 0:
        raise ValueError("oracle: the snippet does not compile:\n" + r.stderr)
    _libs[key] = C.CDLL(so)
    return _libs[key]


def _cscalar(ct, v):
    if ct == "double":
        return C.c_double(float(v))
    return C.c_int(int(v)) if ct == "int" else C.c_longlong(int(v))


def _ctype_of(dtype):
    """(C type in the loop, NumPy dtype of the buffer handed to it) for an array's dtype."""
    if np.issubdtype(dtype, np.integer):
        return ("int", np.int32) if np.dtype(dtype).itemsize == 4 else ("long long", np.int64)
    return ("double", np.float64)


class _Kernel:
    def __init__(self, in_params, out_params, preamble):
        self.inp, self.outp, self.preamble = _parse(in_params), _parse(out_params), preamble

    def _bind(self, args):
        """C type and buffer dtype of every parameter for this call; scalars keep their value."""
        if len(args) != len(self.inp):
            raise TypeError("expected %d inputs" % len(self.inp))
        generic, types = {}, []
        for (t, _), a in zip(self.inp, args):
            if t in _FLOAT_NAMES:
                types.append(("double", np.float64))
            elif t in _INT_NAMES:
                types.append(_INT_NAMES[t])
            else:
                if not np.isscalar(a):
                    got = _ctype_of(np.asarray(a).dtype)
                    if generic.setdefault(t, got) != got:
                        raise TypeError("type parameter %s bound twice" % t)
                types.append(t)
        types = [generic[t] if isinstance(t, str) else t for t in types]
        otypes = []
        for t, _ in self.outp:
            otypes.append(("double", np.float64) if t in _FLOAT_NAMES else _INT_NAMES[t] if t in _INT_NAMES else generic[t])
        tdefs = "".join("typedef %s %s;\n" % (c, t) for t, (c, _) in generic.items())
        return types, otypes, tdefs


class ElementwiseKernel(_Kernel):
    """``ElementwiseKernel('float32 x, float32 y, float32 z', 'float32 w', 'w = x * y + z')(x, y, z)``:
    the operation applied to every element of the broadcast inputs (figure "Example of a
    user-defined kernel")."""

    def __init__(self, in_params, out_params, operation, name="kernel", preamble=""):
        super().__init__(in_params, out_params, preamble)
        self.operation = operation

    def __call__(self, *args):
        types, otypes, tdefs = self._bind(args)
        arrays = [None if np.isscalar(a) else np.asarray(a) for a in args]
        shape = np.broadcast_shapes(*[a.shape for a in arrays if a is not None])
        n = int(np.prod(shape, dtype=np.int64))
        sig, load, bufs = [], [], []
        for (_, name), (ct, npd), a, v in zip(self.inp, types, arrays, args):
            if a is None:
                sig.append("const %s %s" % (ct, name))
                bufs.append(_cscalar(ct, v))
            else:
                sig.append("const %s *%s_" % (ct, name))
                load.append("const %s %s = %s_[i];" % (ct, name, name))
                bufs.append(np.ascontiguousarray(np.broadcast_to(a, shape), dtype=npd))
        outs = [np.zeros(shape, dtype=npd) for _, npd in otypes]
        for (_, name), (ct, _) in zip(self.outp, otypes):
            sig.append("%s *%s_" % (ct, name))
        src = _HEADER + self.preamble + "\n" + tdefs + 'extern "C" void run(long long n, %s) {\n' % ", ".join(sig)
        src += "  for (long long i = 0; i < n; ++i) {\n    " + "\n    ".join(load) + "\n"
        src += "".join("    %s %s = 0;\n" % (ct, name) for (_, name), (ct, _) in zip(self.outp, otypes))
        src += "    { " + self.operation + "; }\n"
        src += "".join("    %s_[i] = %s;\n" % (name, name) for _, name in self.outp) + "  }\n}\n"
        fn = _compile(src).run
        fn.restype = None
        cargs = [b.ctypes.data_as(C.c_void_p) if isinstance(b, np.ndarray) else b for b in bufs]
        cargs += [o.ctypes.data_as(C.c_void_p) for o in outs]
        fn(C.c_longlong(n), *cargs)
        return outs[0] if len(outs) == 1 else tuple(outs)


class ReductionKernel(_Kernel):
    """Fold ``map_expr`` of every element by ``reduce_expr`` (over ``a`` and ``b``) from ``identity``
    in index order, then ``post_map_expr`` assigns the outputs from the folded value ``a``.  The fold
    runs in the type of the first output; ``axis`` is one axis, a tuple of axes, or None for all."""

    def __init__(self, in_params, out_params, map_expr, reduce_expr, post_map_expr, identity, name="reduce", preamble=""):
        super().__init__(in_params, out_params, preamble)
        self.map_expr, self.reduce_expr, self.post, self.identity = map_expr, reduce_expr, post_map_expr, str(identity)

    def __call__(self, *args, axis=None, keepdims=False):
        types, otypes, tdefs = self._bind(args)
        arrays = [None if np.isscalar(a) else np.asarray(a) for a in args]
        shape = np.broadcast_shapes(*[a.shape for a in arrays if a is not None])
        nd = len(shape)
        axes = tuple(range(nd)) if axis is None else tuple(sorted(a % nd for a in (axis if isinstance(axis, (tuple, list)) else (axis,))))
        kept = [d for d in range(nd) if d not in axes]
        n_res = int(np.prod([shape[d] for d in kept], dtype=np.int64))
        R = int(np.prod([shape[d] for d in axes], dtype=np.int64))
        oshape = tuple(1 if d in axes else shape[d] for d in range(nd)) if keepdims else tuple(shape[d] for d in kept)
        rt = otypes[0][0]
        sig, load, bufs, scal = [], [], [], []
        for (_, name), (ct, npd), a, v in zip(self.inp, types, arrays, args):
            if a is None:
                sig.append("const %s %s" % (ct, name))
                bufs.append(_cscalar(ct, v))
            else:
                sig.append("const %s *%s_" % (ct, name))
                load.append("const %s %s = %s_[i];" % (ct, name, name))
                full = np.broadcast_to(a, shape).transpose(kept + list(axes)).reshape(n_res, R)
                bufs.append(np.ascontiguousarray(full, dtype=npd))
        outs = [np.zeros((n_res,), dtype=npd) for _, npd in otypes]
        for (_, name), (ct, _) in zip(self.outp, otypes):
            sig.append("%s *%s_" % (ct, name))
        src = _HEADER + self.preamble + "\n" + tdefs + "typedef %s RT_;\n" % rt
        src += "static RT_ fold_(const RT_ a, const RT_ b) { return (RT_)(%s); }\n" % self.reduce_expr
        src += 'extern "C" void run(long long n_res, long long R, %s) {\n' % ", ".join(sig)
        src += "  for (long long res = 0; res < n_res; ++res) {\n    RT_ acc = (RT_)(%s);\n" % self.identity
        src += "    for (long long r = 0; r < R; ++r) {\n      const long long i = res * R + r;\n      " + "\n      ".join(load) + "\n"
        src += "      acc = fold_(acc, (RT_)(%s));\n    }\n" % self.map_expr
        src += "    const RT_ a = acc;\n"
        src += "".join("    %s %s = 0;\n" % (ct, name) for (_, name), (ct, _) in zip(self.outp, otypes))
        src += "    { " + self.post + "; }\n"
        src += "".join("    %s_[res] = %s;\n" % (name, name) for _, name in self.outp) + "  }\n}\n"
        fn = _compile(src).run
        fn.restype = None
        cargs = [b.ctypes.data_as(C.c_void_p) if isinstance(b, np.ndarray) else b for b in bufs]
        cargs += [o.ctypes.data_as(C.c_void_p) for o in outs]
        fn(C.c_longlong(n_res), C.c_longlong(R), *cargs)
        outs = [o.reshape(oshape) for o in outs]
        return outs[0] if len(outs) == 1 else tuple(outs)
