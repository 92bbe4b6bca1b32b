"""chn_reduce_axis_static -- the entry point for callers that cannot allocate -- against chn_reduce_axis
and the oracle, through the C ABI, on calls that share the GPU's one built-in array."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_1908_00213_amd import binding as B
from util import TOL_BF16, TOL_SUM, check, dev, empty, host, ws

pytestmark = pytest.mark.gpu
RNG = np.random.default_rng(190800213 + 77)


def _both(op, x, d, axis, keepdims=False):
    """(static-scratch result, workspace result) of one reduction, called through the raw C ABI."""
    L = B.lib()
    shape = list(d.shape)
    ax = axis % len(shape)
    oshape = [1 if i == ax else n for i, n in enumerate(shape)] if keepdims else [n for i, n in enumerate(shape) if i != ax]
    need = L.chn_reduce_axis_workspace_bytes(C.byref(B.desc(d)), axis)
    w = ws(need)
    w.fill_(0x7f)
    a, b = empty(oshape), empty(oshape)
    st = B._stream()
    B._check(L.chn_reduce_axis_static(B.REDUCE[op], C.byref(B.desc(d)), axis, int(keepdims), C.byref(B.desc(a)), st))
    B._check(L.chn_reduce_axis(B.REDUCE[op], C.byref(B.desc(d)), axis, int(keepdims), C.byref(B.desc(b)),
                               C.c_void_p(w.data_ptr()), w.numel(), st))
    torch.cuda.synchronize()
    return a, b, need


def test_static_scratch_matches_workspace_call_on_consecutive_calls():
    # first a large sliced column reduction, then smaller ones that find its partial sums in the array
    # (stacks of at most 2048 rows that fit the caches take one launch and no partial sums: the last three)
    cases = [("f32", (3000, 4104), 0), ("f32", (2100, 700), 0), ("bf16", (2055, 2048), 0), ("f32", (2, 2100, 520), 1),
             ("f32", (1100, 700), 0), ("f32", (300, 64), 0), ("f32", (513, 1000), 1)]
    sliced = 0
    for dt, shape, axis in cases:
        x = RNG.uniform(-1, 1, size=shape).astype(np.float32)
        if dt == "bf16":
            from util import bf16r
            x = bf16r(x)
        d = dev(x, dt)
        for op in ("sum", "max"):
            a, b, need = _both(op, x, d, axis)
            sliced += need > 0
            assert torch.equal(a, b), (dt, shape, axis, op)            # same kernels, same order: same bits
            ref = O.reduce_axis(op, x, axis)
            if op == "max":
                assert np.array_equal(host(a), ref)
            else:
                check(host(a), ref, TOL_BF16 if dt == "bf16" else TOL_SUM, O.reduce_axis("sum", np.abs(x), axis), "static %s %s" % (dt, shape))
    assert sliced >= 8                                                 # the array was really in use
    # exact integers: bit-equal to the oracle whatever the previous call left behind
    xi = RNG.integers(-4, 5, size=(2050, 1500)).astype(np.float32)
    a, b, need = _both("sum", xi, dev(xi), 0)
    assert need > 0 and np.array_equal(host(a), O.reduce_axis("sum", xi, 0))
    xi2 = xi[:900, :600].copy()
    a, b, _ = _both("sum", xi2, dev(xi2), 0)
    assert np.array_equal(host(a), O.reduce_axis("sum", xi2, 0))


def test_static_scratch_allocates_nothing_and_refuses_what_does_not_fit():
    L = B.lib()
    x = RNG.uniform(-1, 1, size=(2048, 2048)).astype(np.float32)
    d, out = dev(x), empty((2048,))
    B.reduce_axis_static("sum", d, 0, out)                             # first call on the device: address lookup
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for _ in range(20):
        B.reduce_axis_static("sum", d, 0, out)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0                       # no device memory taken by the calls
    check(host(out), O.reduce_axis("sum", x, 0), TOL_SUM, O.reduce_axis("sum", np.abs(x), 0), "static 2048")
    # a reduction whose partial sums exceed the built-in array: refused on the host, nothing launched
    # (descriptor only -- validation never touches the data)
    big = B.raw_desc(d.data_ptr(), (2, 1 << 16, 2044), ((1 << 16) * 2044 * 4, 2044 * 4, 4), B.F32)
    need = L.chn_reduce_axis_workspace_bytes(C.byref(big), 1)
    assert need > (8 << 20)
    o = B.raw_desc(out.data_ptr(), (2, 2044), (2044 * 4, 4), B.F32)
    assert L.chn_reduce_axis_static(0, C.byref(big), 1, 0, C.byref(o), None) == -8
    assert b"built-in" in L.chn_last_error()
