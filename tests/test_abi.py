"""CPU-side checks of the C ABI: the built library loads, exports every symbol the header declares,
and rejects malformed descriptors on the host before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_1908_00213_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 4096  # fake, aligned, non-NULL device address: validation never dereferences it


def _call_ew(op, ins, out, scalars=None):
    sc = None if scalars is None else (C.c_float * len(scalars))(*scalars)
    return B.lib().chn_elementwise_broadcast(op, len(ins), B._ptrs(ins), C.byref(out), sc,
                                             0 if scalars is None else len(scalars), None)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "chn.h")).read()
    declared = set(re.findall(r"\b(chn_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert L.chn_version() >= 100
    assert L.chn_status_string(0) == b"ok" and L.chn_status_string(-4) == b"shape mismatch"


def test_elementwise_validation():
    f = lambda shape, strides, dt=B.F32, p=P: B.raw_desc(p, shape, strides, dt)
    a = f((4, 5), (20, 4))
    assert _call_ew(B.OP["add"], [a, f((4, 3), (12, 4))], a) == -4            # not broadcastable
    assert b"length 3" in B.lib().chn_last_error()
    assert _call_ew(B.OP["add"], [a], a) == -6                               # wrong arity
    assert _call_ew(99, [a], a) == -6
    assert _call_ew(B.OP["add"], [a, f((4, 5), (20, 4), B.BF16)], a) == -3    # mixed input dtypes
    assert _call_ew(B.OP["add"], [a, a], f((4, 5), (20, 4), B.I32)) == -3
    assert _call_ew(B.OP["add"], [a, a], f((4, 5), (0, 4))) == -5             # zero stride on output
    assert _call_ew(B.OP["add"], [a, f((4, 5), (-20, 4))], a) == -5           # negative stride
    assert _call_ew(B.OP["add"], [a, f((4, 5), (20, 2))], a) == -5            # stride not multiple of item
    assert _call_ew(B.OP["add"], [a, f((4, 5), (20, 4), p=0)], a) == -1       # NULL data
    assert _call_ew(B.OP["scale"], [a], a) == -6                             # missing scalar
    bad = f((4, 5), (20, 4)); bad.ndim = 9
    assert _call_ew(B.OP["copy"], [bad], a) == -2
    assert _call_ew(B.OP["copy"], [f((2, 4, 5), (80, 20, 4))], a) == -4       # input has more dims than out
    # zero-size arrays are fine and launch nothing
    z = f((0, 5), (20, 4))
    assert _call_ew(B.OP["add"], [z, z], z) == 0


def test_elementwise_plan_families():
    L = B.lib()
    f = lambda shape, strides, dt=B.F32: B.raw_desc(P, shape, strides, dt)
    plan = lambda op, ins, out: L.chn_elementwise_plan(B.OP[op], len(ins), B._ptrs(ins), C.byref(out))
    n = 64
    full = f((n, n), (4 * n, 4))
    assert plan("mad_relu", [full, full, f((1, n), (4 * n, 4))], full) == 0      # contiguous + row broadcast
    assert plan("add", [full, f((n,), (4,))], full) == 0                         # bias
    assert plan("add", [full, f((), ())], full) == 0                             # scalar
    assert plan("add", [full, f((n, 1), (4, 4))], full) == 1                     # column broadcast
    assert plan("add", [f((n, n), (8 * n, 4)), full], full) == 1                 # pitched rows
    assert plan("mad_relu", [f((n, n), (4, 4 * n)), full, f((1, n), (4 * n, 4))], full) == 2   # transposed a
    assert plan("copy", [f((n, n), (8 * n, 8))], full) == 3                      # inner stride 2
    # 4-d contiguous collapses to flat; permuted collapses to a 2-d transpose
    c4 = f((2, 3, 4, 8), (384, 128, 32, 4))
    assert plan("relu", [c4], c4) == 0
    assert plan("relu", [f((6, 32), (4, 24))], f((6, 32), (128, 4))) == 2
    # misaligned base pointer cannot use 16-byte vectors
    mis = B.raw_desc(P + 4, (n, n), (4 * n, 4), B.F32)
    assert plan("relu", [mis], full) == 1


def test_reduce_gemm_and_layer_validation():
    L = B.lib()
    f = lambda shape, strides, dt=B.F32, p=P: B.raw_desc(p, shape, strides, dt)
    x = f((8, 16), (64, 4))
    r = lambda op, a, ax, keep, out: L.chn_reduce_axis(op, C.byref(a), ax, keep, C.byref(out), None, 0, None)
    assert r(0, x, 2, 0, f((8,), (4,))) == -7
    assert r(0, x, -3, 0, f((8,), (4,))) == -7
    assert r(0, x, 1, 0, f((16,), (4,))) == -4
    assert r(0, x, 1, 1, f((8,), (4,))) == -4
    assert r(7, x, 1, 0, f((8,), (4,))) == -6
    assert r(0, x, 1, 0, f((8,), (8,))) == -5                 # out must be contiguous
    big = f((8192, 8192), (4 * 8192, 4))
    need = L.chn_reduce_axis_workspace_bytes(C.byref(big), 0)
    assert need > 0 and L.chn_reduce_axis_workspace_bytes(C.byref(big), 1) == 0
    assert r(0, big, 0, 0, f((8192,), (4,))) == -8            # workspace required but missing
    g = lambda A, Bm, Cm, epi=0, bias=None, aux=None, pre=None: L.chn_gemm(
        C.byref(A), C.byref(Bm), C.byref(Cm), 1.0, 0.0, epi, None if bias is None else C.byref(bias),
        None if aux is None else C.byref(aux), None if pre is None else C.byref(pre), None, 0, None)
    A, Bm, Cm = f((8, 16), (64, 4)), f((16, 4), (16, 4)), f((8, 4), (16, 4))
    assert g(A, f((15, 4), (16, 4)), Cm) == -4
    assert g(A, Bm, f((8, 5), (20, 4))) == -4
    assert g(A, f((16, 4), (16, 4), B.BF16), Cm) == -3
    assert g(A, Bm, f((8, 4), (8, 2), B.BF16)) == -3          # fp32 operands need an fp32 C
    assert g(f((8, 16), (128, 8)), Bm, Cm) == -5              # no unit-stride dimension
    assert g(A, Bm, f((8, 4), (4, 32))) == -5                 # C must be row-major
    assert g(A, Bm, Cm, 1) == -1                              # bias epilogue without bias
    assert g(A, Bm, Cm, 1, f((5,), (4,))) == -4
    assert g(A, Bm, Cm, 4) == -1                              # aux missing
    assert g(A, Bm, Cm, 0, None, None, Cm) == -6              # preact_out without BIAS_GELU
    assert g(A, Bm, Cm, 17) == -6
    # row-block column sums beside an activation gradient: shapes in whole 256 x 256 tiles only
    A2, B2, C2 = f((512, 64), (256, 4)), f((64, 256), (1024, 4)), f((512, 256), (1024, 4))
    assert g(A, Bm, Cm, 4, None, Cm, f((1, 4), (16, 4))) == -4              # M, N not multiples of 256
    assert g(A2, B2, C2, 4, None, C2, f((3, 256), (1024, 4))) == -4          # one row per 128 rows of C
    assert g(A2, B2, C2, 5, None, C2, f((4, 256), (512, 2), B.BF16)) == -3   # the sums are fp32
    assert g(A2, B2, C2, 4, None, C2, f((4, 256), (1028, 4))) == -5          # rows off the 16-byte grid
    z, c = f((4, 32), (128, 4)), f((4, 8), (32, 4))
    assert L.chn_lstm_fwd(C.byref(f((4, 31), (124, 4))), None, C.byref(c), C.byref(c), C.byref(c), None, None) == -4
    assert L.chn_lstm_fwd(C.byref(z), C.byref(f((31,), (4,))), C.byref(c), C.byref(c), C.byref(c), None, None) == -4
    lab = f((4,), (4,), B.I32)
    one = f((), (), B.F32)
    assert L.chn_softmax_ce_fwd(C.byref(c), C.byref(f((5,), (4,), B.I32)), -1, C.byref(one), None, None, None, 0, None) == -4
    assert L.chn_softmax_ce_fwd(C.byref(c), C.byref(f((4,), (4,), B.F32)), -1, C.byref(one), None, None, None, 0, None) == -3
    assert L.chn_softmax_ce_fwd(C.byref(c), C.byref(lab), -1, C.byref(one), None, None, None, 0, None) == -8
    assert L.chn_softmax_ce_workspace_bytes(1000) >= 4256
    fb = lambda z, t, d: L.chn_softmax_ce_fwd_bwd(C.byref(z), C.byref(t), -1, C.byref(one), None, 1.0, C.byref(d), None, 0, None)
    big, blab = f((100, 1000), (4000, 4)), f((100,), (4,), B.I32)
    assert fb(c, f((5,), (4,), B.I32), c) == -4                               # one label per row
    assert fb(c, lab, f((4, 9), (36, 4))) == -4                               # the gradient has the logits' shape
    assert fb(c, lab, f((4, 8), (32, 4), B.I32)) == -3
    assert fb(big, blab, big) == -8                                           # many classes: workspace required
    assert L.chn_sgd_update(C.byref(c), C.byref(z), 0.1, None, None) == -4
    assert L.chn_sgd_update(C.byref(c), C.byref(f((4, 8), (64, 4))), 0.1, None, None) == -5
    assert L.chn_sgd_update(C.byref(c), C.byref(c), 0.1, C.byref(c), None) == -3
    assert L.chn_embed_fwd(C.byref(c), C.byref(f((3,), (4,), B.F32)), C.byref(f((3, 8), (32, 4))), None) == -3
    assert L.chn_embed_fwd(C.byref(c), C.byref(f((3,), (4,), B.I32)), C.byref(f((3, 7), (28, 4))), None) == -4


def test_gemm_plan_picks_the_direct_copy_kernel_only_where_it_applies():
    L = B.lib()
    d = lambda shape, strides, dt: B.raw_desc(P, shape, strides, dt)
    def plan(M, N, K, dt, a_t=False, b_t=True, ws=0, pad_k=0):
        isz = 2 if dt == B.BF16 else 4
        A = d((M, K), (isz, isz * M) if a_t else (isz * (K + pad_k), isz), dt)
        Bm = d((K, N), (isz, isz * (K + pad_k)) if b_t else (isz * N, isz), dt)
        Cm = d((M, N), (4 * N, 4), B.F32)
        code = L.chn_gemm_plan(C.byref(A), C.byref(Bm), C.byref(Cm), ws)
        assert code >= 0, B.lib().chn_last_error()
        return code & 3, bool(code & 4), code >> 4
    assert plan(8192, 4096, 4096, B.BF16) == (2, True, 1)                 # x @ W.T
    assert plan(8192, 4096, 4096, B.BF16, b_t=False) == (2, True, 1)      # dY @ W
    assert plan(4096, 4096, 8192, B.BF16, a_t=True, b_t=False) == (2, True, 1)   # dY.T @ X
    assert plan(8192, 4096, 1000, B.BF16, b_t=False) == (2, True, 1)      # ragged last K step
    assert plan(8192, 4096, 4096, B.F32) == (2, True, 1)
    assert plan(4096, 4096, 8192, B.F32, a_t=True, b_t=False)[:2] == (2, False)  # fp32, no K-contiguous operand
    assert plan(4480, 10000, 650, B.F32)[:2] == (2, False)                # rows of 2600 bytes: 8-byte pieces only
    assert plan(8192, 4096, 4098, B.BF16)[1] is False                     # K not a multiple of 8 elements
    assert plan(64, 64, 64, B.BF16) == (0, False, 1)
    tile, dc, splits = plan(1000, 4096, 8192, B.BF16, a_t=True, b_t=False, ws=1)
    assert (tile, dc) == (2, True) and splits > 1                         # few tiles, long K: split
    assert plan(1000, 4096, 8192, B.BF16, a_t=True, b_t=False, ws=0)[2] == 1


def test_later_entry_points_validate_on_the_host():
    """Adam, arg-max and the fused recurrent step reject malformed calls before anything is launched."""
    L = B.lib()
    f = lambda shape, dt=B.F32, p=P, strides=None: B.raw_desc(
        p, shape, strides or [int(s) for s in _row_major(shape, {B.F32: 4, B.BF16: 2, B.I32: 4, B.I64: 8}[dt])], dt)
    r = C.byref
    # Adam
    p_, g_, m_, v_ = f((8, 8)), f((8, 8)), f((8, 8)), f((8, 8))
    adam = lambda ps, gs, ms, vs, step, b1=0.9: L.chn_adam_update_multi(
        len(ps), B._ptrs(ps), B._ptrs(gs), B._ptrs(ms), B._ptrs(vs), 0.001, b1, 0.999, 1e-8, step, None, None)
    assert adam([p_], [g_], [m_], [f((8, 7))], 1) == -4                       # state of another shape
    assert adam([p_], [g_], [m_], [v_], 0) == -6                              # steps count from 1
    assert adam([p_], [g_], [m_], [v_], 1, b1=1.0) == -6                      # beta outside [0, 1)
    assert adam([p_], [f((8, 8), B.BF16)], [m_], [v_], 1) == -3
    assert adam([], [], [], [], 1) == 0
    # arg-max
    x = f((6, 10))
    am = lambda a, axis, out, keep=0: L.chn_argmax_axis(r(a), axis, keep, r(out), None)
    assert am(x, 1, f((6,), B.F32)) == -3                                     # indices are integers
    assert am(x, 1, f((10,), B.I64)) == -4
    assert am(x, 2, f((6,), B.I64)) == -7
    assert am(f((6, 0)), 1, f((6,), B.I64)) == -4                             # nothing to choose from
    assert am(f((0, 10)), 1, f((0,), B.I64)) == 0
    # fused recurrent step
    Bn, H = 4, 64
    zx, hp, Ut, c = f((Bn, 4 * H)), f((Bn, H)), f((4 * H, H)), f((Bn, H))
    fwd = lambda zx, hp, Ut, c_prev, c, h: L.chn_lstm_step_fwd(r(zx), r(hp), r(Ut), None, r(c_prev), r(c), r(h), None, None)
    assert fwd(zx, hp, f((H, 4 * H)), c, c, hp) == -4                         # U instead of its transpose
    assert fwd(zx, f((Bn, H), B.BF16), Ut, c, c, hp) == -3                    # operands of two dtypes
    assert fwd(zx, f((Bn, H), p=P + 4), Ut, c, c, hp) == -5                   # rows off the 16-byte grid
    assert fwd(f((Bn, 160)), f((Bn, 40)), f((160, 40)), f((Bn, 40)), f((Bn, 40)), f((Bn, 40))) == -4   # H not a multiple of 32
    assert b"multiple of 32" in L.chn_last_error()
    bwd = lambda dzn, U, dh, dz: L.chn_lstm_step_bwd(r(dzn), r(U), r(dh), r(zx), r(c), r(c), None, r(dz), r(c), None)
    assert bwd(zx, f((H, 4 * H)), hp, f((Bn, 4 * H), B.BF16)) == -3           # dz must have dh's dtype
    assert bwd(zx, f((4 * H, H)), hp, zx) == -4                               # the transpose where U is expected


def test_whole_sequence_entry_points_validate_on_the_host():
    """What the whole-sequence recurrent kernels refuse before they ask the device anything."""
    L = B.lib()
    f = lambda shape, dt=B.F32, p=P: B.raw_desc(p, shape, [int(s) for s in _row_major(shape, {B.F32: 4, B.BF16: 2, B.I32: 4}[dt])], dt)
    r = C.byref
    Bn, H, T = 4, 64, 3
    zx, Ut, Hs, Cs = f((T * Bn, 4 * H)), f((4 * H, H)), f(((T + 1) * Bn, H)), f(((T + 1) * Bn, H))
    fwd = lambda zx, Ut, Hs, Cs, T_=T, ws=P, n=1 << 20: L.chn_lstm_seq_fwd(r(zx), r(Ut), None, r(Hs), r(Cs), None, T_, ws, n, None)
    assert L.chn_lstm_seq_fwd(r(zx), r(Ut), None, None, r(Cs), None, T, P, 1 << 20, None) == -1            # Hs missing
    assert fwd(zx, Ut, Hs, f((2, 2, 2))) == -2                                    # Cs must be 2-d
    assert fwd(zx, Ut, Hs, Cs, T_=4) == -4                                        # 16 rows do not hold 4 + 1 blocks
    assert fwd(zx, Ut, Hs, Cs, T_=-1) == -4
    assert fwd(f((T * Bn, 176)), f((176, 44)), f(((T + 1) * Bn, 44)), f(((T + 1) * Bn, 44))) == -4   # H not a multiple of 8
    assert b"multiple of 8" in L.chn_last_error()
    assert fwd(zx, Ut, f(((T + 1) * Bn, H), B.I32), Cs) == -3                     # h must be F32 or BF16
    assert L.chn_lstm_seq_workspace_bytes(0) == 0 and L.chn_lstm_seq_workspace_bytes(130) >= 256 + 3 * 4
    assert L.chn_lstm_seq_supported(128, 44, B.F32) == -4 and L.chn_lstm_seq_supported(128, 776, B.F32) == -4
    assert L.chn_lstm_seq_supported(128, 776, B.BF16) == -4                       # 776 is not a multiple of 16
    U, dHs, G, dZ, dc0 = f((H, 4 * H)), f((T * Bn, H)), f((T * Bn, 4 * H)), f((T * Bn, 4 * H)), f((Bn, H))
    bwd = lambda U, dHs, G, Cs, dZ, dc0, T_=T: L.chn_lstm_seq_bwd(r(U), r(dHs), r(G), r(Cs), None, r(dZ), r(dc0), T_, P, 1 << 30, None)
    assert L.chn_lstm_seq_bwd(None, r(dHs), r(G), r(Cs), None, r(dZ), r(dc0), T, P, 1 << 30, None) == -1   # U missing
    assert bwd(U, dHs, G, Cs, dZ, dc0, T_=4) == -4
    assert bwd(f((40, 160)), f((T * Bn, 40)), f((T * Bn, 160)), f(((T + 1) * Bn, 40)), f((T * Bn, 160)), f((Bn, 40))) == -4   # H not a multiple of 16
    assert b"multiple of 16" in L.chn_last_error()
    assert L.chn_lstm_seq_bwd_supported(128, 784, B.F32) == -4 and L.chn_lstm_seq_bwd_supported(128, 1552, B.BF16) == -4   # wider than the registers hold
    assert L.chn_lstm_seq_bwd_workspace_bytes(128, 672) == 256 + 256 + 2 * 4 * 42 * 42 * 2048
    L.chn_lstm_seq_spin_limit(1 << 20)


def _row_major(shape, isz):
    out, acc = [], isz
    for n in reversed(shape):
        out.insert(0, acc)
        acc *= max(n, 1)
    return out


def test_benchmark_refuses_what_it_cannot_measure():
    """bench.py measures one GPU: more are refused with a message (no collectives in this build), and
    without a GPU it exits with an error instead of timing anything on the host."""
    import os
    import subprocess
    import sys
    import torch
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--quick", "--no-cpu"], capture_output=True, text=True, timeout=300)
        assert r.returncode == 3 and "no GPU" in r.stderr and r.stdout.strip() == ""
