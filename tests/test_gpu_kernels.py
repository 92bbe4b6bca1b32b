"""GPU parity: every C-ABI call against the CPU oracle, element by element, on seeded inputs at sizes
that span several tiles plus a ragged tail, with the edge cases each call has."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_1908_00213_amd import binding as B
from tests.util import TOL_BF16, TOL_EW, TOL_SUM, bf16r, check, dev, empty, host, ws

pytestmark = pytest.mark.gpu
RNG = np.random.default_rng(1908_00213)


def rnd(shape, dt="f32", lo=-1.0, hi=1.0):
    a = RNG.uniform(lo, hi, size=shape).astype(np.float32)
    return bf16r(a) if dt == "bf16" else a


def tol_for(dt_in, dt_out, base):
    return TOL_BF16 if "bf16" in (dt_in, dt_out) else base


# ------------------------------------------------------------------------------------ element-wise
@pytest.mark.parametrize("dt_in,dt_out", [("f32", "f32"), ("bf16", "bf16"), ("f32", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("shape", [(300, 520), (257, 1031), (3, 5), (1, 1)])
def test_mad_relu_row_broadcast(dt_in, dt_out, shape):
    a, b, c = rnd(shape, dt_in), rnd(shape, dt_in), rnd((1, shape[1]), dt_in)
    out = empty(shape, dt_out)
    assert B.elementwise_plan("mad_relu", [dev(a, dt_in), dev(b, dt_in), dev(c, dt_in)], out) == 0
    B.elementwise_broadcast("mad_relu", [dev(a, dt_in), dev(b, dt_in), dev(c, dt_in)], out)
    ref = O.elementwise("mad_relu", [a, b, c])
    S = O.elementwise("mad", [np.abs(a), np.abs(b), np.abs(c)])
    check(host(out), ref, tol_for(dt_in, dt_out, TOL_EW), S, "mad_relu")
    if dt_out == "f32" and dt_in == "f32":
        # fused multiply-add differs from the oracle's fp64 only by the final rounding
        assert np.max(np.abs(host(out) - ref)) <= 2.0 ** -23 * 2


OPS1 = ["copy", "relu", "gelu", "sigmoid", "tanh", "exp"]
OPS2 = ["add", "sub", "mul", "relu_bwd", "gelu_bwd", "add_relu", "add_gelu", "gelu_bwd2"]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_every_op_flat(dt):
    shape = (129, 77)
    x, y, z = rnd(shape, dt, -4, 4), rnd(shape, dt, -4, 4), rnd(shape, dt, -4, 4)
    tol = tol_for(dt, dt, TOL_EW)
    for op in OPS1:
        out = B.elementwise_broadcast(op, [dev(x, dt)], empty(shape, dt))
        S = np.abs(x) if op == "gelu" else None
        check(host(out), O.elementwise(op, [x]), tol, S, op)
    for op in OPS2:
        out = B.elementwise_broadcast(op, [dev(x, dt), dev(y, dt)], empty(shape, dt))
        S = {"add": np.abs(x) + np.abs(y), "sub": np.abs(x) + np.abs(y), "add_relu": np.abs(x) + np.abs(y),
             "add_gelu": np.abs(x) + np.abs(y), "gelu_bwd": np.abs(x) * (1 + np.abs(y)), "gelu_bwd2": np.abs(x)}.get(op)
        check(host(out), O.elementwise(op, [x, y]), tol, S, op)
    out = B.elementwise_broadcast("mad", [dev(x, dt), dev(y, dt), dev(z, dt)], empty(shape, dt))
    check(host(out), O.elementwise("mad", [x, y, z]), tol, np.abs(x * y) + np.abs(z), "mad")
    out = B.elementwise_broadcast("scale", [dev(x, dt)], empty(shape, dt), scalars=[-2.5])
    check(host(out), O.elementwise("scale", [x], scalars=[-2.5]), tol, None, "scale")
    out = B.elementwise_broadcast("axpy", [dev(x, dt), dev(y, dt)], empty(shape, dt), scalars=[0.375])
    check(host(out), O.elementwise("axpy", [x, y], scalars=[0.375]), tol, np.abs(x) + np.abs(y), "axpy")
    out = B.elementwise_broadcast("fill", [], empty(shape, dt), scalars=[1.5])
    assert np.all(host(out) == 1.5)
    xp = np.abs(x)
    out = B.elementwise_broadcast("sqrt", [dev(xp, dt)], empty(shape, dt))
    check(host(out), O.elementwise("sqrt", [xp]), tol, None, "sqrt")


def test_paper_examples_on_gpu():
    # figure "Examples using NumPy and CuPy": the norm of [1, 2]; figure "user-defined kernel": x*y+z
    x = dev(np.array([1.0, 2.0], dtype=np.float32))
    sq = B.elementwise_broadcast("mul", [x, x], empty((2,)))
    s = B.reduce_axis("sum", sq, 0, empty(()))
    assert float(s.cpu()) == 5.0
    n = B.elementwise_broadcast("sqrt", [s], empty(()))
    assert abs(float(n.cpu()) - 5 ** 0.5) < 2e-7
    rows = np.array([[1, 2, 3, 5], [-2, 4, 1, -7], [0.5, 0.25, -0.125, 0], [3, -3, 9, 0], [-1.5, -2, 0.5, 3.5]], dtype=np.float32)
    w = B.elementwise_broadcast("mad", [dev(rows[:, 0].copy()), dev(rows[:, 1].copy()), dev(rows[:, 2].copy())], empty((5,)))
    assert np.array_equal(host(w), rows[:, 3])


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_broadcast_patterns(dt):
    tol = tol_for(dt, dt, TOL_EW)
    cases = [
        [(70, 130), (70, 130), (130,)],          # bias, aligned period? 130 is not a vector multiple
        [(70, 136), (70, 136), (136,)],          # aligned period
        [(70, 10), (70, 10), (10,)],             # period shorter than... a tiny class count
        [(70, 130), (70, 1), (1, 130)],          # column broadcast x row broadcast
        [(6, 1, 50), (1, 7, 1), (7, 50)],        # 3-d mixed
        [(5, 6, 7, 8), (8,), ()],                # scalar operand
        [(33,), (1,), (33,)],
    ]
    for shapes in cases:
        xs = [rnd(s, dt) for s in shapes]
        ref = O.elementwise("mad", xs)
        out = B.elementwise_broadcast("mad", [dev(x, dt) for x in xs], empty(ref.shape, dt))
        S = O.elementwise("mad", [np.abs(x) for x in xs])
        check(host(out), ref, tol, S, str(shapes))


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(200, 330), (64, 64), (65, 63), (1000, 7), (200, 328), (264, 136), (1032, 520), (8, 8)])
def test_transposed_view(dt, shape):
    r, c = shape
    a_store = rnd((c, r), dt)                 # a is the transpose view of a contiguous (c, r) buffer
    b, cc = rnd((r, c), dt), rnd((1, c), dt)
    a_dev = dev(a_store, dt).t()
    assert a_dev.stride() == (1, r)
    out = empty((r, c), dt)
    fam = B.elementwise_plan("mad_relu", [a_dev, dev(b, dt), dev(cc, dt)], out)
    assert fam == 2
    B.elementwise_broadcast("mad_relu", [a_dev, dev(b, dt), dev(cc, dt)], out)
    ref = O.elementwise("mad_relu", [a_store.T, b, cc])
    S = O.elementwise("mad", [np.abs(a_store.T), np.abs(b), np.abs(cc)])
    check(host(out), ref, tol_for(dt, dt, TOL_EW), S, "transposed")
    # bit-equal to the same call on a materialised transpose
    out2 = B.elementwise_broadcast("mad_relu", [dev(np.ascontiguousarray(a_store.T), dt), dev(b, dt), dev(cc, dt)], empty((r, c), dt))
    assert torch.equal(out.view(torch.int16 if dt == "bf16" else torch.int32), out2.view(torch.int16 if dt == "bf16" else torch.int32))


def test_gelu_fp32_keeps_relative_accuracy_in_the_negative_tail():
    # gelu(x) = x Phi(x) through an erfc whose relative error stays at a few 1e-6 in the tails: at
    # x = -8 the result is 5e-15 and still has five correct digits
    # (reference: x/2 erfc(-x/sqrt 2) by SciPy's erfc; the oracle's 1 + erf form cancels in float64
    # out there, which the comparison at |x| <= 5 below shows to be the same function)
    from scipy.special import erfc
    x = np.linspace(-8.0, 8.0, 200001).astype(np.float32)
    got = host(B.elementwise_broadcast("gelu", [dev(x)], empty(x.shape)))
    ref = 0.5 * x.astype(np.float64) * erfc(-x.astype(np.float64) / np.sqrt(2.0))
    assert np.all(np.abs(got - ref) <= 2e-5 * np.abs(ref) + 1e-38)
    near = np.abs(x) <= 5
    assert np.allclose(O.elementwise("gelu", [x])[near], ref[near], rtol=1e-9, atol=0)
    gy = np.ones_like(x)
    got = host(B.elementwise_broadcast("gelu_bwd", [dev(gy), dev(x)], empty(x.shape)))
    ref = O.elementwise("gelu_bwd", [gy, x])
    assert np.all(np.abs(got - ref) <= 1e-6)          # (the derivative cancels in the tail: absolute bound)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("n_t", [2, 3])
def test_several_transposed_operands(dt, n_t):
    # every transposed operand has an LDS tile of its own; with three of them the wide tiles no
    # longer fit and the narrow ones are used
    r, c = 392, 264
    stores = [rnd((c, r), dt) for _ in range(3)]
    views = [dev(s_, dt).t() if k < n_t else dev(np.ascontiguousarray(s_.T), dt) for k, s_ in enumerate(stores)]
    out = empty((r, c), dt)
    assert B.elementwise_plan("mad", views, out) == 2
    B.elementwise_broadcast("mad", views, out)
    ref = O.elementwise("mad", [s_.T for s_ in stores])
    check(host(out), ref, tol_for(dt, dt, TOL_EW), O.elementwise("mad", [np.abs(s_.T) for s_ in stores]), "%d transposed" % n_t)


def test_strided_views_and_inplace():
    big = rnd((40, 50))
    d = dev(big)
    v = d[3:37:2, 5:47:3]                      # general strides
    assert B.elementwise_plan("relu", [v], empty(tuple(v.shape))) == 3
    out = B.elementwise_broadcast("relu", [v], empty(tuple(v.shape)))
    check(host(out), O.elementwise("relu", [big[3:37:2, 5:47:3]]), TOL_EW, None, "strided")
    p = d[:, 8:40]                             # pitched rows
    assert B.elementwise_plan("scale", [p], p) == 1
    B.elementwise_broadcast("scale", [p], p, scalars=[2.0])   # in place on a view
    want = big.copy(); want[:, 8:40] *= 2
    assert np.array_equal(host(d), want)
    # output written through a transposed view
    o = empty((50, 40)).t()
    B.elementwise_broadcast("copy", [dev(big)], o)
    assert np.array_equal(host(o), big)
    # zero-size
    z = empty((0, 7))
    B.elementwise_broadcast("add", [z, z], z)


def test_elementwise_large_flat_tail():
    n = 4 * 1024 * 1024 + 3                    # several blocks and a ragged tail
    x, y = rnd((n,)), rnd((n,))
    out = B.elementwise_broadcast("add", [dev(x), dev(y)], empty((n,)))
    assert np.array_equal(host(out), (x + y).astype(np.float64))      # fp32 add is correctly rounded


# ------------------------------------------------------------------------------------ reductions
def _reduce(op, x_np, x_dev, axis, dt_out="f32", keep=False):
    need = B.reduce_axis_workspace_bytes(x_dev, axis)
    ref = O.reduce_axis(op, x_np, axis, keep)
    out = B.reduce_axis(op, x_dev, axis, empty(ref.shape, dt_out), keep, ws(need) if need else None)
    return host(out), ref


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(513, 1030), (4100, 260), (32, 100), (1024, 10), (7, 4099), (1, 50), (50, 1), (2500, 3),
                                   (1024, 1000), (1000, 264), (2048, 72), (130, 4096), (65, 8), (300, 333), (2000, 5)])
def test_reduce_2d_both_axes(dt, shape):
    x = rnd(shape, dt)
    tol = tol_for(dt, "f32", TOL_SUM)
    for axis in (0, 1, -1):
        got, ref = _reduce("sum", x, dev(x, dt), axis)
        check(got, ref, tol, O.reduce_axis("sum", np.abs(x), axis), "sum axis %d" % axis)
        got, ref = _reduce("max", x, dev(x, dt), axis)
        assert np.array_equal(got, ref)
    # transposed views swap the two kernels and must give the same sums
    xt = dev(x, dt).t()
    got, ref = _reduce("sum", x.T, xt, 0)
    check(got, ref, tol, O.reduce_axis("sum", np.abs(x.T), 0), "sum T axis 0")
    got, ref = _reduce("sum", x.T, xt, 1, keep=True)
    check(got, ref, tol, O.reduce_axis("sum", np.abs(x.T), 1, True), "sum T axis 1 keepdims")


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_reduce_short_cache_resident_columns_take_one_launch(dt):
    """The column sums of a short stack of rows (a bias gradient) need no workspace, i.e. no second launch."""
    tol = tol_for(dt, "f32", TOL_SUM)
    for shape, axis in [((1024, 1000), 0), ((1000, 1000), 0), ((2048, 512), 0), ((3, 300, 64), 1), ((5, 1031, 24), 1)]:
        x = rnd(shape, dt)
        d = dev(x, dt)
        assert B.reduce_axis_workspace_bytes(d, axis) == 0
        got, ref = _reduce("sum", x, d, axis)
        check(got, ref, tol, O.reduce_axis("sum", np.abs(x), axis), "short columns %s" % (shape,))
        got, ref = _reduce("max", x, d, axis)
        assert np.array_equal(got, ref)
    x = RNG.integers(-4, 5, size=(1000, 1000)).astype(np.float32)
    got, ref = _reduce("sum", x, dev(x, dt), 0)
    assert np.array_equal(got, ref)
    x = rnd((1024, 1000), dt)
    got, ref = _reduce("sum", x[:, 8:968], dev(x, dt)[:, 8:968], 0)  # a pitched column slice
    check(got, ref, tol, O.reduce_axis("sum", np.abs(x[:, 8:968]), 0), "pitched short columns")


def test_reduce_exact_integers_bit_equal():
    for dt in ("f32", "bf16"):
        x = RNG.integers(-4, 5, size=(2050, 1500)).astype(np.float32)
        for axis in (0, 1):
            got, ref = _reduce("sum", x, dev(x, dt), axis)
            assert np.array_equal(got, ref)
    assert np.array_equal(_reduce("sum", np.ones((777, 33), np.float32), dev(np.ones((777, 33), np.float32)), 0)[0], np.full(33, 777.0))


def test_reduce_nd_keepdims_bf16_out_empty_and_deterministic():
    x = rnd((6, 70, 40))
    for axis in (0, 1, 2):
        got, ref = _reduce("sum", x, dev(x), axis, keep=(axis == 1))
        check(got, ref, TOL_SUM, O.reduce_axis("sum", np.abs(x), axis, axis == 1), "3-d axis %d" % axis)
    v = dev(x)[:, ::2, 1:39]                    # general strided view
    got, ref = _reduce("sum", x[:, ::2, 1:39], v, 1)
    check(got, ref, TOL_SUM, O.reduce_axis("sum", np.abs(x[:, ::2, 1:39]), 1), "strided view")
    got, ref = _reduce("sum", x, dev(x), 2, dt_out="bf16")
    check(got, ref, TOL_BF16, None, "bf16 out")
    e = empty((5, 0))
    out = B.reduce_axis("sum", e, 1, empty((5,)))
    assert np.all(host(out) == 0)
    out = B.reduce_axis("max", e, 1, empty((5,)))
    assert np.all(host(out) == -np.inf)
    B.reduce_axis("sum", e, 0, empty((0,)))
    big = rnd((3000, 700))
    d = dev(big)
    need = B.reduce_axis_workspace_bytes(d, 0)
    assert need > 0
    a = B.reduce_axis("sum", d, 0, empty((700,)), ws=ws(need))
    b = B.reduce_axis("sum", d, 0, empty((700,)), ws=ws(need))
    assert torch.equal(a, b)                   # fixed summation order: bit-reproducible
    s0 = host(a).sum()
    s1 = host(B.reduce_axis("sum", d, 1, empty((3000,)))).sum()
    assert abs(s0 - s1) <= 1e-4 * np.abs(big).sum()


def _np_fold(op, x, axes, keep):
    """Several axes folded one at a time by the oracle (its single-axis call is pinned against NumPy)."""
    out = np.asarray(x, dtype=np.float64)
    for a in sorted((a % out.ndim for a in axes), reverse=True):
        out = O.reduce_axis(op, out, a, True)
    return out if keep else out.reshape([n for d, n in enumerate(out.shape) if d not in [a % out.ndim for a in axes]])


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_reduce_several_axes_at_once(dt):
    tol = tol_for(dt, "f32", TOL_SUM)
    cases = [((6, 70, 40), (0, 2)), ((6, 70, 40), (0, 1)), ((6, 70, 40), (1, 2)), ((6, 70, 40), None), ((5, 3, 33, 65), (1, 3)),
             ((5, 3, 33, 65), (0, 2, 3)), ((300, 1100), None), ((2, 1200, 1024), None), ((1 << 21,), None), ((4, 1 << 20), (1,)),
             ((2, 3, 0, 5), (1, 3)), ((7, 1, 9), (0, 1))]
    for shape, axes in cases:
        x = rnd(shape, dt)
        d = dev(x, dt)
        ax = tuple(range(len(shape))) if axes is None else axes
        for keep in (False, True):
            ref = _np_fold("sum", x, ax, keep)
            need = B.reduce_axis_workspace_bytes(d, axes)
            out = B.reduce_axis("sum", d, axes, empty(ref.shape), keepdims=keep, ws=ws(need))
            check(host(out), ref, tol, _np_fold("sum", np.abs(x), ax, keep), "sum %s over %s" % (shape, axes))
            if x.size:
                got = B.reduce_axis("max", d, axes, empty(ref.shape), keepdims=keep, ws=ws(need))
                assert np.array_equal(host(got), _np_fold("max", x, ax, keep))
        if x.size:
            again = B.reduce_axis("sum", d, axes, empty(ref.shape), keepdims=True, ws=ws(need))
            assert torch.equal(again, out)                            # fixed order
    # a transposed / sliced view, a bf16 result, exact integers, and the no-allocation entry point
    x = rnd((40, 50, 64), dt)
    v = dev(x, dt).permute(2, 0, 1)[1:63]
    xv = np.transpose(x, (2, 0, 1))[1:63]
    out = B.reduce_axis("sum", v, (0, 2), empty((40,)), ws=ws(B.reduce_axis_workspace_bytes(v, (0, 2))))
    check(host(out), _np_fold("sum", xv, (0, 2), False), tol, _np_fold("sum", np.abs(xv), (0, 2), False), "view")
    xi = RNG.integers(-4, 5, size=(33, 40, 130)).astype(np.float32)
    di = dev(xi, dt)
    need = B.reduce_axis_workspace_bytes(di, (0, 2))
    assert np.array_equal(host(B.reduce_axis("sum", di, (0, 2), empty((40,)), ws=ws(need))), xi.sum(axis=(0, 2), dtype=np.float64))
    assert np.array_equal(host(B.reduce_axis("sum", di, None, empty(()), ws=ws(B.reduce_axis_workspace_bytes(di, None)))), xi.sum(dtype=np.float64))
    assert torch.equal(B.reduce_axis_static("sum", di, (0, 2), empty((40,))), B.reduce_axis("sum", di, (0, 2), empty((40,)), ws=ws(need)))
    ob = B.reduce_axis("sum", di, (0, 2), empty((40,), "bf16"), ws=ws(need))
    check(host(ob), xi.sum(axis=(0, 2), dtype=np.float64), TOL_BF16, None, "bf16 result")
    with pytest.raises(B.ChnError):
        B.reduce_axis("sum", di, (0, 2), empty((40,)))                # workspace required
    with pytest.raises(B.ChnError):
        B.reduce_axis("sum", di, (0, 2), empty((41,)), ws=ws(need))   # wrong shape


@pytest.mark.parametrize("dt,shape", [("f32", (1500, 2048)), ("f32", (2, 1100, 2052)), ("bf16", (3000, 4104)), ("bf16", (1027, 8192))])
def test_reduce_wide_columns_ignore_what_the_workspace_held(dt, shape):
    """Wide column reductions leave partial sums in the caller's workspace.  Its previous contents
    (random bytes, all ones, the leftovers of a call of another shape or of the same call) must not
    matter, the bits must not change from call to call, and a recorded launch must replay them."""
    x = rnd(shape, dt)
    d = dev(x, dt)
    axis = len(shape) - 2
    need = B.reduce_axis_workspace_bytes(d, axis)
    assert need > 0
    ref = O.reduce_axis("sum", x, axis)
    scale = O.reduce_axis("sum", np.abs(x), axis)
    tol = tol_for(dt, "f32", TOL_SUM)
    y = dev(rnd((1100, 2048)))
    w = ws(max(need, B.reduce_axis_workspace_bytes(y, 0)) + 4096)
    results = []
    for fill in ("random", "ones", "other", "same", "same"):
        if fill == "random":
            w.copy_(torch.from_numpy(RNG.integers(0, 256, size=w.numel(), dtype=np.uint8)))
        elif fill == "ones":
            w.fill_(255)
        elif fill == "other":
            B.reduce_axis("sum", y, 0, empty((2048,)), ws=w)
        out = B.reduce_axis("sum", d, axis, empty(ref.shape), ws=w)
        check(host(out), ref, tol, scale, "workspace " + fill)
        results.append(out)
    for r in results[1:]:
        assert torch.equal(r, results[0])        # fixed summation order
    got, refm = _reduce("max", x, d, axis)
    assert np.array_equal(got, refm)
    g = torch.cuda.CUDAGraph()
    out = empty(ref.shape)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        B.reduce_axis("sum", d, axis, out, ws=w)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            B.reduce_axis("sum", d, axis, out, ws=w)
    for _ in range(3):
        out.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, results[0])
        eager = B.reduce_axis("sum", d, axis, empty(ref.shape), ws=w)
        torch.cuda.synchronize()
        assert torch.equal(eager, results[0])


# ------------------------------------------------------------------------------------ softmax CE
@pytest.mark.parametrize("N,Cn,dt,lab", [(37, 10, "f32", np.int32), (300, 1000, "f32", np.int64), (70, 4100, "f32", np.int32),
                                         (129, 1000, "bf16", np.int32), (33, 2051, "bf16", np.int64), (5, 33, "f32", np.int32)])
def test_softmax_ce(N, Cn, dt, lab):
    z = rnd((N, Cn), dt, -6, 6)
    t = RNG.integers(0, Cn, size=(N,)).astype(lab)
    t[::7] = -1
    zd, td = dev(z, dt), dev(t)
    loss, rows, lse = empty(()), empty((N,)), empty((N,))
    w = ws(B.softmax_ce_workspace_bytes(N))
    B.softmax_ce_fwd(zd, td, loss, rows, lse, ws=w)
    rl, rrows, rlse, nv = O.softmax_ce_fwd(z, t)
    check(host(lse), rlse, TOL_EW * 10, None, "lse")
    check(host(rows), rrows, TOL_SUM, np.abs(rlse), "loss rows")
    assert np.all(host(rows)[t == -1] == 0)
    check(host(loss), np.array(rl), TOL_SUM, None, "loss mean")
    # without optional outputs the mean is identical
    loss2 = B.softmax_ce_fwd(zd, td, empty(()), ws=w)
    assert torch.equal(loss, loss2)
    ref = O.softmax_ce_bwd(z, t, -1, 1.5)
    for out_dt in ("f32", "bf16"):
        for use_lse in (True, False):
            dz = B.softmax_ce_bwd(zd, td, empty((N, Cn), out_dt), lse if use_lse else None, 1.5, ws=w)
            check(host(dz), ref, tol_for(dt, out_dt, TOL_EW * 10), 1.5 / nv, "dlogits")
            assert np.all(host(dz)[t == -1] == 0)
    g = host(B.softmax_ce_bwd(zd, td, empty((N, Cn)), lse, 1.0, ws=w))
    assert np.max(np.abs(g.sum(axis=1))) < 1e-6                       # each row of the gradient sums to 0
    # one-hot position is exact: the only negative entry of a row sits at its label
    valid = np.where(t != -1)[0]
    assert np.array_equal(np.argmin(g[valid], axis=1), t[valid])
    if dt == "f32":                                                    # in place
        zc = zd.clone()
        B.softmax_ce_bwd(zc, td, zc, None, 1.5, ws=w)
        check(host(zc), ref, TOL_EW * 10, 1.5 / nv, "in place")


@pytest.mark.parametrize("N,Cn,lab", [(37, 10, np.int32), (301, 1000, np.int64), (5, 65, np.int32), (130, 4100, np.int32)])
def test_softmax_ce_second_order(N, Cn, lab):
    z = rnd((N, Cn), "f32", -5, 5)
    u = rnd((N, Cn), "f32", -2, 2)
    t = RNG.integers(0, Cn, size=(N,)).astype(lab)
    t[::6] = -1
    t[3] = Cn + 5                                                  # a stray label counts as ignored
    zd, ud, td = dev(z), dev(u), dev(t)
    w = ws(B.softmax_ce_workspace_bytes(N))
    ref_dz, ref_du = O.softmax_ce_bwd2(z, t, u, -1, 1.5)
    nv = int(((t >= 0) & (t < Cn)).sum())
    lse = empty((N,))
    B.softmax_ce_fwd(zd, td, empty(()), None, lse, ws=w)
    for use_lse in (False, True):
        dz, du = empty((N, Cn)), empty(())
        B.softmax_ce_bwd2(zd, td, ud, dz, du, lse if use_lse else None, 1.5, ws=w)
        check(host(dz), ref_dz, TOL_EW * 10, 1.5 / nv * np.abs(u).max(), "second-order dlogits")
        assert abs(float(du.cpu()) - ref_du) <= 1e-5 * (np.abs(u).sum() / nv)
        assert np.all(host(dz)[(t < 0) | (t >= Cn)] == 0)
    dz2 = B.softmax_ce_bwd2(zd, td, ud, empty((N, Cn)), None, lse, 1.5, ws=w)   # without the scalar output
    assert torch.equal(dz2, dz)


@pytest.mark.parametrize("N,Cn,lab", [(300, 10, np.int32), (70, 1000, np.int64), (9000, 10, np.int32), (64, 4100, np.int32)])
def test_softmax_ce_and_embedding_never_follow_a_stray_index(N, Cn, lab):
    """Labels outside [0, C) count as ignored; ids outside [0, V) gather zeros and receive no gradient.
    (Every kernel family: separate forward / backward, the fused call, its one-workgroup form.)"""
    z = rnd((N, Cn), "f32", -6, 6)
    t = RNG.integers(0, Cn, size=(N,)).astype(lab)
    t[::7] = -1
    t[3::11] = Cn
    t[5::13] = -100
    t[1] = np.iinfo(lab).max
    zd, td = dev(z), dev(t)
    w = ws(B.softmax_ce_workspace_bytes(N))
    rl, rrows, rlse, nv = O.softmax_ce_fwd(z, t)
    assert nv == int(((t >= 0) & (t < Cn)).sum())
    loss, rows, lse = empty(()), empty((N,)), empty((N,))
    B.softmax_ce_fwd(zd, td, loss, rows, lse, ws=w)
    check(host(rows), rrows, TOL_SUM, np.abs(rlse), "loss rows")
    check(host(loss), np.array(rl), TOL_SUM, None, "loss mean")
    ref = O.softmax_ce_bwd(z, t, -1, 1.5)
    dz = B.softmax_ce_bwd(zd, td, empty((N, Cn)), lse, 1.5, ws=w)
    check(host(dz), ref, TOL_EW * 10, 1.5 / nv, "dlogits")
    bad = (t < 0) | (t >= Cn)
    assert np.all(host(dz)[bad] == 0) and np.all(host(rows)[bad] == 0)
    loss2, dz2 = empty(()), empty((N, Cn))
    B.softmax_ce_fwd_bwd(zd, td, loss2, dz2, None, 1.5, ws=w)
    check(host(loss2), np.array(rl), TOL_SUM, None, "fused loss")
    check(host(dz2), ref, TOL_EW * 10, 1.5 / nv, "fused dlogits")
    assert np.all(host(dz2)[bad] == 0)
    # embedding
    V, D = 50, 72
    E = rnd((V, D))
    ids = RNG.integers(0, V, size=(N,)).astype(lab)
    ids[2::9] = V
    ids[4::10] = -3
    ids[0] = np.iinfo(lab).max
    out = B.embed_fwd(dev(E), dev(ids), empty((N, D)))
    assert np.array_equal(host(out), O.embed_fwd(E, ids))
    assert np.all(host(out)[(ids < 0) | (ids >= V)] == 0)
    dout = rnd((N, D))
    dt_ = B.embed_bwd(dev(ids), dev(dout), empty((V, D)))
    check(host(dt_), O.embed_bwd(ids, dout, V), TOL_SUM, O.embed_bwd(ids, np.abs(dout), V), "embed_bwd with stray ids")


@pytest.mark.parametrize("N,Cn,dt,lab", [(37, 10, "f32", np.int32), (1024, 10, "f32", np.int64), (3000, 33, "bf16", np.int32),   # one block
                                         (100, 16, "f32", np.int32), (100, 17, "f32", np.int32), (2000, 64, "f32", np.int64), (2, 1, "f32", np.int32),
                                         (8193, 10, "f32", np.int32), (300, 1000, "f32", np.int64), (70, 4100, "f32", np.int32),
                                         (129, 1000, "bf16", np.int32), (33, 2051, "bf16", np.int64), (5, 65, "f32", np.int32),
                                         # long rows: held in registers between scan and gradient up to 12288 classes, streamed twice beyond
                                         (40, 10000, "f32", np.int32), (9, 12288, "f32", np.int64), (9, 12296, "f32", np.int32),
                                         (17, 8192, "bf16", np.int32)])
def test_softmax_ce_loss_and_gradient_in_one_call(N, Cn, dt, lab):
    z = rnd((N, Cn), dt, -6, 6)
    t = RNG.integers(0, Cn, size=(N,)).astype(lab)
    t[::7] = -1
    zd, td = dev(z, dt), dev(t)
    w = ws(B.softmax_ce_workspace_bytes(N))
    rl, _, rlse, nv = O.softmax_ce_fwd(z, t)
    ref = O.softmax_ce_bwd(z, t, -1, 1.5)
    for out_dt in ("f32", "bf16"):
        loss, lse, dz = empty(()), empty((N,)), empty((N, Cn), out_dt)
        B.softmax_ce_fwd_bwd(zd, td, loss, dz, lse, 1.5, ws=w)
        check(host(loss), np.array(rl), TOL_SUM, None, "loss mean")
        check(host(lse), rlse, TOL_EW * 10, None, "lse")
        check(host(dz), ref, tol_for(dt, out_dt, TOL_EW * 10), 1.5 / nv, "dlogits")
        assert np.all(host(dz)[t == -1] == 0)
    # against the two separate calls (the gradient kernel is shared on the many-class path)
    l2, lse2 = empty(()), empty((N,))
    B.softmax_ce_fwd(zd, td, l2, None, lse2, ws=w)
    d2 = B.softmax_ce_bwd(zd, td, empty((N, Cn)), lse2, 1.5, ws=w)
    loss, dz = empty(()), empty((N, Cn))
    B.softmax_ce_fwd_bwd(zd, td, loss, dz, None, 1.5, ws=w)          # lse not asked for
    assert abs(float(loss.cpu()) - float(l2.cpu())) <= 1e-6 * abs(float(l2.cpu()))
    assert np.max(np.abs(host(dz) - host(d2))) <= 1e-6 * 1.5 / nv
    # written over the logits
    zc = zd.clone()
    loss3 = empty(())
    B.softmax_ce_fwd_bwd(zc, td, loss3, zc, None, 1.5, ws=w)
    check(host(zc), ref, tol_for(dt, dt, TOL_EW * 10), 1.5 / nv, "in place")
    check(host(loss3), np.array(rl), TOL_SUM, None, "loss mean, in place")
    with pytest.raises(B.ChnError):
        B.softmax_ce_fwd_bwd(zd, td, loss, empty((N, Cn + 1)), None, 1.0, ws=w)
    # every row ignored; no rows at all
    tn = np.full(N, -1, lab)
    B.softmax_ce_fwd_bwd(zd, dev(tn), loss, dz, None, 1.0, ws=w)
    assert float(loss.cpu()) == 0.0 and np.all(host(dz) == 0)
    loss.fill_(7.0)
    B.softmax_ce_fwd_bwd(empty((0, Cn), dt), dev(np.zeros(0, lab)), loss, empty((0, Cn)), None, 1.0, ws=w)
    assert float(loss.cpu()) == 0.0


def test_softmax_ce_closed_forms():
    for Cn in (10, 1000, 10000):
        z = np.zeros((4, Cn), dtype=np.float32)
        t = np.array([0, Cn - 1, 5, 7], dtype=np.int32)
        w = ws(B.softmax_ce_workspace_bytes(4))
        loss = B.softmax_ce_fwd(dev(z), dev(t), empty(()), ws=w)
        assert abs(float(loss.cpu()) - np.log(Cn)) < 1e-5 * np.log(Cn)
        dz = host(B.softmax_ce_bwd(dev(z), dev(t), empty((4, Cn)), ws=w))
        want = np.full((4, Cn), 0.25 / Cn); want[np.arange(4), t] -= 0.25
        check(dz, want, TOL_EW, None, "uniform")
    # all rows ignored
    z = rnd((6, 50)); t = np.full(6, -1, np.int32)
    w = ws(B.softmax_ce_workspace_bytes(6))
    assert float(B.softmax_ce_fwd(dev(z), dev(t), empty(()), ws=w).cpu()) == 0.0
    assert np.all(host(B.softmax_ce_bwd(dev(z), dev(t), empty((6, 50)), ws=w)) == 0)


# ------------------------------------------------------------------------------------ LSTM cell
@pytest.mark.parametrize("Bn,H", [(128, 650), (3, 5), (17, 129)])
def test_lstm_cell(Bn, H):
    z, bias, cp = rnd((Bn, 4 * H), lo=-3, hi=3), rnd((4 * H,)), rnd((Bn, H), lo=-2, hi=2)
    c, h, g = empty((Bn, H)), empty((Bn, H)), empty((Bn, 4 * H))
    B.lstm_fwd(dev(z), dev(bias), dev(cp), c, h, g)
    rc, rh, rg = O.lstm_fwd(z, bias, cp)
    check(host(g), rg, TOL_EW, None, "gates")
    H_ = H
    Sc = np.abs(rg[:, H_:2 * H_] * cp) + np.abs(rg[:, :H_] * rg[:, 2 * H_:3 * H_])   # |f c_prev| + |i g|
    check(host(c), rc, TOL_EW, Sc, "c")
    check(host(h), rh, TOL_EW, Sc, "h")
    c2, h2 = empty((Bn, H)), empty((Bn, H))
    B.lstm_fwd(dev(z + bias), None, dev(cp), c2, h2, None)          # bias is just added to z
    check(host(c2), rc, TOL_EW, Sc + 1e-2, "c no-bias")
    dh, dcn = rnd((Bn, H)), rnd((Bn, H))
    # teacher-forced: the backward gets the GPU forward's own retained outputs
    gh, ch = host(g), host(c)
    dz, dcp = empty((Bn, 4 * H)), empty((Bn, H))
    B.lstm_bwd(g, dev(cp), c, dev(dh), dev(dcn), dz, dcp)
    rdz, rdcp = O.lstm_bwd(gh, cp, ch, dh, dcn)
    # dc = dc_next + dh*o*(1 - tanh(c)^2) is a two-term sum: its terms set the error scale
    Sdc = np.abs(dcn) + np.abs(dh * gh[:, 3 * H:] * (1 - np.tanh(ch) ** 2))
    Sdz = np.concatenate([Sdc, Sdc * np.abs(cp), Sdc, np.abs(dh)], axis=1)
    check(host(dz), rdz, TOL_EW, Sdz, "dz")
    check(host(dcp), rdcp, TOL_EW, Sdc, "dc_prev")
    B.lstm_bwd(g, dev(cp), c, dev(dh), None, dz, dcp)
    rdz0, rdcp0 = O.lstm_bwd(gh, cp, ch, dh, None)
    check(host(dz), rdz0, TOL_EW, Sdz, "dz no dc_next")
    # pitched rows: z is a row block of a larger time-major buffer
    zz = dev(np.concatenate([z, z], axis=1))[:, :4 * H]
    c3, h3 = empty((Bn, H)), empty((Bn, H))
    B.lstm_fwd(zz, dev(bias), dev(cp), c3, h3, None)
    assert torch.equal(c3, c) and torch.equal(h3, h)
    # mixed precision: h stored in bf16 is the fp32 h rounded to nearest even; dh read and dz stored
    # in bf16 are the fp32 kernel on the same (bf16-exact) dh, rounded at the store
    hb = empty((Bn, H), "bf16")
    B.lstm_fwd(dev(z), dev(bias), dev(cp), c3, hb, None)
    assert np.array_equal(host(hb), O.round_bf16(host(h))) and torch.equal(c3, c)
    dhb = bf16r(dh)
    dzb, dz32 = empty((Bn, 4 * H), "bf16"), empty((Bn, 4 * H))
    B.lstm_bwd(g, dev(cp), c, dev(dhb, "bf16"), dev(dcn), dzb, dcp)
    dcp_b = dcp.clone()
    B.lstm_bwd(g, dev(cp), c, dev(dhb), dev(dcn), dz32, dcp)
    assert np.array_equal(host(dzb), O.round_bf16(host(dz32))) and torch.equal(dcp_b, dcp)
    rdzb, _ = O.lstm_bwd(gh, cp, ch, dhb, dcn)
    check(host(dzb), rdzb, TOL_BF16, Sdz, "dz bf16")


def test_lstm_zero_preactivation_closed_form():
    cp = rnd((4, 8))
    c, h, g = empty((4, 8)), empty((4, 8)), empty((4, 32))
    B.lstm_fwd(dev(np.zeros((4, 32), np.float32)), None, dev(cp), c, h, g)
    assert np.array_equal(host(c), 0.5 * cp.astype(np.float64))
    check(host(h), 0.5 * np.tanh(0.5 * cp.astype(np.float64)), TOL_EW, None, "h")
    assert np.array_equal(host(g)[:, :8], np.full((4, 8), 0.5)) and np.all(host(g)[:, 16:24] == 0)


# ------------------------------------------------------------------------------------ SGD
def test_sgd():
    for n in (89610 // 9, 1000 * 784, 7, 4096 * 4 + 5):
        p, g = rnd((n,)), rnd((n,))
        pd, lp = dev(p), empty((n,), "bf16")
        B.sgd_update(pd, dev(g), 0.01, lp)
        ref = O.sgd_update(p, g, np.float32(0.01))
        check(host(pd), ref, TOL_EW, np.abs(p), "sgd")
        assert np.array_equal(host(lp), O.round_bf16(host(pd)))       # working copy = RNE of the new master
    p = rnd((300, 70))
    pd = dev(p)
    B.sgd_update(pd, dev(rnd((300, 70))), 0.0)
    assert np.array_equal(host(pd), p)
    B.sgd_update(pd, dev(np.ones((300, 70), np.float32)), 0.25)
    assert np.array_equal(host(pd), (p - np.float32(0.25)).astype(np.float64))
    # multi-tensor form equals the single calls bit for bit
    shapes = [(100, 784), (100,), (10, 100), (10,), (0,), (3, 3)] * 9        # > 40 tensors: two launches
    ps, gs = [rnd(s) for s in shapes], [rnd(s) for s in shapes]
    a = [dev(x) for x in ps]; b = [dev(x) for x in ps]; gd = [dev(x) for x in gs]
    lows = [empty(s, "bf16") if i % 2 == 0 else None for i, s in enumerate(shapes)]
    B.sgd_update_multi(a, gd, 0.05, lows)
    for x, g_ in zip(b, gd):
        B.sgd_update(x, g_, 0.05)
    for x, y, l in zip(a, b, lows):
        assert torch.equal(x, y)
        if l is not None:
            assert np.array_equal(host(l), O.round_bf16(host(x)))


# ------------------------------------------------------------------------------------ embedding
@pytest.mark.parametrize("V,D,N,idt", [(1000, 650, 500, np.int32), (50, 7, 300, np.int64), (10, 1100, 20, np.int32)])
def test_embedding(V, D, N, idt):
    E = rnd((V, D))
    ids = RNG.integers(0, V, size=(N,)).astype(idt)
    ids[:5] = ids[0]                              # guaranteed collisions
    out = B.embed_fwd(dev(E), dev(ids), empty((N, D)))
    assert np.array_equal(host(out), O.embed_fwd(E, ids))                    # bit copies
    Eb = bf16r(E)
    outb = B.embed_fwd(dev(Eb, "bf16"), dev(ids), empty((N, D), "bf16"))
    assert np.array_equal(host(outb), O.embed_fwd(Eb, ids))
    dout = rnd((N, D))
    dE = B.embed_bwd(dev(ids), dev(dout), empty((V, D)))
    ref = O.embed_bwd(ids, dout, V)
    check(host(dE), ref, TOL_SUM, O.embed_bwd(ids, np.abs(dout), V), "dE")
    untouched = np.setdiff1d(np.arange(V), ids)
    assert np.all(host(dE)[untouched] == 0)
    dE2 = B.embed_bwd(dev(ids), dev(dout), empty((V, D)))
    assert torch.equal(dE, dE2)                                              # bit-reproducible
    acc = dev(E)
    B.embed_bwd(dev(ids), dev(dout), acc, accumulate=True)
    check(host(acc), O.embed_bwd(ids, dout, V, E), TOL_SUM, O.embed_bwd(ids, np.abs(dout), V, np.abs(E)), "accumulate")
    di = RNG.integers(-3, 4, size=(N, D)).astype(np.float32)                 # integers: exact in any order
    assert np.array_equal(host(B.embed_bwd(dev(ids), dev(di), empty((V, D)))), O.embed_bwd(ids, di, V))


# ------------------------------------------------------------------------------------ Adam
def test_adam_update_multi_follows_the_oracle_over_several_steps():
    rng = np.random.default_rng(31)
    shapes = [(1000, 37), (5,), (4096,), (3, 3, 3), (0,), (129, 64)]
    P = [rng.standard_normal(s).astype(np.float32) for s in shapes]
    pd = [dev(p) for p in P]
    md, vd = [torch.zeros_like(p) for p in pd], [torch.zeros_like(p) for p in pd]
    low = [torch.zeros(s, dtype=torch.bfloat16, device="cuda") if i % 2 == 0 else None for i, s in enumerate(shapes)]
    ref = [(p.astype(np.float64), np.zeros(p.shape), np.zeros(p.shape)) for p in P]
    for step in range(1, 4):
        G = [rng.standard_normal(s).astype(np.float32) * 10.0 ** rng.integers(-3, 2) for s in shapes]
        before = [(host(p), host(m), host(v)) for p, m, v in zip(pd, md, vd)]
        B.adam_update_multi(pd, [dev(g) for g in G], md, vd, 0.01, step, 0.9, 0.999, 1e-8, lowp_copies=low)
        for i, g in enumerate(G):
            # teacher-forced on the GPU's own state: one step of fp32 arithmetic
            rp, rm, rv = O.adam_update(before[i][0], g, before[i][1], before[i][2], 0.01, step)
            check(host(md[i]), rm, TOL_EW, np.abs(before[i][1]) + np.abs(g), "m")
            check(host(vd[i]), rv, TOL_EW, None, "v")
            check(host(pd[i]), rp, TOL_EW, np.abs(before[i][0]) + 0.01 * 10, "p")
            # and end to end against the oracle's own trajectory
            ref[i] = O.adam_update(ref[i][0], g, ref[i][1], ref[i][2], 0.01, step)
            check(host(pd[i]), ref[i][0], 1e-5, np.abs(ref[i][0]) + 0.01 * 10 * step, "p trajectory")
            if low[i] is not None:
                assert np.array_equal(host(low[i]), O.round_bf16(host(pd[i])))
    with pytest.raises(B.ChnError):
        B.adam_update_multi(pd[:1], [dev(G[0])], md[:1], vd[:1], 0.01, 0)           # steps count from 1
    with pytest.raises(B.ChnError):
        B.adam_update_multi(pd[:1], [dev(G[0])], md[:1], vd[1:2], 0.01, 1)          # state of another shape


# ------------------------------------------------------------------------------------ fused recurrent step
@pytest.mark.parametrize("Bn,H,dt", [(128, 672, "f32"), (128, 672, "bf16"), (5, 32, "f32"), (33, 64, "bf16"), (70, 96, "f32")])
def test_lstm_step_fused_product_and_cell(Bn, H, dt):
    tol = TOL_SUM if dt == "f32" else TOL_BF16
    q = (lambda a: a) if dt == "f32" else bf16r
    zx, bias, cp = rnd((Bn, 4 * H), lo=-2, hi=2), rnd((4 * H,)), rnd((Bn, H), lo=-2, hi=2)
    hp, U = q(rnd((Bn, H))), q(rnd((H, 4 * H), lo=-0.1, hi=0.1))
    c, h, g = empty((Bn, H)), empty((Bn, H), dt), empty((Bn, 4 * H))
    Ut = dev(np.ascontiguousarray(U.T), dt)
    B.lstm_step_fwd(dev(zx), dev(hp, dt), Ut, dev(bias), dev(cp), c, h, g)
    z = O.gemm(hp, U, zx, 1.0, 1.0)
    rc, rh, rg = O.lstm_fwd(z, bias, cp)
    Sz = O.gemm(np.abs(hp), np.abs(U)) + np.abs(zx) + np.abs(bias)
    Sg = np.concatenate([0.25 * Sz[:, :H], 0.25 * Sz[:, H:2 * H], Sz[:, 2 * H:3 * H], 0.25 * Sz[:, 3 * H:]], axis=1)   # |d act / dz| <= 1/4, 1
    check(host(g), rg, TOL_SUM, Sg + 1e-1, "gates")
    Sc = np.abs(rg[:, H:2 * H] * cp) + np.abs(rg[:, :H] * rg[:, 2 * H:3 * H]) + Sg[:, :H] + Sg[:, H:2 * H] * np.abs(cp) + Sg[:, 2 * H:3 * H]
    check(host(c), rc, TOL_SUM, Sc, "c")
    check(host(h), rh, tol, Sc + Sg[:, 3 * H:], "h")
    # the unfused calls on the same operands give the same step
    z2 = dev(zx).clone()
    B.gemm(dev(hp, dt), dev(U, dt), z2, beta=1.0)
    c2, h2, g2 = empty((Bn, H)), empty((Bn, H), dt), empty((Bn, 4 * H))
    B.lstm_fwd(z2, dev(bias), dev(cp), c2, h2, g2)
    check(host(c), host(c2), TOL_SUM, Sc, "c fused vs unfused")
    # no bias, no gates, pitched zx (a row block of a wider buffer)
    wide = dev(np.concatenate([zx, zx], axis=1))[:, :4 * H]
    c3, h3 = empty((Bn, H)), empty((Bn, H), dt)
    B.lstm_step_fwd(wide, dev(hp, dt), Ut, None, dev(cp), c3, h3, None)
    rc0, _, _ = O.lstm_fwd(z, None, cp)
    check(host(c3), rc0, TOL_SUM, Sc, "c no bias")

    # backward: dh <- dh + dz_next U^T, then the cell backward from the GPU's own retained outputs
    dhin, dzn, dcn = q(rnd((Bn, H))), q(rnd((Bn, 4 * H), lo=-0.5, hi=0.5)), rnd((Bn, H))
    gh, ch = host(g), host(c)
    dh = dev(dhin, dt)
    dz, dcp = empty((Bn, 4 * H), dt), empty((Bn, H))
    B.lstm_step_bwd(dev(dzn, dt), dev(U, dt), dh, g, dev(cp), c, dev(dcn), dz, dcp)
    dh_ref = O.gemm(dzn, U.T, dhin, 1.0, 1.0)
    Sdh = O.gemm(np.abs(dzn), np.abs(U.T)) + np.abs(dhin)
    check(host(dh), dh_ref, tol, Sdh, "dh total")
    dh_seen = host(dh)                                          # what the cell saw (rounded in mixed precision)
    rdz, rdcp = O.lstm_bwd(gh, cp, ch, dh_seen, dcn)
    Sdc = np.abs(dcn) + np.abs(dh_seen)
    Sdz = np.concatenate([Sdc, Sdc * (1 + np.abs(cp)), Sdc, np.abs(dh_seen)], axis=1)
    check(host(dz), rdz, TOL_EW * 10 if dt == "f32" else TOL_BF16, Sdz, "dz")
    check(host(dcp), rdcp, TOL_EW * 10, Sdc, "dc_prev")
    # last step of the window: nothing flows back from a later step
    dh = dev(dhin, dt)
    B.lstm_step_bwd(None, None, dh, g, dev(cp), c, None, dz, dcp)
    assert np.array_equal(host(dh), dhin.astype(np.float64))
    rdz, rdcp = O.lstm_bwd(gh, cp, ch, dhin, None)
    check(host(dz), rdz, TOL_EW * 10 if dt == "f32" else TOL_BF16, Sdz, "dz last")


def test_lstm_step_refuses_what_it_cannot_tile():
    Bn, H = 4, 40                                               # not a multiple of 32
    z, cp = torch.zeros(Bn, 4 * H, device="cuda"), torch.zeros(Bn, H, device="cuda")
    with pytest.raises(B.ChnError) as e:
        B.lstm_step_fwd(z, cp, torch.zeros(4 * H, H, device="cuda"), None, cp, cp.clone(), cp.clone(), None)
    assert e.value.status == -4
    H = 64
    z, cp = torch.zeros(Bn, 4 * H, device="cuda"), torch.zeros(Bn, H, device="cuda")
    hb = torch.zeros(Bn, H, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.ChnError) as e:                        # operands of two dtypes
        B.lstm_step_fwd(z, hb, torch.zeros(4 * H, H, device="cuda"), None, cp, cp.clone(), hb.clone(), None)
    assert e.value.status == -3
    with pytest.raises(B.ChnError) as e:                        # rows of h_prev off the 16-byte grid
        B.lstm_step_fwd(z, torch.zeros(Bn, H + 1, device="cuda")[:, 1:], torch.zeros(4 * H, H, device="cuda"), None, cp,
                        cp.clone(), cp.clone(), None)
    assert e.value.status == -5


# ------------------------------------------------------------------------------------ argmax
@pytest.mark.parametrize("shape,axis", [((300, 1000), 1), ((300, 1000), 0), ((7, 65, 9), 1), ((7, 65, 9), -1), ((5,), 0),
                                        ((64, 10), 1), ((2, 3, 4, 5), 2)])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_argmax_axis(shape, axis, dt):
    x = rnd(shape, dt)
    x.reshape(-1)[::7] = np.float32(0.5)                         # ties, exact in both storage types
    for odt in (torch.int64, torch.int32):
        oshape = [n for d, n in enumerate(shape) if d != axis % len(shape)]
        out = torch.empty(oshape, dtype=odt, device="cuda")
        B.argmax_axis(dev(x, dt), axis, out)
        assert np.array_equal(host(out), O.argmax_axis(x, axis))
    xt = dev(x, dt)
    if len(shape) == 2:                                          # a transposed view swaps the roles of the axes
        out = torch.empty(shape[axis], dtype=torch.int64, device="cuda")
        B.argmax_axis(xt.t(), axis, out)
        assert np.array_equal(host(out), O.argmax_axis(x.T, axis))
    kd = torch.empty([1 if d == axis % len(shape) else n for d, n in enumerate(shape)], dtype=torch.int64, device="cuda")
    B.argmax_axis(xt, axis, kd, keepdims=True)
    assert np.array_equal(host(kd), O.argmax_axis(x, axis, keepdims=True))


def test_argmax_is_the_accuracy_of_a_classifier_and_its_errors():
    logits = rnd((1024, 10))
    labels = RNG.integers(0, 10, 1024)
    out = torch.empty(1024, dtype=torch.int64, device="cuda")
    B.argmax_axis(dev(logits), 1, out)
    assert float((out.cpu().numpy() == labels).mean()) == float((O.argmax_axis(logits, 1) == labels).mean())
    for bad_out, axis, status in ((torch.empty(1024, device="cuda"), 1, -3), (torch.empty(10, dtype=torch.int64, device="cuda"), 1, -4),
                                  (out, 2, -7)):
        with pytest.raises(B.ChnError) as e:
            B.argmax_axis(dev(logits), axis, bad_out)
        assert e.value.status == status
    with pytest.raises(B.ChnError):
        B.argmax_axis(torch.empty(4, 0, device="cuda"), 1, torch.empty(4, dtype=torch.int64, device="cuda"))
