"""Pins for the CPU oracle: it is checked against things other than itself before any GPU result is
compared with it -- values/formulas the paper prints, closed forms, invariants, brute force on tiny
inputs, central finite differences for every backward, and NumPy/SciPy special cases (the paper
defines the array layer as NumPy-compatible, Section "GPU Support by CuPy")."""
import math
import os

import numpy as np
import pytest
import scipy.special as sps

from oracle import oracle as O
from oracle import steps as OS

GOLD = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(20190800213)


# ---------------------------------------------------------------- values / formulas in the paper
def test_norm_example_from_paper():
    rows = {}
    for line in open(os.path.join(GOLD, "norm_example.txt")):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":")
        rows[k.strip()] = [float(t) for t in v.split()]
    x = np.array(rows["x"])
    sq = O.elementwise("mul", [x, x])
    s = O.reduce_axis("sum", sq, 0)
    assert s == rows["sum_of_squares"][0] == 5.0
    n = O.elementwise("sqrt", [s.reshape(1)])[0]
    assert abs(n - rows["norm"][0]) < 1e-15
    assert abs(n - np.linalg.norm(x)) < 1e-15


def test_my_mad_from_paper():
    rows = np.array([[float(t) for t in line.split()] for line in open(os.path.join(GOLD, "my_mad.txt"))
                     if not line.startswith("#") and line.strip()])
    w = O.elementwise("mad", [rows[:, 0], rows[:, 1], rows[:, 2]])
    assert np.array_equal(w, rows[:, 3])
    assert np.array_equal(O.elementwise("mad_relu", [rows[:, 0], rows[:, 1], rows[:, 2]]),
                          np.maximum(rows[:, 3], 0))


# ---------------------------------------------------------------- broadcasting / strides vs NumPy
@pytest.mark.parametrize("shapes", [
    [(4, 5), (4, 5), (1, 5)], [(4, 5), (4, 1), (5,)], [(3, 1, 5), (1, 4, 1), (4, 5)],
    [(2, 3, 4, 5), (5,), ()], [(6,), (1,), (6,)], [(0, 5), (1, 5), (5,)],
])
def test_broadcast_matches_numpy(shapes):
    xs = [RNG.standard_normal(s) for s in shapes]
    want = xs[0] * xs[1] + xs[2]
    got = O.elementwise("mad", xs)
    assert got.shape == want.shape
    assert np.array_equal(got, want)
    # broadcast result == result on materialised tiles
    full = [np.ascontiguousarray(np.broadcast_to(x, want.shape)) for x in xs]
    assert np.array_equal(got, O.elementwise("mad", full))


def test_broadcast_rejects_mismatch():
    with pytest.raises(ValueError):
        O.elementwise("add", [np.zeros((4, 5)), np.zeros((4, 3))], out_shape=(4, 5))


def test_transposed_view_equals_materialised_transpose():
    a = RNG.standard_normal((7, 9)).astype(np.float32)
    b = RNG.standard_normal((9, 7)).astype(np.float32)
    c = RNG.standard_normal((1, 7)).astype(np.float32)
    got = O.elementwise("mad_relu", [a.T, b, c])
    want = O.elementwise("mad_relu", [np.ascontiguousarray(a.T), b, c])
    assert np.array_equal(got, want)
    assert np.array_equal(got, np.maximum(a.T.astype(np.float64) * b + c, 0))
    # strided slice views too
    big = RNG.standard_normal((10, 12))
    v = big[1:9:2, 2:11:3]
    assert np.array_equal(O.elementwise("copy", [v]), v)


@pytest.mark.parametrize("name,ref", [
    ("add", lambda x, y: x + y), ("sub", lambda x, y: x - y), ("mul", lambda x, y: x * y),
    ("add_relu", lambda x, y: np.maximum(x + y, 0)),
    ("relu_bwd", lambda gy, y: gy * (y > 0)),
])
def test_binary_ops_vs_numpy(name, ref):
    x, y = RNG.standard_normal((5, 6)), RNG.standard_normal((5, 6))
    assert np.array_equal(O.elementwise(name, [x, y]), ref(x, y))


def test_unary_ops_vs_library():
    x = RNG.standard_normal(200) * 3
    assert np.array_equal(O.elementwise("relu", [x]), np.maximum(x, 0))
    assert np.allclose(O.elementwise("sigmoid", [x]), sps.expit(x), rtol=1e-15, atol=0)
    assert np.allclose(O.elementwise("tanh", [x]), np.tanh(x), rtol=1e-15, atol=0)
    want = 0.5 * x * (1 + sps.erf(x / math.sqrt(2)))
    assert np.allclose(O.elementwise("gelu", [x]), want, rtol=1e-14, atol=1e-300)
    assert np.allclose(O.elementwise("gelu", [x]), x * sps.ndtr(x), rtol=1e-9, atol=1e-15)
    assert np.array_equal(O.elementwise("scale", [x], scalars=[2.5]), 2.5 * x)
    assert np.array_equal(O.elementwise("axpy", [x, x[::-1]], scalars=[-0.5]), x + -0.5 * x[::-1])
    assert np.array_equal(O.elementwise("fill", [], out_shape=(3, 2), scalars=[7.0]), np.full((3, 2), 7.0))
    assert O.elementwise("gelu", [np.zeros(1)])[0] == 0.0
    assert O.elementwise("gelu_bwd", [np.ones(1), np.zeros(1)])[0] == 0.5


def test_relu_at_zero_has_zero_gradient():
    y = np.array([0.0, -0.0, 1e-30, -1.0])
    assert np.array_equal(O.elementwise("relu_bwd", [np.ones(4), y]), [0, 0, 1, 0])


# ---------------------------------------------------------------- reductions
@pytest.mark.parametrize("shape,axis", [((5, 7), 0), ((5, 7), 1), ((5, 7), -1), ((3, 4, 5), 1),
                                        ((3, 4, 5), 0), ((1, 6), 0), ((6, 1), 1), ((0, 4), 0), ((4, 0), 1)])
@pytest.mark.parametrize("keep", [False, True])
def test_reduce_vs_bruteforce_and_numpy(shape, axis, keep):
    x = RNG.integers(-4, 5, size=shape).astype(np.float64)  # integers: any order is exact
    got = O.reduce_axis("sum", x, axis, keep)
    assert np.array_equal(got, x.sum(axis=axis, keepdims=keep))
    if x.shape[axis] > 0:
        assert np.array_equal(O.reduce_axis("max", x, axis, keep), x.max(axis=axis, keepdims=keep))
    else:
        assert np.all(O.reduce_axis("max", x, axis, keep) == -np.inf)


def test_reduce_invariants():
    y = RNG.standard_normal((33, 17))
    s0, s1 = O.reduce_axis("sum", y, 0), O.reduce_axis("sum", y, 1)
    assert abs(s0.sum() - s1.sum()) < 1e-12
    assert np.array_equal(O.reduce_axis("sum", y.T, 1), s0)          # transposed view
    assert np.array_equal(O.reduce_axis("sum", np.ones((9, 4)), 0), np.full(4, 9.0))
    with pytest.raises(ValueError):
        O.reduce_axis("sum", y, 2)


# ---------------------------------------------------------------- GEMM
def test_gemm_vs_bruteforce_identity_ones():
    A = RNG.integers(-4, 5, size=(5, 7)).astype(np.float64)
    B = RNG.integers(-4, 5, size=(7, 3)).astype(np.float64)
    want = np.zeros((5, 3))
    for m in range(5):
        for n in range(3):
            for k in range(7):
                want[m, n] += A[m, k] * B[k, n]
    assert np.array_equal(O.gemm(A, B), want)
    assert np.array_equal(O.gemm(A, np.eye(7)), A)
    assert np.array_equal(O.gemm(np.ones((4, 7)), np.ones((7, 6))), np.full((4, 6), 7.0))
    C0 = RNG.integers(-4, 5, size=(5, 3)).astype(np.float64)
    assert np.array_equal(O.gemm(A, B, C0, 2.0, -3.0), 2 * want - 3 * C0)
    assert np.array_equal(O.gemm_entries(A, B, [0, 4, 2], [2, 0, 1]), want[[0, 4, 2], [2, 0, 1]])
    # a transposed operand (the Linear layer's x @ W.T) and a non-commuting check: A@B != (B.T@A.T)
    W = RNG.integers(-4, 5, size=(3, 7)).astype(np.float32)
    assert np.array_equal(O.gemm(A, W.T), A @ W.T.astype(np.float64))
    assert np.array_equal(O.gemm(A.T, A), A.T @ A)
    with pytest.raises(ValueError):
        O.gemm(A, A)


def test_gemm_vs_numpy_random():
    A, B = RNG.standard_normal((13, 29)), RNG.standard_normal((29, 11))
    assert np.allclose(O.gemm(A, B), A @ B, rtol=1e-13, atol=1e-13)


def test_dW_is_sum_of_outer_products():
    dy, x = RNG.standard_normal((6, 4)), RNG.standard_normal((6, 5))
    want = sum(np.outer(dy[n], x[n]) for n in range(6))
    assert np.allclose(O.gemm(dy.T, x), want, rtol=1e-14, atol=1e-14)


# ---------------------------------------------------------------- finite differences
def _fd(f, x, eps=1e-6):
    """Central finite-difference gradient of scalar f at array x (float64)."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        h = eps * max(1.0, abs(x[i]))
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        g[i] = (f(xp) - f(xm)) / (2 * h)
    return g


def _close(a, b, tol=1e-6):
    scale = max(1e-3, float(np.max(np.abs(b))))
    assert float(np.max(np.abs(a - b))) <= tol * scale, (np.max(np.abs(a - b)), scale)


def test_fd_relu_gelu_bwd():
    x = RNG.standard_normal(40)
    x = x[np.abs(x) > 1e-3]
    gy = RNG.standard_normal(x.shape)
    _close(O.elementwise("gelu_bwd", [gy, x]), _fd(lambda v: float(np.dot(gy, O.elementwise("gelu", [v]))), x))
    y = O.elementwise("relu", [x])
    _close(O.elementwise("relu_bwd", [gy, y]), _fd(lambda v: float(np.dot(gy, O.elementwise("relu", [v]))), x))


def test_fd_softmax_ce():
    z = RNG.standard_normal((5, 7))
    t = np.array([0, 6, 3, -1, 2])
    dz = O.softmax_ce_bwd(z, t, -1, 1.7)
    _close(dz, _fd(lambda v: 1.7 * O.softmax_ce_fwd(v, t)[0], z))
    assert np.all(dz[3] == 0)


def test_softmax_ce_closed_forms_and_invariants():
    for Cn in (10, 1000, 10000):
        z = np.zeros((3, Cn))
        t = np.array([0, Cn - 1, Cn // 2])
        loss, rows, lse, nv = O.softmax_ce_fwd(z, t)
        assert abs(loss - math.log(Cn)) < 1e-12 and nv == 3
        dz = O.softmax_ce_bwd(z, t)
        want = np.full((3, Cn), 1.0 / Cn)
        want[np.arange(3), t] -= 1.0
        assert np.allclose(dz, want / 3, rtol=1e-13, atol=1e-16)
    z = RNG.standard_normal((6, 9)) * 5
    t = RNG.integers(0, 9, 6)
    loss, rows, lse, nv = O.softmax_ce_fwd(z, t)
    assert np.allclose(lse, sps.logsumexp(z, axis=1), rtol=1e-14)
    assert np.allclose(rows, -sps.log_softmax(z, axis=1)[np.arange(6), t], rtol=1e-13)
    assert abs(loss - rows.mean()) < 1e-14
    dz = O.softmax_ce_bwd(z, t)
    assert np.max(np.abs(dz.sum(axis=1))) < 1e-16 and abs(dz.sum()) < 1e-15
    p = dz * 6 + np.eye(9)[t]
    assert np.allclose(p.sum(axis=1), 1.0, rtol=1e-14)
    assert np.allclose(p, sps.softmax(z, axis=1), rtol=1e-12)
    # large logits do not overflow; all rows ignored gives zero loss and zero gradient
    assert np.isfinite(O.softmax_ce_fwd(z * 1000, t)[0])
    assert O.softmax_ce_fwd(z, np.full(6, -1))[0] == 0.0
    assert np.all(O.softmax_ce_bwd(z, np.full(6, -1)) == 0.0)
    # label picking is by exact index: moving the label moves the loss to exactly that column
    z2 = np.zeros((1, 4)); z2[0, 2] = 3.0
    l2 = [O.softmax_ce_fwd(z2, np.array([k]))[0] for k in range(4)]
    assert l2[0] == l2[1] == l2[3] and abs((l2[0] - l2[2]) - 3.0) < 1e-15


def test_lstm_closed_form_and_fd():
    B, H = 3, 4
    cp = RNG.standard_normal((B, H))
    c, h, g = O.lstm_fwd(np.zeros((B, 4 * H)), None, cp)
    assert np.array_equal(g[:, :H], np.full((B, H), 0.5)) and np.array_equal(g[:, 2 * H:3 * H], np.zeros((B, H)))
    assert np.allclose(c, 0.5 * cp, rtol=1e-15) and np.allclose(h, 0.5 * np.tanh(0.5 * cp), rtol=1e-15)
    # gate order i,f,g,o: drive one gate block at a time
    z = np.zeros((1, 4)); cp1 = np.array([[2.0]])
    z[0] = [0, 50, 0, 0]          # f -> 1 : c = c_prev
    assert abs(O.lstm_fwd(z, None, cp1)[0][0, 0] - 2.0) < 1e-12
    z[0] = [50, -50, 50, 0]       # i -> 1, f -> 0, g -> 1 : c = 1
    assert abs(O.lstm_fwd(z, None, cp1)[0][0, 0] - 1.0) < 1e-12
    z[0] = [0, 50, 0, -50]        # o -> 0 : h = 0
    assert abs(O.lstm_fwd(z, None, cp1)[1][0, 0]) < 1e-12
    # bias is added to z
    zb, bias = RNG.standard_normal((B, 4 * H)), RNG.standard_normal(4 * H)
    for u, v in zip(O.lstm_fwd(zb, bias, cp), O.lstm_fwd(zb + bias, None, cp)):
        assert np.array_equal(u, v)
    # finite differences of L = <wh, h> + <wc, c> with respect to z and c_prev
    wh, wc = RNG.standard_normal((B, H)), RNG.standard_normal((B, H))

    def L(zz, cc):
        c_, h_, _ = O.lstm_fwd(zz, bias, cc)
        return float((wh * h_).sum() + (wc * c_).sum())
    c_, h_, g_ = O.lstm_fwd(zb, bias, cp)
    dz, dcp = O.lstm_bwd(g_, cp, c_, wh, wc)
    _close(dz, _fd(lambda v: L(v, cp), zb))
    _close(dcp, _fd(lambda v: L(zb, v), cp))
    dz0, _ = O.lstm_bwd(g_, cp, c_, wh, None)
    dz00, _ = O.lstm_bwd(g_, cp, c_, wh, np.zeros((B, H)))
    assert np.array_equal(dz0, dz00)


def test_sgd_closed_forms():
    p, g = RNG.standard_normal(50), RNG.standard_normal(50)
    assert np.array_equal(O.sgd_update(p, g, 0.0), p)
    assert np.array_equal(O.sgd_update(p, np.ones(50), 0.25), p - 0.25)
    assert np.array_equal(O.sgd_update(p, g, 0.01), p - 0.01 * g)


def test_embedding_exact_and_fd():
    E = RNG.standard_normal((6, 3)).astype(np.float32)
    ids = np.array([5, 0, 5, 2, 5])
    out = O.embed_fwd(E, ids)
    assert np.array_equal(out.astype(np.float32), E[ids])      # gathered rows equal the source bits
    dout = RNG.integers(-3, 4, size=(5, 3)).astype(np.float64)
    dE = O.embed_bwd(ids, dout, 6)
    want = np.zeros((6, 3))
    for n, v in enumerate(ids):
        want[v] += dout[n]
    assert np.array_equal(dE, want) and np.all(dE[[1, 3, 4]] == 0)
    assert np.array_equal(O.embed_bwd(ids, dout, 6, np.ones((6, 3))), want + 1)
    w = RNG.standard_normal((5, 3))
    _close(O.embed_bwd(ids, w, 6), _fd(lambda T: float((w * O.embed_fwd(T, ids)).sum()), E.astype(np.float64)))


def test_round_bf16_matches_format_definition():
    import torch
    x = np.concatenate([RNG.standard_normal(2000) * 10.0 ** RNG.integers(-30, 30, 2000),
                        [1.00390625, 1.01171875, -1.00390625, 0.0, 2.0 ** -133, 3.3e38]])
    x32 = x.astype(np.float32)
    got = O.round_bf16(x32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, want)
    assert np.array_equal(O.round_bf16(got), got)               # idempotent
    # ties stated by hand: 1 + 2^-8 lies midway between 1 (even mantissa) and 1 + 2^-7;
    # 1 + 3*2^-8 midway between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    ties = O.round_bf16(np.array([1.00390625, 1.01171875, -1.00390625, -1.01171875, 1.00390625 + 2.0 ** -30, 257.0, 259.0]))
    assert list(ties) == [1.0, 1.015625, -1.0, -1.015625, 1.0078125, 256.0, 260.0]


# ---------------------------------------------------------------- whole steps
def _tiny_mlp(act):
    sizes = (5, 4, 3)
    params = [(RNG.standard_normal((sizes[i + 1], sizes[i])) * 0.7, RNG.standard_normal(sizes[i + 1]) * 0.1)
              for i in range(2)]
    x = RNG.standard_normal((6, 5))
    t = RNG.integers(0, 3, 6)
    return params, x, t


@pytest.mark.parametrize("act", ["relu", "gelu"])
def test_fd_whole_mlp_step(act):
    params, x, t = _tiny_mlp(act)
    r = OS.mlp_step(params, x, t, 0.05, act)
    assert abs(r["loss"] - OS.mlp_loss(params, x, t, act)) < 1e-15
    for l in range(2):
        for j in range(2):
            def f(v, l=l, j=j):
                q = [list(p) for p in params]
                q[l][j] = v
                return OS.mlp_loss([tuple(p) for p in q], x, t, act)
            _close(r["grads"][l][j], _fd(f, params[l][j]), 2e-6)
            assert np.array_equal(r["params"][l][j], params[l][j] - 0.05 * r["grads"][l][j])
    # db equals the axis-0 sum of the upstream gradient; gradient on a batch = mean over its halves
    ra = OS.mlp_step(params, x[:3], t[:3], 0.05, act)
    rb = OS.mlp_step(params, x[3:], t[3:], 0.05, act)
    for l in range(2):
        for j in range(2):
            assert np.allclose(r["grads"][l][j], 0.5 * (ra["grads"][l][j] + rb["grads"][l][j]),
                               rtol=1e-12, atol=1e-14)


def test_mlp_step_lowp_rounds_only_storage():
    params, x, t = _tiny_mlp("gelu")
    x = O.round_bf16(x)
    r32 = OS.mlp_step(params, x, t, 0.05, "gelu", lowp=False)
    r16 = OS.mlp_step(params, x, t, 0.05, "gelu", lowp=True)
    assert abs(r32["loss"] - r16["loss"]) < 3e-2 * max(1.0, abs(r32["loss"]))
    for a in r16["acts"]:
        assert np.array_equal(O.round_bf16(a), a)
    assert r16["loss"] != r32["loss"]


def test_exp_and_second_derivative_of_gelu():
    x = np.linspace(-5, 5, 401)
    assert np.allclose(O.elementwise("exp", [x]), np.exp(x), rtol=1e-15)
    g = RNG.standard_normal(401)
    got = O.elementwise("gelu_bwd2", [g, x])
    # closed form phi(z)(2 - z^2), and the central difference of the pinned first derivative
    phi = np.exp(-0.5 * x * x) / math.sqrt(2 * math.pi)
    assert np.allclose(got, g * phi * (2 - x * x), rtol=1e-13, atol=1e-16)
    one = np.ones_like(x)
    h = 1e-5
    fd = (O.elementwise("gelu_bwd", [one, x + h]) - O.elementwise("gelu_bwd", [one, x - h])) / (2 * h)
    assert np.max(np.abs(got - g * fd)) < 1e-8
    assert O.elementwise("gelu_bwd2", [np.ones(1), np.zeros(1)])[0] == pytest.approx(2 / math.sqrt(2 * math.pi), rel=1e-15)


def test_fd_softmax_ce_second_order():
    # <u, G(z, g)> with G the (pinned) first-order gradient: its derivatives by central differences
    z = RNG.standard_normal((6, 5))
    t = RNG.integers(0, 5, 6)
    t[2] = -1
    u = RNG.standard_normal((6, 5))
    g0 = 1.7
    dz, dg = O.softmax_ce_bwd2(z, t, u, -1, g0)
    _close(dz, _fd(lambda v: float((u * O.softmax_ce_bwd(v, t, -1, g0)).sum()), z), 2e-6)
    h = 1e-5
    fd = ((u * O.softmax_ce_bwd(z, t, -1, g0 + h)).sum() - (u * O.softmax_ce_bwd(z, t, -1, g0 - h)).sum()) / (2 * h)
    assert abs(dg - fd) < 1e-8
    assert np.all(dz[2] == 0) and np.max(np.abs(dz.sum(axis=1))) < 1e-15      # rows of p (u - p.u) sum to zero
    # zero logits: p = 1/C, so dz = (g / N_valid) (u - mean(u)) / C
    dz0, _ = O.softmax_ce_bwd2(np.zeros((6, 5)), t, u, -1, g0)
    want = g0 / 5 * (u - u.mean(axis=1, keepdims=True)) / 5
    want[2] = 0
    assert np.allclose(dz0, want, rtol=1e-13, atol=1e-16)


def test_stray_indices_are_ignored_not_followed():
    # a label outside [0, C) behaves exactly like the ignore label; an id outside [0, V) gathers zeros and
    # takes part in no gradient sum -- checked against the same problem with those rows marked / removed
    z = RNG.standard_normal((9, 5))
    t = RNG.integers(0, 5, 9)
    stray, marked = t.copy(), t.copy()
    stray[[1, 4, 7]] = [5, -100, 2 ** 40]
    marked[[1, 4, 7]] = -1
    a, b = O.softmax_ce_fwd(z, stray), O.softmax_ce_fwd(z, marked)
    assert a[0] == b[0] and np.array_equal(a[1], b[1]) and a[3] == b[3] == 6
    assert np.array_equal(O.softmax_ce_bwd(z, stray, -1, 2.0), O.softmax_ce_bwd(z, marked, -1, 2.0))
    keep = [0, 2, 3, 5, 6, 8]
    assert abs(a[0] - O.softmax_ce_fwd(z[keep], t[keep])[0]) < 1e-15
    E = RNG.standard_normal((6, 3))
    ids = np.array([0, 6, 5, -1, 2, 10 ** 12])
    out = O.embed_fwd(E, ids)
    assert np.array_equal(out[[0, 2, 4]], E[[0, 5, 2]]) and np.all(out[[1, 3, 5]] == 0)
    w = RNG.standard_normal((6, 3))
    assert np.array_equal(O.embed_bwd(ids, w, 6), O.embed_bwd(ids[[0, 2, 4]], w[[0, 2, 4]], 6))


# ---- the mixed-precision ("lowp") branches: WHERE the steps round to bfloat16 ---------------------------
# The scheme (weights: fp32 master + bf16 working copy; activations and activation gradients bf16;
# dW, db, logits, loss, cell state, gates and masters wide) is checked three ways: which arrays are
# bf16-exact and which are not, the identity when the rounding is switched off, and a tiny case
# composed here from plain NumPy / SciPy with a rounding written independently of the oracle's.
def _is_bf16(a):
    a = np.asarray(a, dtype=np.float64)
    return bool(np.array_equal(O.round_bf16(a), a))


def _rne_bf16(a):
    """bfloat16 rounding from the format's definition, without the oracle's C routine: scale the value
    so that eight significant bits sit left of the point, round half to even (Python's round), scale back."""
    out = np.empty(np.shape(a), dtype=np.float64)
    flat, src = out.reshape(-1), np.asarray(a, dtype=np.float64).reshape(-1)
    for i, v in enumerate(src):
        if v == 0.0:
            flat[i] = 0.0
            continue
        _, e = math.frexp(v)                     # |v| = f * 2^e, f in [0.5, 1)
        flat[i] = float(round(v * 2.0 ** (8 - e))) * 2.0 ** (e - 8)
    return out


def _softmax_grad(z, t):
    p = sps.softmax(z, axis=1)
    p[np.arange(len(t)), t] -= 1.0
    return p / len(t)


def _gelu(v):
    return 0.5 * v * (1.0 + sps.erf(v / math.sqrt(2.0)))


def _gelu_grad(v):
    return 0.5 * (1.0 + sps.erf(v / math.sqrt(2.0))) + v * np.exp(-0.5 * v * v) / math.sqrt(2.0 * math.pi)


@pytest.mark.parametrize("act", ["relu", "gelu"])
def test_mlp_step_lowp_storage_points(act, monkeypatch):
    sizes = (7, 6, 5, 4)
    params = [(RNG.standard_normal((sizes[i + 1], sizes[i])) * 0.6, RNG.standard_normal(sizes[i + 1]) * 0.1) for i in range(3)]
    x = O.round_bf16(RNG.standard_normal((9, 7)))
    t = RNG.integers(0, 4, 9)
    r = OS.mlp_step(params, x, t, 0.05, act, lowp=True)
    st = r["stored"]
    # bf16-stored: working copies, activations, retained pre-activations, every activation gradient
    for name in ("Wc", "acts", "zs", "dvs"):
        assert len(st[name]) >= 2
        for a in st[name]:
            assert _is_bf16(a), name
    # kept wide: logits, weight and bias gradients, input gradients before the activation derivative, new masters
    wide = [r["logits"]] + [g for pair in r["grads"] for g in pair] + [p for pair in r["params"] for p in pair] + [d for d in r["dhs"] if d is not None]
    for a in wide:
        assert not _is_bf16(a)
    # masters are updated from the masters (not from the rounded copies) with the unrounded gradients
    for (W, b), (dW, db), (Wn, bn) in zip(params, r["grads"], r["params"]):
        assert np.array_equal(Wn, W - 0.05 * dW) and np.array_equal(bn, b - 0.05 * db)
    # composed by hand from NumPy / SciPy with an independent rounding
    Wc = [_rne_bf16(W) for W, _ in params]
    h, hs, zs = x, [x], []
    for l in range(2):
        v = h @ Wc[l].T + params[l][1]
        zs.append(_rne_bf16(v))
        h = _rne_bf16(np.maximum(v, 0.0) if act == "relu" else _gelu(v))      # activation of the UNROUNDED v
        hs.append(h)
    logits = h @ Wc[2].T + params[2][1]
    np.testing.assert_allclose(r["logits"], logits, rtol=1e-13, atol=1e-14)
    dv = _rne_bf16(_softmax_grad(logits, t))
    for l in (2, 1, 0):
        np.testing.assert_allclose(r["grads"][l][0], dv.T @ hs[l], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(r["grads"][l][1], dv.sum(0), rtol=1e-12, atol=1e-15)
        assert np.array_equal(st["dvs"][l], dv)                                 # same bf16 values, bit for bit
        if l > 0:
            dh = dv @ Wc[l]
            # the derivative is taken from what was STORED: the bf16 output (ReLU) or the bf16 pre-activation (GELU)
            dv = _rne_bf16(dh * (hs[l] > 0) if act == "relu" else dh * _gelu_grad(zs[l - 1]))
    for l in range(2):
        assert np.array_equal(st["acts"][l], hs[l + 1]) and np.array_equal(st["zs"][l], zs[l])
    # with the rounding switched off the lowp step IS the fp64 step
    monkeypatch.setattr(OS, "ROUND", lambda a: a)
    a, b = OS.mlp_step(params, x, t, 0.05, act, lowp=True), OS.mlp_step(params, x, t, 0.05, act, lowp=False)
    assert a["loss"] == b["loss"] and np.array_equal(a["logits"], b["logits"])
    for (aW, ab), (bW, bb) in zip(a["grads"] + a["params"], b["grads"] + b["params"]):
        assert np.array_equal(aW, bW) and np.array_equal(ab, bb)


def test_mlp_step_lowp_one_layer_by_hand():
    # 2 x 2, one layer, numbers small enough to follow: the working copy rounds 1 + 2^-8 down to 1 and
    # 1 + 3*2^-8 up to 1 + 2^-6; logits are x Wc^T + b, unrounded
    W = np.array([[1.00390625, 0.5], [1.01171875, -0.25]])
    b = np.array([0.125, 0.0])
    x = np.array([[1.0, 2.0], [3.0, -1.0]])
    t = np.array([0, 1])
    r = OS.mlp_step([(W, b)], x, t, 0.5, "relu", lowp=True)
    Wc = np.array([[1.0, 0.5], [1.015625, -0.25]])
    assert np.array_equal(r["stored"]["Wc"][0], Wc)
    logits = np.array([[1.0 + 1.0 + 0.125, 1.015625 - 0.5], [3.0 - 0.5 + 0.125, 3.046875 + 0.25]])
    assert np.array_equal(r["logits"], logits)
    p = np.exp(logits) / np.exp(logits).sum(1, keepdims=True)
    dz = (p - np.eye(2)[t]) / 2.0
    dv = _rne_bf16(dz)
    assert np.array_equal(r["stored"]["dvs"][0], dv) and not np.array_equal(dv, dz)
    np.testing.assert_allclose(r["grads"][0][0], dv.T @ x, rtol=1e-15)
    np.testing.assert_allclose(r["params"][0][0], W - 0.5 * (dv.T @ x), rtol=1e-15)     # from the master W, not from Wc
    assert abs(r["loss"] - float(np.mean(-np.log(p[np.arange(2), t])))) < 1e-15


def _tiny_lm(scale=0.5):
    V, E, H, B, T = 7, 3, 4, 2, 3
    P = {"E": RNG.standard_normal((V, E)), "W": RNG.standard_normal((E, 4 * H)) * scale,
         "U": RNG.standard_normal((H, 4 * H)) * scale, "b": RNG.standard_normal(4 * H) * 0.1,
         "W_out": RNG.standard_normal((V, H)) * scale, "b_out": RNG.standard_normal(V) * 0.1}
    ids = np.array([[1, 1], [3, 1], [1, 6]])
    return P, ids, RNG.integers(0, V, (T, B))


def test_lstm_lm_step_lowp_storage_points(monkeypatch):
    P, ids, tg = _tiny_lm()
    T, B = ids.shape
    H, V = 4, 7
    r = OS.lstm_lm_step(P, ids, tg, 0.1, lowp=True)
    st, un = r["stored"], r["unrounded"]
    # bf16-stored: what feeds a product
    for k in ("E", "W", "U", "W_out"):
        assert _is_bf16(st["Wc"][k]) and not _is_bf16(P[k])
    for name in ("X", "Hall", "dlogits", "dHall", "dZ"):
        assert _is_bf16(st[name]), name
    assert all(_is_bf16(d) for d in st["dH"])
    # kept wide: gate pre-activations, gates, cell state and its gradient, logits, dX, parameter gradients, masters
    for a in [un["Zx"], un["dX"], r["logits"]] + un["Gs"] + un["Cs"] + un["dC"] + list(r["grads"].values()) + list(r["params"].values()):
        assert not _is_bf16(a)
    for k in r["grads"]:
        assert np.array_equal(r["params"][k], P[k] - 0.1 * r["grads"][k])
    # composed by hand (NumPy / SciPy, independent rounding), same storage points
    Wc = {k: _rne_bf16(P[k]) for k in ("E", "W", "U", "W_out")}
    X = Wc["E"][ids.reshape(-1)]
    Zx = X @ Wc["W"]
    h, c = np.zeros((B, H)), np.zeros((B, H))
    Hp, Cp, Cs, Gs, Hs = [], [], [], [], []
    for s in range(T):
        z = Zx[s * B:(s + 1) * B] + h @ Wc["U"] + P["b"]
        i, f, g, o = sps.expit(z[:, :H]), sps.expit(z[:, H:2 * H]), np.tanh(z[:, 2 * H:3 * H]), sps.expit(z[:, 3 * H:])
        Hp.append(h); Cp.append(c)
        c = f * c + i * g
        h = _rne_bf16(o * np.tanh(c))                 # h is stored in bf16, c is not
        Cs.append(c); Gs.append((i, f, g, o)); Hs.append(h)
    Hall = np.concatenate(Hs)
    logits = Hall @ Wc["W_out"].T + P["b_out"]
    np.testing.assert_allclose(r["logits"], logits, rtol=1e-12, atol=1e-14)
    assert np.array_equal(st["Hall"], Hall)
    dlog = _rne_bf16(_softmax_grad(logits, tg.reshape(-1)))
    assert np.array_equal(st["dlogits"], dlog)
    dHall = _rne_bf16(dlog @ Wc["W_out"])
    dZ = np.zeros((T * B, 4 * H))
    dc, rec = np.zeros((B, H)), None
    for s in range(T - 1, -1, -1):
        dh = dHall[s * B:(s + 1) * B]
        if rec is not None:
            dh = _rne_bf16(dh + rec)                  # rounded again once the recurrent part is in
        i, f, g, o = Gs[s]
        tc = np.tanh(Cs[s])
        dct = dc + dh * o * (1 - tc * tc)
        dz = np.concatenate([dct * g * i * (1 - i), dct * Cp[s] * f * (1 - f), dct * i * (1 - g * g), dh * tc * o * (1 - o)], axis=1)
        dc = dct * f                                  # the cell-state gradient is never rounded
        dz = _rne_bf16(dz)
        dZ[s * B:(s + 1) * B] = dz
        rec = dz @ Wc["U"].T
    assert np.array_equal(st["dZ"], dZ)
    np.testing.assert_allclose(r["grads"]["U"], np.concatenate(Hp).T @ dZ, rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(r["grads"]["W"], X.T @ dZ, rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(r["grads"]["b"], dZ.sum(0), rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(r["grads"]["W_out"], dlog.T @ Hall, rtol=1e-11, atol=1e-15)
    dE = np.zeros((V, 3))
    np.add.at(dE, ids.reshape(-1), dZ @ Wc["W"].T)    # dX itself is not rounded
    np.testing.assert_allclose(r["grads"]["E"], dE, rtol=1e-11, atol=1e-15)
    # rounding switched off: the lowp step is the fp64 step, bit for bit
    monkeypatch.setattr(OS, "ROUND", lambda a: a)
    a, b = OS.lstm_lm_step(P, ids, tg, 0.1, lowp=True), OS.lstm_lm_step(P, ids, tg, 0.1, lowp=False)
    assert a["loss"] == b["loss"]
    for k in a["grads"]:
        assert np.array_equal(a["grads"][k], b["grads"][k]) and np.array_equal(a["params"][k], b["params"][k])


def test_fd_lstm_lm_step_bptt():
    V, E, H, B, T = 7, 3, 4, 2, 3
    P = {"E": RNG.standard_normal((V, E)), "W": RNG.standard_normal((E, 4 * H)) * 0.5,
         "U": RNG.standard_normal((H, 4 * H)) * 0.5, "b": RNG.standard_normal(4 * H) * 0.1,
         "W_out": RNG.standard_normal((V, H)) * 0.5, "b_out": RNG.standard_normal(V) * 0.1}
    ids = np.array([[1, 1], [3, 1], [1, 6]])          # repeated ids: embedding rows collide
    tg = RNG.integers(0, V, (T, B))
    r = OS.lstm_lm_step(P, ids, tg, 0.1)
    for k in P:
        def f(v, k=k):
            Q = dict(P)
            Q[k] = v
            return OS.lstm_lm_forward(Q, ids, tg)["loss"]
        _close(r["grads"][k], _fd(f, P[k]), 5e-6)
        assert np.array_equal(r["params"][k], P[k] - 0.1 * r["grads"][k])
    # topology changes with the trace: another window length still gives correct gradients
    r2 = OS.lstm_lm_step(P, ids[:2], tg[:2], 0.1)
    _close(r2["grads"]["U"], _fd(lambda v: OS.lstm_lm_forward({**P, "U": v}, ids[:2], tg[:2])["loss"], P["U"]), 5e-6)


def test_adam_first_step_is_a_signed_step_and_constant_gradients_keep_it_so():
    # with zero state the corrected moments after step 1 are g and g^2: the move is lr * g / (|g| + eps);
    # a gradient that never changes keeps m_hat = g and v_hat = g^2 at every step
    rng = np.random.default_rng(21)
    p0, g = rng.standard_normal(50), rng.standard_normal(50)
    p, m, v = p0, np.zeros(50), np.zeros(50)
    for t in range(1, 6):
        p_new, m, v = O.adam_update(p, g, m, v, 0.01, t, 0.9, 0.999, 1e-8)
        np.testing.assert_allclose(p_new, p - 0.01 * g / (np.abs(g) + 1e-8), rtol=1e-12, atol=1e-15)
        p = p_new
    np.testing.assert_allclose(m, (1 - 0.9 ** 5) * g, rtol=1e-12)
    np.testing.assert_allclose(v, (1 - 0.999 ** 5) * g * g, rtol=1e-12)


def test_adam_two_steps_by_hand():
    # beta1 = beta2 = 0.5, lr = 1, eps = 0, gradients 2 then -4 on a single parameter
    p, m, v = O.adam_update(np.array([10.0]), np.array([2.0]), np.zeros(1), np.zeros(1), 1.0, 1, 0.5, 0.5, 0.0)
    assert (p[0], m[0], v[0]) == (9.0, 1.0, 2.0)
    p, m, v = O.adam_update(p, np.array([-4.0]), m, v, 1.0, 2, 0.5, 0.5, 0.0)
    # m = 0.5 - 2 = -1.5, v = 1 + 8 = 9; m_hat = -2, v_hat = 12
    assert (m[0], v[0]) == (-1.5, 9.0)
    assert p[0] == pytest.approx(9.0 + 2.0 / np.sqrt(12.0), rel=1e-15)


def test_argmax_first_of_equal_maxima_by_brute_force():
    rng = np.random.default_rng(33)
    x = rng.integers(0, 4, (5, 6, 7)).astype(np.float64)         # many ties
    for axis in (0, 1, 2, -1):
        got = O.argmax_axis(x, axis)
        assert np.array_equal(got, np.argmax(x, axis=axis))      # NumPy documents the first-occurrence rule
        moved = np.moveaxis(x, axis, -1)
        for pos in np.ndindex(moved.shape[:-1]):
            row = list(moved[pos])
            assert got[pos] == row.index(max(row))
    assert O.argmax_axis(x, 1, keepdims=True).shape == (5, 1, 7)
