"""Host logic of the define-by-run tape, run on the CPU with the oracle's functions as kernels.

What is pinned here, against things other than the tape itself:
* gradients against central finite differences of the forward value (every function, graphs with a
  variable used twice, a diamond, shared weights over time);
* whole steps against the hand-ordered oracle steps (same kernels, so equality up to the order of
  gradient accumulation);
* the memory rules of Sections "Global Memory Usage Reduction" and "Function-wise Local Memory
  Usage Reduction": what each function retains, that every function node is cut out by backward,
  that arrays die as soon as nothing needs them;
* the traversal order of Section "On Demand Graph Construction": each function node's backward
  runs once, after those of all its consumers.
"""
import gc
import weakref

import numpy as np
import pytest

from oracle import oracle as O
from oracle import steps as OS
from paper_1908_00213_amd import tape as T
from paper_1908_00213_amd import workloads as W
from tests.oracle_backend import OracleBackend


@pytest.fixture
def F():
    with T.using_backend(OracleBackend()) as b:
        yield b


def fd_grad(f, arrays, eps=1e-6):
    """Central differences of the scalar f() with respect to every entry of every array (in place)."""
    out = []
    for a in arrays:
        g = np.zeros_like(a)
        it = np.nditer(a, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = a[i]
            a[i] = old + eps
            hi = f()
            a[i] = old - eps
            lo = f()
            a[i] = old
            g[i] = (hi - lo) / (2 * eps)
        out.append(g)
    return out


def rnd(rng, *shape):
    return rng.standard_normal(shape)


# ---- gradients against finite differences -----------------------------------------------------------
@pytest.mark.parametrize("act", [None, "relu", "gelu"])
def test_linear_with_fused_activation_matches_finite_differences(F, act):
    rng = np.random.default_rng(1)
    x, Wm, b, t = rnd(rng, 5, 4), rnd(rng, 3, 4), rnd(rng, 3), np.array([0, 2, 1, 1, 0])

    def loss(record=False):
        xs = [T.Variable(x), T.Parameter(Wm), T.Parameter(b)]
        l = T.softmax_cross_entropy(T.linear(*xs, act=act), t)
        return (l, xs) if record else float(l.array)

    l, xs = loss(True)
    l.backward()
    for v, g in zip(xs, fd_grad(loss, [x, Wm, b])):
        np.testing.assert_allclose(v.grad, g, rtol=1e-6, atol=1e-8)


def test_variable_used_twice_and_diamond_accumulate(F):
    rng = np.random.default_rng(2)
    x, Wa, Wb, t = rnd(rng, 4, 3), rnd(rng, 3, 3), rnd(rng, 3, 3), np.array([2, 0, 1, 1])

    def loss(record=False):
        xv, A, Bv = T.Variable(x), T.Parameter(Wa), T.Parameter(Wb)
        h = T.gelu(T.matmul(xv, A))                    # h feeds three consumers
        y = T.add(T.add(T.matmul(h, Bv), T.relu(h)), T.matmul(h, A))   # A used twice
        l = T.softmax_cross_entropy(y, t)
        return (l, [xv, A, Bv]) if record else float(l.array)

    l, vs = loss(True)
    l.backward()
    for v, g in zip(vs, fd_grad(loss, [x, Wa, Wb])):
        np.testing.assert_allclose(v.grad, g, rtol=1e-6, atol=1e-8)


def test_lstm_language_model_matches_finite_differences_and_oracle_step(F):
    w = W.config4(seed=5, vocab=11, embed=3, hidden=4, batch=2, bptt=3)
    P = {k: v.astype(np.float64) for k, v in w.params.items()}
    P["b"] = np.random.default_rng(3).standard_normal(P["b"].shape) * 0.1
    ids, tg = w.ids.reshape(-1).astype(np.int64), w.targets.reshape(-1).astype(np.int64)

    model = T.LSTMLanguageModel(P)
    loss, _ = model.loss(ids, tg, w.bptt)
    loss.backward()
    ref = OS.lstm_lm_step(P, w.ids, w.targets, 0.1)
    assert float(loss.array) == pytest.approx(ref["loss"], rel=1e-13)
    for k, p in model.P.items():
        np.testing.assert_allclose(p.grad, ref["grads"][k], rtol=1e-10, atol=1e-13, err_msg=k)

    def f():
        with T.no_backprop_mode():
            return float(T.LSTMLanguageModel(P).loss(ids, tg, w.bptt)[0].array)

    for k in ("U", "b", "W"):
        g, = fd_grad(f, [P[k]])
        np.testing.assert_allclose(model.P[k].grad, g, rtol=2e-5, atol=1e-8, err_msg=k)
    # the optimiser applies the oracle's update to every parameter once
    T.SGD(model.params(), 0.1).update()
    for k in P:
        np.testing.assert_allclose(P[k], ref["params"][k], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("fuse", [False, True])
def test_n_step_lstm_mixed_precision_code_path(F, fuse):
    """The bf16-storage variant walks different calls (working copies of the parameters, the fused
    backward step).  On the oracle backend nothing is rounded, so it must reproduce the fp32 step."""
    F.fuse_lstm_step = fuse
    w = W.config4(seed=8, vocab=13, embed=3, hidden=4, batch=2, bptt=4)
    P = {k: v.astype(np.float64) for k, v in w.params.items()}
    P["b"] = np.random.default_rng(6).standard_normal(P["b"].shape) * 0.1
    ids, tg = w.ids.reshape(-1).astype(np.int64), w.targets.reshape(-1).astype(np.int64)
    ref = OS.lstm_lm_step(P, w.ids, w.targets, 0.1)
    model = T.LSTMLanguageModel({k: v.copy() for k, v in P.items()}, n_step=True, lowp=True)
    assert all((model.P[k].lowp is not None) == (k in ("E", "W", "U", "W_out")) for k in P)
    F.calls.clear()
    loss, _ = model.loss(ids, tg, w.bptt)
    loss.backward()
    names = [n for n, _ in F.calls]
    assert (names.count("lstm_step_bwd") == w.bptt) == fuse and (names.count("lstm_bwd") == w.bptt) != fuse
    assert float(loss.array) == pytest.approx(ref["loss"], rel=1e-13)
    for k, p in model.P.items():
        np.testing.assert_allclose(p.grad, ref["grads"][k], rtol=1e-10, atol=1e-13, err_msg=k)
    with pytest.raises(ValueError):
        T.LSTMLanguageModel(P, n_step=False, lowp=True)


@pytest.mark.parametrize("fuse", [False, True])
def test_n_step_lstm_equals_the_oracle_step_and_the_step_by_step_graph(F, fuse):
    """One function node for all time steps: same loss and gradients as the hand-ordered oracle step
    and as the graph of per-step nodes, with far fewer nodes; both forward code paths (one call per
    step where the backend fuses product and cell, two otherwise)."""
    F.fuse_lstm_step = fuse
    w = W.config4(seed=7, vocab=13, embed=3, hidden=4, batch=2, bptt=4)
    P = {k: v.astype(np.float64) for k, v in w.params.items()}
    P["b"] = np.random.default_rng(4).standard_normal(P["b"].shape) * 0.1
    ids, tg = w.ids.reshape(-1).astype(np.int64), w.targets.reshape(-1).astype(np.int64)
    ref = OS.lstm_lm_step(P, w.ids, w.targets, 0.1)

    model = T.LSTMLanguageModel({k: v.copy() for k, v in P.items()}, n_step=True)
    F.calls.clear()
    loss, (c, h) = model.loss(ids, tg, w.bptt)
    fwd_calls = [n for n, _ in F.calls]
    assert ("lstm_step_fwd" in fwd_calls) == fuse and fwd_calls.count("lstm_step_fwd" if fuse else "lstm_fwd") == w.bptt
    assert T.live_function_nodes() == 5               # embedding, input product, recurrent layer, output layer, loss
    loss.backward()
    assert float(loss.array) == pytest.approx(ref["loss"], rel=1e-13)
    for k, p in model.P.items():
        np.testing.assert_allclose(p.grad, ref["grads"][k], rtol=1e-10, atol=1e-13, err_msg=k)
    assert not T.live_function_nodes()

    stepwise = T.LSTMLanguageModel({k: v.copy() for k, v in P.items()})
    l2, (c2, h2) = stepwise.loss(ids, tg, w.bptt)
    l2.backward()
    np.testing.assert_allclose(c.array, c2.array, rtol=1e-13)
    np.testing.assert_allclose(h.array, h2.array, rtol=1e-13)
    for k in P:
        np.testing.assert_allclose(model.P[k].grad, stepwise.P[k].grad, rtol=1e-10, atol=1e-13, err_msg=k)


def test_padded_lstm_parameters_are_inert():
    """Rounding the widths up with zero weights changes neither the loss nor the gradients of the real
    entries, and the added entries get zero gradients (checked on the hand-ordered oracle step)."""
    w = W.config4(seed=9, vocab=17, embed=5, hidden=6, batch=3, bptt=4)
    w.params["b"] = (np.random.default_rng(5).standard_normal(w.params["b"].shape) * 0.1).astype(np.float32)
    Pp = W.pad_lstm_params(w.params, multiple=8)
    assert Pp["U"].shape == (8, 32) and Pp["W"].shape == (8, 32) and Pp["E"].shape == (17, 8)
    a = OS.lstm_lm_step(w.params, w.ids, w.targets, 0.1)
    b = OS.lstm_lm_step(Pp, w.ids, w.targets, 0.1)
    assert b["loss"] == pytest.approx(a["loss"], rel=1e-13)
    E, H = 5, 6
    real = {"E": lambda g: g[:, :E], "W": lambda g: g.reshape(8, 4, 8)[:E, :, :H].reshape(E, 4 * H),
            "U": lambda g: g.reshape(8, 4, 8)[:H, :, :H].reshape(H, 4 * H), "b": lambda g: g.reshape(4, 8)[:, :H].reshape(4 * H),
            "W_out": lambda g: g[:, :H], "b_out": lambda g: g}
    for k in a["grads"]:
        np.testing.assert_allclose(real[k](b["grads"][k]), a["grads"][k], rtol=1e-12, atol=1e-15, err_msg=k)
        assert abs(b["grads"][k]).sum() == pytest.approx(abs(a["grads"][k]).sum(), rel=1e-12)   # nothing outside


def test_n_step_lstm_gradients_of_state_and_every_output_by_finite_differences(F):
    """All three outputs used, a non-zero initial state that needs gradients, and a second consumer of
    the stacked hidden states: checked against central differences of the forward value."""
    rng = np.random.default_rng(21)
    Tn, Bn, H = 3, 2, 3
    c0, h0 = rng.standard_normal((Bn, H)) * 0.5, rng.standard_normal((Bn, H)) * 0.5
    zx, U, b = rng.standard_normal((Tn * Bn, 4 * H)), rng.standard_normal((H, 4 * H)) * 0.4, rng.standard_normal(4 * H) * 0.1
    wc, wh, ws = rng.standard_normal((Bn, H)), rng.standard_normal((Bn, H)), rng.standard_normal((Tn * Bn, H))

    def value(vs):
        c, h, hs = T.n_step_lstm(*vs, Tn)
        return T.add(T.add(T.sum_all(T.mul(c, T.Variable(wc, requires_grad=False))),
                           T.sum_all(T.mul(h, T.Variable(wh, requires_grad=False)))),
                     T.add(T.sum_all(T.mul(hs, T.Variable(ws, requires_grad=False))), T.sum_all(T.mul(hs, hs))))

    vs = [T.Variable(a) for a in (c0, h0, zx, U, b)]
    value(vs).backward()

    def f():
        with T.no_backprop_mode():
            return float(value([T.Variable(a) for a in (c0, h0, zx, U, b)]).array)

    for v, g, name in zip(vs, fd_grad(f, [c0, h0, zx, U, b]), ("c0", "h0", "zx", "U", "b")):
        np.testing.assert_allclose(v.grad, g, rtol=2e-6, atol=1e-8, err_msg=name)
    # only the last hidden state used: the other two gradients arrive as None
    vs = [T.Variable(a) for a in (c0, h0, zx, U, b)]
    T.sum_all(T.mul(T.n_step_lstm(*vs, Tn)[1], T.Variable(wh, requires_grad=False))).backward()

    def f2():
        with T.no_backprop_mode():
            return float(T.sum_all(T.mul(T.n_step_lstm(*[T.Variable(a) for a in (c0, h0, zx, U, b)], Tn)[1],
                                         T.Variable(wh, requires_grad=False))).array)

    for v, g, name in zip(vs, fd_grad(f2, [c0, h0, zx, U, b]), ("c0", "h0", "zx", "U", "b")):
        np.testing.assert_allclose(v.grad, g, rtol=2e-6, atol=1e-8, err_msg=name)


@pytest.mark.parametrize("act,fused", [("relu", True), ("relu", False), ("gelu", True), ("gelu", False)])
def test_mlp_step_equals_the_hand_ordered_oracle_step(F, act, fused):
    w = W.make_mlp("t", (7, 6, 5, 4), 9, act, seed=11)
    params = [(Wm.astype(np.float64), np.random.default_rng(l).standard_normal(b.shape))
              for l, (Wm, b) in enumerate(w.params)]
    ref = OS.mlp_step(params, w.xs[0], w.ts[0], 0.05, act)
    model = T.MLP([(a.copy(), b.copy()) for a, b in params], act, fused_activation=fused)
    opt = T.SGD(model.params(), 0.05)
    loss = model.loss(w.xs[0].astype(np.float64), w.ts[0].astype(np.int64))
    loss.backward()
    assert float(loss.array) == pytest.approx(ref["loss"], rel=1e-14)
    for l, layer in enumerate(model.layers):
        np.testing.assert_allclose(layer.W.grad, ref["grads"][l][0], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(layer.b.grad, ref["grads"][l][1], rtol=1e-12, atol=1e-15)
    opt.update()
    for l, layer in enumerate(model.layers):
        np.testing.assert_allclose(layer.W.array, ref["params"][l][0], rtol=1e-13)
        np.testing.assert_allclose(layer.b.array, ref["params"][l][1], rtol=1e-13, atol=1e-16)
    # the first layer's input is data: no product is spent on its gradient
    n_gemm = sum(1 for c in F.calls if c[0] == "gemm")
    assert n_gemm == 3 + 3 + 2


# ---- topology is whatever the forward code did -------------------------------------------------------
def test_graph_may_change_from_one_iteration_to_the_next(F):
    rng = np.random.default_rng(4)
    Wm, b = rnd(rng, 4, 4) * 0.5, rnd(rng, 4) * 0.1
    x, t = rnd(rng, 3, 4), np.array([1, 3, 0])
    layer = T.Linear(Wm, b)

    def forward(depth):
        h = T.Variable(x, requires_grad=False)
        for _ in range(depth):                        # the same link applied `depth` times
            h = layer(h, act="relu")
        return T.softmax_cross_entropy(h, t)

    for depth in (1, 3, 2):
        for p in layer.params():
            p.cleargrad()
        l = forward(depth)
        l.backward()

        def f():
            with T.no_backprop_mode():
                return float(forward(depth).array)

        gW, gb = fd_grad(f, [Wm, b])
        np.testing.assert_allclose(layer.W.grad, gW, rtol=1e-6, atol=1e-8)
        np.testing.assert_allclose(layer.b.grad, gb, rtol=1e-6, atol=1e-8)
        assert T.live_function_nodes() == 0


def test_gradients_accumulate_until_cleared_and_unchain_truncates(F):
    rng = np.random.default_rng(6)
    Wm, x, t = rnd(rng, 3, 3), rnd(rng, 2, 3), np.array([0, 2])
    p = T.Parameter(Wm)
    T.softmax_cross_entropy(T.matmul(T.Variable(x, False), p), t).backward()
    g1 = p.grad.copy()
    T.softmax_cross_entropy(T.matmul(T.Variable(x, False), p), t).backward()
    np.testing.assert_allclose(p.grad, 2 * g1, rtol=1e-14)
    p.cleargrad()
    assert p.grad is None
    # truncation: a variable cut from its history is a leaf; nothing behind it receives a gradient
    h = T.matmul(T.Variable(x, False), p)
    h.unchain()
    q = T.Parameter(rnd(rng, 3, 3))
    T.softmax_cross_entropy(T.matmul(h, q), t).backward()
    assert p.grad is None and q.grad is not None and h.grad is not None


def test_non_unit_seed_scales_every_gradient(F):
    rng = np.random.default_rng(7)
    Wm, x, t = rnd(rng, 3, 3), rnd(rng, 2, 3), np.array([1, 2])
    p = T.Parameter(Wm)
    T.softmax_cross_entropy(T.matmul(T.Variable(x, False), p), t).backward()
    g = p.grad.copy()
    p.cleargrad()
    l = T.softmax_cross_entropy(T.matmul(T.Variable(x, False), p), t)
    l.grad = np.full((), 2.5)
    l.backward()
    np.testing.assert_allclose(p.grad, 2.5 * g, rtol=1e-14)
    with pytest.raises(ValueError):
        T.matmul(T.Variable(x, False), p).backward()       # not a scalar and no gradient given


# ---- traversal order ------------------------------------------------------------------------------------
def test_each_backward_runs_once_after_all_its_consumers(F):
    order = []

    class Probe(T.FunctionNode):
        def __init__(self, tag):
            super().__init__()
            self.tag = tag

        def forward(self, xs):
            return (sum(xs) * 1.0,)

        def backward(self, indexes, gys):
            order.append(self.tag)
            return tuple(gys[0] for _ in indexes)

    a = T.Variable(np.ones(()))
    b = Probe("b").apply((a,))[0]
    c = Probe("c").apply((b,))[0]
    d = Probe("d").apply((b, c))[0]          # b reaches the root along two paths of unequal length
    e = Probe("e").apply((d, a, c))[0]
    e.backward()
    assert sorted(order) == ["b", "c", "d", "e"]
    assert order.index("e") < order.index("d") < order.index("c") < order.index("b")
    # paths from e to a: direct; d-b; d-c-b; c-b  => de/da = 4
    assert float(a.grad) == 4.0


# ---- what is retained, and when it is let go ---------------------------------------------------------
def test_functions_retain_only_what_their_backward_needs(F):
    rng = np.random.default_rng(8)
    x = T.Variable(rnd(rng, 2, 3))
    y = T.relu(x)
    assert x.node.data is None and y.creator.get_retained_outputs()[0] is y.array    # from the output
    z = T.gelu(x)
    assert x.node.data is x.array and z.creator.get_retained_outputs() == ()          # from the input
    s = T.add(y, z)
    assert y.node.data is None and z.node.data is None and s.creator.get_retained_inputs() == ()
    c0 = T.Variable(rnd(rng, 2, 3))
    pre = T.Variable(rnd(rng, 2, 12))
    c1, h1 = T.lstm(c0, pre)
    f = c1.creator
    assert pre.node.data is None and c0.node.data is c0.array and f.get_retained_outputs()[0] is c1.array
    # releasing the function releases the claim on its inputs
    f.unchain()
    assert c0.node.data is None and c1.creator is None and h1.creator is None


def test_intermediate_arrays_die_as_backward_passes_them(F):
    rng = np.random.default_rng(9)
    Wm, t = rnd(rng, 4, 4), np.array([0, 1, 2])
    p = T.Parameter(Wm)
    h = T.Variable(rnd(rng, 3, 4), requires_grad=False)
    refs = []
    for _ in range(4):
        h = T.matmul(h, p)
        h = T.relu(h)
        refs.append(weakref.ref(h.array))
    loss = T.softmax_cross_entropy(h, t)
    del h
    gc.disable()                      # reference counting alone must do it
    try:
        assert all(r() is not None for r in refs)       # retained by the graph, not by the user
        alive_during = []

        class Spy(OracleBackend):
            def gemm(self, *a, **k):
                alive_during.append(sum(r() is not None for r in refs))
                return super().gemm(*a, **k)

        with T.using_backend(Spy()):
            loss.backward()
        assert all(r() is None for r in refs)
        assert T.live_function_nodes() == 0
        # while walking back, every function node already passed has given its arrays back
        assert alive_during == sorted(alive_during, reverse=True) and alive_during[-1] <= 1
    finally:
        gc.enable()


def test_dropping_the_user_handle_frees_an_unretained_result(F):
    x = T.Variable(np.ones((2, 2)))
    y = T.add(x, x)                   # addition retains nothing
    z = T.add(y, y)
    r = weakref.ref(y.array)
    gc.disable()
    try:
        del y
        assert r() is None            # the node is still in the graph, the array is gone
        z.grad = np.ones((2, 2))
        z.backward()
        np.testing.assert_array_equal(x.grad, 4 * np.ones((2, 2)))
    finally:
        gc.enable()


def test_retain_grad_keeps_intermediate_gradients(F):
    x = T.Variable(np.ones((2, 2)))
    y = T.relu(x)
    z = T.add(y, y)
    z.grad = np.ones((2, 2))
    z.backward(retain_grad=True)
    np.testing.assert_array_equal(y.grad, 2 * np.ones((2, 2)))
    y2 = T.relu(x)
    z2 = T.add(y2, y2)
    z2.grad = np.ones((2, 2))
    z2.backward()
    assert y2.grad is None


def test_no_backprop_mode_records_nothing(F):
    p = T.Parameter(np.ones((2, 2)))
    with T.no_backprop_mode():
        y = T.matmul(T.Variable(np.ones((2, 2))), p)
    assert y.creator is None and p.node.data is None and T.live_function_nodes() == 0


# ---- double backpropagation ---------------------------------------------------------------------------
def test_gradients_of_gradients_closed_form(F):
    # y = sum x^3: dy/dx = 3 x^2, d/dx sum(dy/dx) = 6 x, once more: 6
    x = T.Variable(np.array([[1.0, -2.0, 0.5], [3.0, 0.25, -1.5]]))
    y = T.sum_all(T.mul(T.mul(x, x), x))
    g1, = T.grad([y], [x], enable_double_backprop=True)
    np.testing.assert_allclose(g1.array, 3 * x.array ** 2, rtol=1e-14)
    g2, = T.grad([T.sum_all(g1)], [x], enable_double_backprop=True)
    np.testing.assert_allclose(g2.array, 6 * x.array, rtol=1e-14)
    T.sum_all(g2).backward()
    np.testing.assert_allclose(x.grad, 6 * np.ones((2, 3)), rtol=1e-14)
    # grad() stores nothing, and without the flag its result has no history
    x2 = T.Variable(np.array([[2.0, 3.0]]))
    g, = T.grad([T.sum_all(T.mul(x2, x2))], [x2])
    assert x2.grad is None and g.creator is None
    np.testing.assert_allclose(g.array, 2 * x2.array, rtol=1e-14)


@pytest.mark.parametrize("first", ["tanh", "relu_fused", "relu"])
def test_gradient_penalty_matches_finite_differences(F, first):
    # penalty(theta) = || d f / d x ||^2 with f a two-layer network: differentiating it needs the
    # backward pass of f to be differentiable
    rng = np.random.default_rng(17)
    W1, b1, W2, b2 = rnd(rng, 5, 4), rnd(rng, 5), rnd(rng, 3, 5), rnd(rng, 3)
    x, c = rnd(rng, 6, 4), rnd(rng, 6, 3)

    def penalty(double):
        ps = [T.Parameter(W1), T.Parameter(b1), T.Parameter(W2), T.Parameter(b2)]
        xv = T.Variable(x)
        if first == "tanh":
            h = T.tanh(T.linear(xv, ps[0], ps[1]))
        elif first == "relu":
            h = T.relu(T.linear(xv, ps[0], ps[1]))
        else:
            h = T.linear(xv, ps[0], ps[1], act="relu")
        f = T.sum_all(T.mul(T.linear(h, ps[2], ps[3]), T.Variable(c, False)))
        g, = T.grad([f], [xv], enable_double_backprop=double)
        return T.sum_all(T.mul(g, g)), ps, xv

    pen, ps, xv = penalty(True)
    pen.backward()
    num = fd_grad(lambda: float(penalty(False)[0].array), [W1, b1, W2, x])
    for v, g in zip([ps[0], ps[1], ps[2], xv], num):
        got = np.zeros_like(g) if v.grad is None else v.grad
        np.testing.assert_allclose(got, g, rtol=2e-5, atol=1e-7)
    assert ps[3].grad is None or not np.any(ps[3].grad)          # the penalty does not depend on the last bias
    if first == "tanh":
        assert np.any(ps[1].grad)                                # ... but through tanh'' on the first one


@pytest.mark.parametrize("what", ["gelu_fused", "gelu", "softmax_ce", "embedding", "lstm"])
def test_gradient_penalty_through_the_remaining_functions(F, what):
    """|| d loss / d input ||^2 differentiated through the fused-GELU linear layer, the GELU function, the softmax
    cross-entropy, the embedding lookup and the LSTM cell: each needs a differentiable backward of its own."""
    rng = np.random.default_rng(41)
    n, d, hdim, k, V = 6, 4, 5, 3, 7
    W1, b1, W2, b2 = rnd(rng, hdim, d), rnd(rng, hdim), rnd(rng, k, hdim), rnd(rng, k)
    x, c = rnd(rng, n, d), rnd(rng, n, k)
    t = rng.integers(0, k, n)
    t[1] = -1
    E = rnd(rng, V, d)
    ids = np.array([1, 1, 3, 0, 6, 3])
    Wz, bz, cp = rnd(rng, 4 * hdim, d), rnd(rng, 4 * hdim), rnd(rng, n, hdim)
    arrays = {"gelu_fused": [W1, b1, W2, x], "gelu": [W1, b1, W2, x], "softmax_ce": [W1, b1, W2, b2, x], "embedding": [E, W1, b1, W2],
              "lstm": [Wz, bz, cp, x, W2]}[what]

    def penalty(double):
        vs = [T.Parameter(a) for a in arrays]
        if what in ("gelu_fused", "gelu"):
            Wa, ba, Wb, xv = vs
            h = T.linear(xv, Wa, ba, act="gelu") if what == "gelu_fused" else T.gelu(T.linear(xv, Wa, ba))
            f = T.sum_all(T.mul(T.linear(h, Wb, T.Variable(b2, False)), T.Variable(c, False)))
            wrt = xv
        elif what == "softmax_ce":
            Wa, ba, Wb, bb, xv = vs
            f = T.softmax_cross_entropy(T.linear(T.tanh(T.linear(xv, Wa, ba)), Wb, bb), t)
            wrt = xv
        elif what == "embedding":
            Ev, Wa, ba, Wb = vs
            h = T.tanh(T.linear(T.embed_id(ids, Ev), Wa, ba))
            f = T.sum_all(T.mul(T.linear(h, Wb, T.Variable(b2, False)), T.Variable(c, False)))
            wrt = Ev
        else:
            Wa, ba, cv, xv, Wb = vs
            cn, hn = T.lstm(cv, T.linear(xv, Wa, T.Variable(np.zeros(4 * hdim), False)), ba, twice_differentiable=True)
            f = T.add(T.sum_all(T.mul(T.linear(hn, Wb, T.Variable(b2, False)), T.Variable(c, False))), T.sum_all(T.mul(cn, cn)))
            wrt = xv
        g, = T.grad([f], [wrt], enable_double_backprop=double)
        return T.sum_all(T.mul(g, g)), vs

    pen, vs = penalty(True)
    pen.backward()
    num = fd_grad(lambda: float(penalty(False)[0].array), arrays)
    for v, g in zip(vs, num):
        got = np.zeros_like(g) if v.grad is None else v.grad
        np.testing.assert_allclose(got, g, rtol=5e-5, atol=2e-7)
    assert any(np.any(v.grad) for v in vs if v.grad is not None)


def test_lstm_without_the_flag_says_what_a_differentiable_backward_needs(F):
    rng = np.random.default_rng(43)
    cv, zv = T.Variable(rnd(rng, 2, 3)), T.Variable(rnd(rng, 2, 12))
    _, h = T.lstm(cv, zv)
    with pytest.raises(NotImplementedError, match="twice_differentiable"):
        T.grad([T.sum_all(h)], [zv], enable_double_backprop=True)
    g, = T.grad([T.sum_all(h)], [zv])                            # first order needs no flag
    assert g.array.shape == (2, 12)


def test_backward_with_double_backprop_keeps_the_graph_and_gives_grad_var(F):
    x = T.Variable(np.array([[0.5, -1.0]]))
    y = T.sum_all(T.mul(T.tanh(x), T.tanh(x)))
    y.backward(enable_double_backprop=True)
    assert x.grad_var is not None and x.grad_var.creator is not None and x.grad is x.grad_var.array
    t = np.tanh(x.array)
    np.testing.assert_allclose(x.grad, 2 * t * (1 - t ** 2), rtol=1e-13)
    gx = x.grad_var
    x.cleargrad()
    T.sum_all(gx).backward()                                     # d/dx of the gradient itself
    np.testing.assert_allclose(x.grad, 2 * (1 - t ** 2) ** 2 - 4 * t ** 2 * (1 - t ** 2), rtol=1e-12)


def test_a_released_output_node_is_replayed_for_the_differentiable_backward(F):
    class TanhAndDouble(T.FunctionNode):
        def forward(self, xs):
            self.retain_outputs((0,))
            return (np.tanh(xs[0]), 2.0 * xs[0])

        def backward_vars(self, indexes, gys):
            y, = self.get_retained_output_vars()
            parts = []
            if gys[0] is not None:
                parts.append(T.sub(gys[0], T.mul(gys[0], T.mul(y, y))))
            if gys[1] is not None:
                parts.append(T.scale(gys[1], 2.0))
                parts.append(T.scale(T.mul(y, y), 0.0))          # touches y: its node must exist
            out = parts[0]
            for p in parts[1:]:
                out = T.add(out, p)
            return (out,)

    x = T.Variable(np.array([[0.3, -0.7]]))
    f = TanhAndDouble()
    y0, y1 = f.apply((x,))
    backup = y0.array
    del y0                                                       # nobody refers to the first output any more
    assert f.outputs[0]() is None
    g, = T.grad([T.sum_all(y1)], [x], enable_double_backprop=True)
    np.testing.assert_allclose(g.array, 2 * np.ones((1, 2)))
    node = f.outputs[0]()
    assert node is not None and node.creator is f and node.rank == f.rank + 1
    assert f.get_retained_output_vars()[0].array is backup


def test_double_backprop_leaves_no_reference_cycles(F):
    rng = np.random.default_rng(19)
    gc.collect()
    gc.disable()
    try:
        W = T.Parameter(rnd(rng, 4, 4))
        x = T.Variable(rnd(rng, 3, 4))
        h = T.tanh(T.matmul(x, W))
        f = T.sum_all(T.mul(h, h))
        f.backward(enable_double_backprop=True)                  # gradients with history, stored on the variables
        refs = [weakref.ref(a) for a in (h.array, x.grad_var.array, W.grad_var.array, x.array)]
        nodes = [weakref.ref(n) for n in (h.node, x.node, W.node, x.grad_var.node)]
        pen = T.sum_all(T.mul(x.grad_var, x.grad_var))
        W.cleargrad()
        pen.backward()
        assert W.grad is not None
        del W, x, h, f, pen
        assert all(r() is None for r in refs) and all(n() is None for n in nodes)    # by reference counting alone
    finally:
        gc.enable()


def test_a_function_made_of_two_user_kernels_differentiates(F):
    from oracle import user_kernel as OU
    fk = OU.ElementwiseKernel("T x, T y", "T z", "z = log(1 + exp(x)) * y", "softplus_times")
    bk = OU.ElementwiseKernel("T x, T y, T gz", "T gx, T gy", "gx = gz * y / (1 + exp(-x)); gy = gz * log(1 + exp(x))", "softplus_times_bwd")
    op = T.user_elementwise(fk, bk)
    rng = np.random.default_rng(29)
    x, y, Wm, t = rnd(rng, 4, 3), rnd(rng, 4, 3), rnd(rng, 3, 3), np.array([0, 2, 1, 1])

    def loss(record=False):
        vs = [T.Variable(x), T.Variable(y), T.Parameter(Wm)]
        l = T.softmax_cross_entropy(T.matmul(op(vs[0], vs[1]), vs[2]), t)
        return (l, vs) if record else float(l.array)

    l, vs = loss(True)
    l.backward()
    for v, g in zip(vs, fd_grad(loss, [x, y, Wm])):
        np.testing.assert_allclose(v.grad, g, rtol=1e-6, atol=1e-8)


def test_adam_optimiser_keeps_state_per_parameter_and_counts_steps(F):
    rng = np.random.default_rng(13)
    Wm, b, x, t = rnd(rng, 3, 4), rnd(rng, 3), rnd(rng, 5, 4), np.array([0, 1, 2, 1, 0])
    layer = T.Linear(Wm.copy(), b.copy())
    opt = T.Adam(layer.params(), lr=0.05)
    ref = {"W": (Wm.copy(), np.zeros_like(Wm), np.zeros_like(Wm)), "b": (b.copy(), np.zeros_like(b), np.zeros_like(b))}
    for step in (1, 2, 3):
        opt.cleargrads()
        T.softmax_cross_entropy(layer(T.Variable(x, False)), t).backward()
        gW, gb = layer.W.grad.copy(), layer.b.grad.copy()
        opt.update()
        ref["W"] = O.adam_update(ref["W"][0], gW, ref["W"][1], ref["W"][2], 0.05, step)
        ref["b"] = O.adam_update(ref["b"][0], gb, ref["b"][1], ref["b"][2], 0.05, step)
        np.testing.assert_allclose(layer.W.array, ref["W"][0], rtol=1e-13)
        np.testing.assert_allclose(layer.b.array, ref["b"][0], rtol=1e-13)
    assert opt.t == 3 and [c for c in F.calls if c[0] == "adam"] == [("adam", 2)] * 3


def test_gpu_backend_refuses_to_exist_without_the_library(monkeypatch):
    from paper_1908_00213_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libchn.so")
    with pytest.raises(Exception):
        T.GpuBackend()
