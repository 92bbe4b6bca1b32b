"""GPU parity of training steps driven by the define-by-run tape (every kernel through the C ABI)
against the oracle's hand-ordered steps, and against the same tape run on the CPU with the oracle's
functions as kernels where the oracle has no ready-made step (carried state, changing topology).
Errors are measured against each tensor's own scale, as for the recorded step drivers."""
import gc

import numpy as np
import pytest
import torch

from oracle import oracle as O
from oracle import steps as OS
from paper_1908_00213_amd import steps, tape as T, workloads as W
from tests.oracle_backend import OracleBackend
from tests.util import bf16r, check, host

pytestmark = pytest.mark.gpu


def cmp(got, ref, tol, what):
    ref = np.asarray(ref, dtype=np.float64)
    check(host(got), ref, tol, float(np.max(np.abs(ref))) if ref.size else 0.0, what)


def run_mlp(w, lowp, tol, fused=True):
    F = T.backend()
    x, t = w.xs[0], w.ts[0]
    if lowp:
        x = bf16r(x)
    model = T.MLP([(F.from_numpy(Wm), F.from_numpy(b)) for Wm, b in w.params], w.act, lowp, fused)
    opt = T.SGD(model.params(), w.lr)
    xd = F.from_numpy(x, "bf16" if lowp else None)
    td = F.from_numpy(t)
    loss = model.loss(xd, td)
    loss.backward()
    r = OS.mlp_step(w.params, x, t, np.float32(w.lr), w.act, lowp)
    assert abs(float(loss.array.cpu()) - r["loss"]) <= tol * max(1.0, abs(r["loss"]))
    grads = [(host(l.W.grad), host(l.b.grad)) for l in model.layers]
    for l, (dW, db) in enumerate(r["grads"]):
        cmp(model.layers[l].W.grad, dW, tol, "dW%d" % l)
        cmp(model.layers[l].b.grad, db, tol, "db%d" % l)
        assert model.layers[l].W.grad.dtype == torch.float32
    opt.update()
    lr = np.float32(w.lr)
    for l, layer in enumerate(model.layers):
        for p, old, g in ((layer.W, w.params[l][0], grads[l][0]), (layer.b, w.params[l][1], grads[l][1])):
            check(host(p.array), O.sgd_update(old, g, lr), 1e-6, np.abs(old) + lr * np.abs(g), "update %d" % l)
        if lowp:
            assert np.array_equal(host(layer.W.lowp), O.round_bf16(host(layer.W.array)))
    assert T.live_function_nodes() == 0
    return model, opt, xd, td


def test_tape_mlp_steps_match_the_oracle():
    run_mlp(W.config1(), False, 1e-4)
    run_mlp(W.config1(), False, 1e-4, fused=False)
    run_mlp(W.config3(n_batches=1), False, 1e-4)
    run_mlp(W.config3(n_batches=1), True, 2e-2)
    w = W.config5(n_batches=1, scale=8)
    run_mlp(w, True, 2e-2)
    run_mlp(w, False, 1e-4)
    run_mlp(w, True, 2e-2, fused=False)


def test_tape_mlp_equals_the_recorded_step_bit_for_bit_in_fp32():
    # same kernels on the same operands; only who decides the order of the calls differs (the recorded
    # step is told to take the loss and its gradient as two calls, as a tape has to)
    w = W.config3(n_batches=1)
    model, opt, xd, td = run_mlp(w, False, 1e-4)
    tr = steps.MLPTrainer(w.params, w.batch, w.act, w.lr, False, fused_loss=False)
    tr.step(xd, td)
    for l, layer in enumerate(model.layers):
        assert torch.equal(layer.W.grad, tr.dW[l]) and torch.equal(layer.b.grad, tr.db[l])
        assert torch.equal(layer.W.array, tr.W[l]) and torch.equal(layer.b.array, tr.b[l])


def test_tape_second_iteration_uses_updated_weights_and_cleared_gradients():
    w = W.config1()
    model, opt, xd, td = run_mlp(w, False, 1e-4)          # one step taken
    r1 = OS.mlp_step(w.params, w.xs[0], w.ts[0], np.float32(w.lr), w.act)
    opt.cleargrads()
    loss = model.loss(xd, td)
    loss.backward()
    r2 = OS.mlp_step(r1["params"], w.xs[0], w.ts[0], np.float32(w.lr), w.act)
    assert abs(float(loss.array.cpu()) - r2["loss"]) < 1e-4
    cmp(model.layers[0].W.grad, r2["grads"][0][0], 1e-4, "dW0 second step")


@pytest.mark.parametrize("cfg", [dict(vocab=300, embed=72, hidden=72, batch=16, bptt=6),
                                 dict(vocab=1000, embed=130, hidden=130, batch=24, bptt=4)])
def test_tape_lstm_language_model_step_matches_the_oracle(cfg):
    F = T.backend()
    w = W.config4(**cfg)
    w.params["b"] = (np.random.default_rng(3).standard_normal(w.params["b"].shape) * 0.1).astype(np.float32)
    model = T.LSTMLanguageModel({k: F.from_numpy(v) for k, v in w.params.items()})
    ids, tg = F.from_numpy(w.ids.reshape(-1)), F.from_numpy(w.targets.reshape(-1))
    loss, _ = model.loss(ids, tg, w.bptt)
    loss.backward()
    r = OS.lstm_lm_step(w.params, w.ids, w.targets, np.float32(w.lr))
    assert abs(float(loss.array.cpu()) - r["loss"]) <= 1e-4 * abs(r["loss"])
    for k in w.params:
        cmp(model.P[k].grad, r["grads"][k], 1e-4, "d" + k)
    unused = np.setdiff1d(np.arange(w.vocab), w.ids.reshape(-1))
    assert np.all(host(model.P["E"].grad)[unused] == 0)
    g = {k: host(p.grad) for k, p in model.P.items()}
    T.SGD(model.params(), w.lr).update()
    lr = np.float32(w.lr)
    for k in w.params:
        check(host(model.P[k].array), O.sgd_update(w.params[k], g[k], lr), 1e-6,
              np.abs(w.params[k]) + lr * np.abs(g[k]), "update " + k)
    assert T.live_function_nodes() == 0


@pytest.mark.parametrize("cfg", [dict(vocab=300, embed=72, hidden=96, batch=16, bptt=6),      # width the fused step takes
                                 dict(vocab=1000, embed=130, hidden=130, batch=24, bptt=4)])   # product and cell apart
def test_tape_n_step_lstm_matches_the_oracle_and_carries_state(cfg):
    """The whole recurrent layer as one function node: the step against the oracle's, then two windows
    with the state carried over against the step-by-step graph on the CPU oracle backend."""
    F = T.backend()
    w = W.config4(**cfg)
    w.params["b"] = (np.random.default_rng(3).standard_normal(w.params["b"].shape) * 0.1).astype(np.float32)
    model = T.LSTMLanguageModel({k: F.from_numpy(v) for k, v in w.params.items()}, n_step=True)
    ids, tg = F.from_numpy(w.ids.reshape(-1)), F.from_numpy(w.targets.reshape(-1))
    loss, _ = model.loss(ids, tg, w.bptt)
    assert T.live_function_nodes() == 5
    loss.backward()
    r = OS.lstm_lm_step(w.params, w.ids, w.targets, np.float32(w.lr))
    assert abs(float(loss.array.cpu()) - r["loss"]) <= 1e-4 * abs(r["loss"])
    for k in w.params:
        cmp(model.P[k].grad, r["grads"][k], 1e-4, "d" + k)
    assert T.live_function_nodes() == 0

    # widths rounded up by inert units (what lets a width like 130 use the fused step): same numbers
    padded = T.LSTMLanguageModel({k: F.from_numpy(v) for k, v in W.pad_lstm_params(w.params).items()}, n_step=True)
    lp, _ = padded.loss(ids, tg, w.bptt)
    lp.backward()
    assert abs(float(lp.array.cpu()) - r["loss"]) <= 1e-4 * abs(r["loss"])
    Hp = padded.P["U"].array.shape[0]
    gU = host(padded.P["U"].grad).reshape(Hp, 4, Hp)[:w.hidden, :, :w.hidden].reshape(w.hidden, 4 * w.hidden)
    check(gU, r["grads"]["U"], 1e-4, float(np.max(np.abs(r["grads"]["U"]))), "dU of the padded model")

    idn, tgn = w.ids.reshape(-1).astype(np.int64), w.targets.reshape(-1).astype(np.int64)
    Bn, cut = w.batch, w.bptt // 2

    def two_windows(Fb, n_step):
        m = T.LSTMLanguageModel({k: Fb.from_numpy(v) for k, v in w.params.items()}, n_step=n_step)
        out, state = [], None
        for lo, hi in ((0, cut), (cut, w.bptt)):
            for p in m.params():
                p.cleargrad()
            sl = slice(lo * Bn, hi * Bn)
            l, state = m.loss(Fb.from_numpy(idn[sl]), Fb.from_numpy(tgn[sl]), hi - lo, state)
            l.backward()
            for v in state:
                v.unchain()
            out.append((float(Fb.to_numpy(l.array)), {k: Fb.to_numpy(p.grad) for k, p in m.P.items()}))
        return out

    got = two_windows(F, True)
    with T.using_backend(OracleBackend()) as Fo:
        ref = two_windows(Fo, False)
    for (lg, gg), (lr_, gr) in zip(got, ref):
        assert abs(lg - lr_) <= 1e-4 * abs(lr_)
        for k in gr:
            check(gg[k], gr[k], 1e-4, float(np.max(np.abs(gr[k]))), "d" + k)


@pytest.mark.parametrize("cfg", [dict(vocab=300, embed=72, hidden=96, batch=16, bptt=6),      # both steps fused
                                 dict(vocab=1000, embed=136, hidden=136, batch=24, bptt=4)])   # separate calls
def test_tape_n_step_lstm_mixed_precision_matches_the_oracle(cfg):
    """bf16 storage of everything that feeds a product, against the oracle's step with the same
    storage points; then the optimiser refreshes the working copies from the fp32 masters."""
    F = T.backend()
    w = W.config4(**cfg)
    w.params["b"] = (np.random.default_rng(3).standard_normal(w.params["b"].shape) * 0.1).astype(np.float32)
    model = T.LSTMLanguageModel({k: F.from_numpy(v) for k, v in w.params.items()}, n_step=True, lowp=True)
    ids, tg = F.from_numpy(w.ids.reshape(-1)), F.from_numpy(w.targets.reshape(-1))
    loss, _ = model.loss(ids, tg, w.bptt)
    loss.backward()
    r = OS.lstm_lm_step(w.params, w.ids, w.targets, np.float32(w.lr), lowp=True)
    assert abs(float(loss.array.cpu()) - r["loss"]) <= 2e-2 * abs(r["loss"])
    for k in w.params:
        assert model.P[k].grad.dtype == torch.float32
        cmp(model.P[k].grad, r["grads"][k], 2e-2, "d" + k)
    T.SGD(model.params(), w.lr).update()
    for k in ("E", "W", "U", "W_out"):
        assert np.array_equal(host(model.P[k].lowp), O.round_bf16(host(model.P[k].array))), k
    assert T.live_function_nodes() == 0


def test_tape_window_length_changes_and_state_is_carried_across_windows():
    # truncated back-propagation over two windows of different length: the second starts from the
    # first one's final state, cut from its history.  Reference: the same tape on the CPU with the
    # oracle's functions as kernels.
    w = W.config4(vocab=120, embed=40, hidden=48, batch=8, bptt=7)
    w.params["b"] = (np.random.default_rng(4).standard_normal(w.params["b"].shape) * 0.1).astype(np.float32)
    ids, tg = w.ids.reshape(-1).astype(np.int64), w.targets.reshape(-1).astype(np.int64)
    Bn = w.batch

    def two_windows(F):
        model = T.LSTMLanguageModel({k: F.from_numpy(v) for k, v in w.params.items()})
        out, state = [], None
        for lo, hi in ((0, 3), (3, 7)):
            for p in model.params():
                p.cleargrad()
            sl = slice(lo * Bn, hi * Bn)
            loss, state = model.loss(F.from_numpy(ids[sl]), F.from_numpy(tg[sl]), hi - lo, state)
            loss.backward()
            for v in state:
                v.unchain()
            out.append((float(F.to_numpy(loss.array)), {k: F.to_numpy(p.grad) for k, p in model.P.items()}))
        return out

    got = two_windows(T.backend())
    with T.using_backend(OracleBackend()) as Fo:
        ref = two_windows(Fo)
    for (lg, gg), (lr_, gr) in zip(got, ref):
        assert abs(lg - lr_) <= 1e-4 * abs(lr_)
        for k in gr:
            check(gg[k], gr[k], 1e-4, float(np.max(np.abs(gr[k]))), "d" + k)


def test_tape_depth_chosen_per_iteration():
    rng = np.random.default_rng(12)
    Wm = (rng.standard_normal((64, 64)) * 0.2).astype(np.float32)
    b = (rng.standard_normal(64) * 0.1).astype(np.float32)
    x = rng.standard_normal((48, 64)).astype(np.float32)
    t = rng.integers(0, 64, 48)

    def run(F, depth):
        layer = T.Linear(F.from_numpy(Wm), F.from_numpy(b))
        h = F.from_numpy(x)
        for _ in range(depth):
            h = layer(h, act="gelu")
        loss = T.softmax_cross_entropy(h, F.from_numpy(t))
        loss.backward()
        return float(F.to_numpy(loss.array)), F.to_numpy(layer.W.grad), F.to_numpy(layer.b.grad)

    for depth in (3, 1, 4):
        got = run(T.backend(), depth)
        with T.using_backend(OracleBackend()) as Fo:
            ref = run(Fo, depth)
        assert abs(got[0] - ref[0]) <= 1e-5 * abs(ref[0])
        check(got[1], ref[1], 1e-4, float(np.max(np.abs(ref[1]))), "dW depth %d" % depth)
        check(got[2], ref[2], 1e-4, float(np.max(np.abs(ref[2]))), "db depth %d" % depth)


def test_tape_returns_device_memory_while_walking_back():
    F = T.backend()
    n, width, depth = 2048, 1024, 8
    rng = np.random.default_rng(1)
    layers = [T.Linear(F.from_numpy((rng.standard_normal((width, width)) * 0.03).astype(np.float32)),
                       F.from_numpy(np.zeros(width, dtype=np.float32))) for _ in range(depth)]
    x = F.from_numpy(rng.standard_normal((n, width)).astype(np.float32))
    t = F.from_numpy(rng.integers(0, width, n))
    act_bytes = n * width * 4

    def forward():
        h = x
        for l in layers:
            h = l(h, act="relu")
        return T.softmax_cross_entropy(h, t)

    gc.collect()
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()
    loss = forward()
    held = torch.cuda.memory_allocated() - base
    assert held >= depth * act_bytes                       # every layer's output is retained
    seen = []
    orig = F.gemm

    def spy(*a, **k):
        seen.append(torch.cuda.memory_allocated() - base)
        return orig(*a, **k)

    F.gemm = spy
    gc.disable()
    try:
        loss.backward()
    finally:
        gc.enable()
        del F.gemm
    grads = depth * (width * width + width) * 4
    # activations are given back layer by layer: when the walk reaches the first layer, what is
    # allocated beyond the parameters' gradients is that layer's own working set (its retained
    # output, the gradient that arrived, the masked gradient), not the eight retained outputs that
    # were there when the walk began
    assert seen[-1] - grads <= seen[0] - 4 * act_bytes
    del loss
    torch.cuda.synchronize()
    after = torch.cuda.memory_allocated() - base
    assert after <= grads + 4 * act_bytes                  # parameters' gradients and little else
    assert T.live_function_nodes() == 0
    # no_backprop_mode: nothing is retained at all
    with T.no_backprop_mode():
        l2 = forward()
    assert torch.cuda.memory_allocated() - base - after <= 2 * act_bytes
    assert abs(float(l2.array.cpu()) - np.log(width)) < 2.0


@pytest.mark.parametrize("first", ["tanh", "relu_fused"])
def test_tape_double_backprop_gradient_penalty(first):
    # the gradient of || d f / d x ||^2 needs a differentiable backward pass; the same tape code runs on
    # the GPU and, as the reference, on the CPU with the oracle's functions as kernels
    rng = np.random.default_rng(23)
    n, d, hdim, k = 200, 96, 130, 24
    W1 = (rng.standard_normal((hdim, d)) / np.sqrt(d)).astype(np.float32)
    b1 = (rng.standard_normal(hdim) * 0.1).astype(np.float32)
    W2 = (rng.standard_normal((k, hdim)) / np.sqrt(hdim)).astype(np.float32)
    b2 = np.zeros(k, dtype=np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    c = rng.standard_normal((n, k)).astype(np.float32)

    def run(F):
        ps = [T.Parameter(F.from_numpy(a)) for a in (W1, b1, W2, b2)]
        xv = T.Variable(F.from_numpy(x))
        lin = T.linear(xv, ps[0], ps[1], act="relu") if first == "relu_fused" else T.tanh(T.linear(xv, ps[0], ps[1]))
        f = T.sum_all(T.mul(T.linear(lin, ps[2], ps[3]), T.Variable(F.from_numpy(c), False)))
        g, = T.grad([f], [xv], enable_double_backprop=True)
        pen = T.sum_all(T.mul(g, g))
        pen.backward()
        # a parameter the penalty does not depend on (the first bias behind a ReLU) receives nothing
        pg = [np.zeros(a.shape) if p.grad is None else F.to_numpy(p.grad) for p, a in zip(ps[:3], (W1, b1, W2))]
        gx = np.zeros(x.shape) if xv.grad is None else F.to_numpy(xv.grad)    # piecewise linear f: no dependence on x either
        return float(F.to_numpy(pen.array)), F.to_numpy(g.array), pg, gx

    got = run(T.backend())
    with T.using_backend(OracleBackend()) as Fo:
        ref = run(Fo)
    assert abs(got[0] - ref[0]) <= 1e-4 * abs(ref[0])
    check(got[1], ref[1], 1e-4, float(np.max(np.abs(ref[1]))), "d f / d x")
    for a, b, name in zip(got[2], ref[2], ("W1", "b1", "W2")):
        check(a, b, 1e-4, float(np.max(np.abs(b))) + 1e-30, "d penalty / d " + name)
    check(got[3], ref[3], 1e-4, float(np.max(np.abs(ref[3]))) + 1e-30, "d penalty / d x")


@pytest.mark.parametrize("what", ["gelu_fused", "softmax_ce", "embedding", "lstm"])
def test_tape_double_backprop_through_the_remaining_functions(what):
    """The gradient of || d loss / d input ||^2 through the fused-GELU linear layer, the softmax cross-entropy, the
    embedding lookup and the LSTM cell: the same tape code on the GPU and, as the reference, on the CPU with the
    oracle's functions as kernels (whose second-order pieces are pinned by finite differences on the CPU)."""
    rng = np.random.default_rng(29)
    n, d, hdim, k, V = 200, 96, 128, 24, 50
    f32 = lambda a: a.astype(np.float32)
    W1, b1 = f32(rng.standard_normal((hdim, d)) / np.sqrt(d)), f32(rng.standard_normal(hdim) * 0.1)
    W2, b2 = f32(rng.standard_normal((k, hdim)) / np.sqrt(hdim)), np.zeros(k, np.float32)
    Wz, bz = f32(rng.standard_normal((4 * hdim, d)) / np.sqrt(d)), f32(rng.standard_normal(4 * hdim) * 0.1)
    x, c, cp = f32(rng.standard_normal((n, d))), f32(rng.standard_normal((n, k))), f32(rng.standard_normal((n, hdim)))
    E = f32(rng.standard_normal((V, d)))
    ids = rng.integers(0, V, n)
    t = rng.integers(0, k, n)
    t[::9] = -1

    def run(F):
        P = lambda a: T.Parameter(F.from_numpy(a))
        const = lambda a: T.Variable(F.from_numpy(a), False)
        if what == "gelu_fused":
            vs = [P(W1), P(b1), P(W2), P(x)]
            f = T.sum_all(T.mul(T.linear(T.linear(vs[3], vs[0], vs[1], act="gelu"), vs[2], const(b2)), const(c)))
            wrt = vs[3]
        elif what == "softmax_ce":
            vs = [P(W1), P(b1), P(W2), P(b2), P(x)]
            f = T.softmax_cross_entropy(T.linear(T.tanh(T.linear(vs[4], vs[0], vs[1])), vs[2], vs[3]), F.from_numpy(t))
            wrt = vs[4]
        elif what == "embedding":
            vs = [P(E), P(W1), P(b1), P(W2)]
            f = T.sum_all(T.mul(T.linear(T.tanh(T.linear(T.embed_id(F.from_numpy(ids), vs[0]), vs[1], vs[2])), vs[3], const(b2)), const(c)))
            wrt = vs[0]
        else:
            vs = [P(Wz), P(bz), P(cp), P(x), P(W2)]
            cn, hn = T.lstm(vs[2], T.linear(vs[3], vs[0], const(np.zeros(4 * hdim, np.float32))), vs[1], twice_differentiable=True)
            f = T.add(T.sum_all(T.mul(T.linear(hn, vs[4], const(b2)), const(c))), T.sum_all(T.mul(cn, cn)))
            wrt = vs[3]
        g, = T.grad([f], [wrt], enable_double_backprop=True)
        pen = T.sum_all(T.mul(g, g))
        pen.backward()
        return float(F.to_numpy(pen.array)), F.to_numpy(g.array), [None if v.grad is None else F.to_numpy(v.grad) for v in vs]

    got = run(T.backend())
    with T.using_backend(OracleBackend()) as Fo:
        ref = run(Fo)
    assert abs(got[0] - ref[0]) <= 2e-4 * abs(ref[0])
    check(got[1], ref[1], 2e-4, float(np.max(np.abs(ref[1]))), "first-order gradient")
    assert any(b is not None and np.any(b) for b in ref[2])
    for i, (a, b) in enumerate(zip(got[2], ref[2])):
        assert (a is None) == (b is None)
        if b is not None:
            check(a, b, 3e-4, float(np.max(np.abs(b))) + 1e-30, "d penalty / d input %d" % i)


def test_tape_function_made_of_two_user_kernels():
    # a new differentiable operation from two snippets compiled at run time; reference: the same tape
    # on the CPU with the oracle's evaluation of the same snippets
    from oracle import user_kernel as OU
    from paper_1908_00213_amd import binding as B
    fwd = ("T x, T y", "T z", "z = log(1 + exp(x)) * y", "softplus_times")
    bwd = ("T x, T y, T gz", "T gx, T gy", "gx = gz * y / (1 + exp(-x)); gy = gz * log(1 + exp(x))", "softplus_times_bwd")
    rng = np.random.default_rng(31)
    x, y = rng.standard_normal((300, 96)).astype(np.float32), rng.standard_normal((300, 96)).astype(np.float32)
    Wm = (rng.standard_normal((96, 40)) * 0.1).astype(np.float32)
    t = rng.integers(0, 40, 300)

    def run(F, mk):
        op = T.user_elementwise(mk(*fwd), mk(*bwd))
        vs = [T.Variable(F.from_numpy(x)), T.Variable(F.from_numpy(y)), T.Parameter(F.from_numpy(Wm))]
        l = T.softmax_cross_entropy(T.matmul(op(vs[0], vs[1]), vs[2]), F.from_numpy(t))
        l.backward()
        return float(F.to_numpy(l.array)), [F.to_numpy(v.grad) for v in vs]

    got = run(T.backend(), B.ElementwiseKernel)
    with T.using_backend(OracleBackend()) as Fo:
        ref = run(Fo, OU.ElementwiseKernel)
    assert abs(got[0] - ref[0]) <= 1e-5 * abs(ref[0])
    for a, b in zip(got[1], ref[1]):
        check(a, b, 1e-4, float(np.max(np.abs(b))), "gradient")
