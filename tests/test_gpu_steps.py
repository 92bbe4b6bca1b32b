"""GPU parity of whole training steps (forward + backward + SGD issued call by call through the C ABI)
against the oracle's steps on the same seeded inputs: loss, every gradient and every updated
parameter.  End-to-end errors are measured against each tensor's own scale (its largest magnitude),
because a gradient entry is a long signed sum whose terms are of that size."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from oracle import steps as OS
from paper_1908_00213_amd import steps, workloads as W
from tests.util import bf16r, check, host

pytestmark = pytest.mark.gpu


def cmp(got, ref, tol, what):
    ref = np.asarray(ref, dtype=np.float64)
    check(host(got), ref, tol, float(np.max(np.abs(ref))) if ref.size else 0.0, what)


def run_mlp(w, lowp, tol):
    x, t = w.xs[0], w.ts[0]
    if lowp:
        x = bf16r(x)
    tr = steps.MLPTrainer(w.params, w.batch, w.act, w.lr, lowp)
    xd = torch.from_numpy(x).cuda()
    xd = xd.to(torch.bfloat16) if lowp else xd
    td = torch.from_numpy(t).cuda()
    loss = tr.step(xd, td)
    r = OS.mlp_step(w.params, x, t, np.float32(w.lr), w.act, lowp)
    assert abs(float(loss.cpu()) - r["loss"]) <= tol * max(1.0, abs(r["loss"])), (float(loss.cpu()), r["loss"])
    cmp(tr.logits, r["logits"], tol, "logits")
    lr = np.float32(w.lr)
    for l, ((dW, db), (Wn, bn)) in enumerate(zip(r["grads"], r["params"])):
        cmp(tr.dW[l], dW, tol, "dW%d" % l)
        cmp(tr.db[l], db, tol, "db%d" % l)
        # updated parameters: end to end they inherit lr * (gradient error); against the oracle's
        # update of the GPU's own gradient (teacher-forced) they must agree to fp32 rounding
        W0, b0 = w.params[l]
        for got, old, g_gpu, new_ref, g_ref in ((tr.W[l], W0, tr.dW[l], Wn, dW), (tr.b[l], b0, tr.db[l], bn, db)):
            check(host(got), O.sgd_update(old, host(g_gpu), lr), 1e-6, np.abs(old) + lr * np.abs(host(g_gpu)), "update %d" % l)
            check(host(got), new_ref, 1e-6, np.abs(old) + float(lr) * tol * float(np.max(np.abs(g_ref))) / 1e-6, "param %d" % l)
        if lowp:
            assert np.array_equal(host(tr.Wl[l]), O.round_bf16(host(tr.W[l])))
    return tr, xd, td


def test_config1_tiny_mlp_step():
    tr, xd, td = run_mlp(W.config1(), False, 1e-4)
    # library calls per step: 3 forward products, loss with its gradient, 3 dW + 3 db + 2 dx, 1 update
    assert tr.n_launch_calls(xd, td) == 13


def test_config3_mlp_step_fp32_and_bf16():
    run_mlp(W.config3(n_batches=1), False, 1e-4)
    run_mlp(W.config3(n_batches=1), True, 2e-2)


def test_config5_scaled_wide_mlp_gelu_bf16_and_fp32():
    w = W.config5(n_batches=1, scale=8)         # 512-512-512-512-1000, batch 1024
    tr, _, _ = run_mlp(w, True, 2e-2)
    # at these sizes (whole 256 x 256 tiles) the hidden layers' bias gradients come from the row-block
    # column sums that the activation-gradient products leave behind
    assert sorted(tr.rowsums) == [1, 2, 3]
    run_mlp(w, False, 1e-4)
    wr = W.make_mlp("t", (256, 512, 256, 16), 512, "relu", 7, 1)
    tr, _, _ = run_mlp(wr, False, 1e-4)
    assert sorted(tr.rowsums) == [1, 2]
    run_mlp(wr, True, 2e-2)


def test_mlp_second_step_uses_updated_weights():
    w = W.config1()
    tr = steps.MLPTrainer(w.params, w.batch, w.act, 0.5, False)
    xd, td = torch.from_numpy(w.xs[0]).cuda(), torch.from_numpy(w.ts[0]).cuda()
    l1 = float(tr.step(xd, td).cpu())
    l2 = float(tr.step(xd, td).cpu())
    r1 = OS.mlp_step(w.params, w.xs[0], w.ts[0], np.float32(0.5), w.act)
    r2 = OS.mlp_step(r1["params"], w.xs[0], w.ts[0], np.float32(0.5), w.act)
    assert abs(l1 - r1["loss"]) < 1e-4 and abs(l2 - r2["loss"]) < 1e-4 and l2 < l1


def test_gradient_on_batch_is_mean_of_halves():
    # the data-parallel identity of Section "Data and Model Parallelism", on one GPU
    w = W.make_mlp("t", (40, 30, 7), 64, "relu", 5, 1)
    grads = []
    for sl in (slice(0, 64), slice(0, 32), slice(32, 64)):
        n = sl.stop - sl.start
        tr = steps.MLPTrainer(w.params, n, "relu", 0.0, False)
        tr.step(torch.from_numpy(w.xs[0][sl]).cuda(), torch.from_numpy(w.ts[0][sl]).cuda())
        grads.append([host(g) for g in tr.dW + tr.db])
    for full, a, b in zip(*grads):
        check(full, 0.5 * (a + b), 1e-4, float(np.max(np.abs(full))), "halves")


@pytest.mark.parametrize("mode", ["sequence", "step", "unfused"])   # one launch for all steps of a pass / one per step / product and cell apart
@pytest.mark.parametrize("cfg", [dict(vocab=300, embed=72, hidden=72, batch=16, bptt=6),
                                 dict(vocab=1000, embed=130, hidden=130, batch=24, bptt=4)])
def test_config4_scaled_lstm_lm_step(cfg, mode):
    w = W.config4(**cfg)
    w.params["b"] = (np.random.default_rng(3).standard_normal(w.params["b"].shape) * 0.1).astype(np.float32)
    tr = steps.LSTMTrainer(w.params, w.bptt, w.batch, w.lr, fused_step=mode != "unfused", whole_sequence=mode == "sequence", whole_sequence_bwd=mode == "sequence")
    ids, tg = torch.from_numpy(w.ids).cuda(), torch.from_numpy(w.targets).cuda()
    loss = tr.step(ids, tg)
    assert tr.sequence_complete() and tr.whole_sequence == tr.whole_sequence_bwd == (mode == "sequence")
    r = OS.lstm_lm_step(w.params, w.ids, w.targets, np.float32(w.lr))
    assert abs(float(loss.cpu()) - r["loss"]) <= 1e-4 * abs(r["loss"])
    lr = np.float32(w.lr)
    for k in w.params:
        cmp(tr.g[k], r["grads"][k], 1e-4, "d" + k)
        check(host(tr.P[k]), O.sgd_update(w.params[k], host(tr.g[k]), lr), 1e-6,
              np.abs(w.params[k]) + lr * np.abs(host(tr.g[k])), "update " + k)
        check(host(tr.P[k]), r["params"][k], 1e-6,
              np.abs(w.params[k]) + float(lr) * 1e-4 * float(np.max(np.abs(r["grads"][k]))) / 1e-6, k)
    # rows of E that no token used keep a zero gradient and are unchanged bit for bit
    unused = np.setdiff1d(np.arange(w.vocab), w.ids.reshape(-1))
    assert np.all(host(tr.g["E"])[unused] == 0)
    assert np.array_equal(host(tr.P["E"])[unused], w.params["E"][unused].astype(np.float64))
    # a different window length (another graph topology) through the same code
    tr2 = steps.LSTMTrainer(w.params, 2, w.batch, w.lr)
    l2 = tr2.step(ids[:2].contiguous(), tg[:2].contiguous())
    r2 = OS.lstm_lm_step(w.params, w.ids[:2], w.targets[:2], np.float32(w.lr))
    assert abs(float(l2.cpu()) - r2["loss"]) <= 1e-4 * abs(r2["loss"])
    cmp(tr2.g["U"], r2["grads"]["U"], 1e-4, "dU T=2")


@pytest.mark.parametrize("mode", ["sequence", "step", "unfused"])   # one launch for all steps of a pass / one per step / product and cell apart
@pytest.mark.parametrize("cfg", [dict(vocab=300, embed=72, hidden=72, batch=16, bptt=6),
                                 dict(vocab=1000, embed=130, hidden=130, batch=24, bptt=4)])
def test_config4_scaled_lstm_lm_step_mixed_precision(cfg, mode):
    w = W.config4(**cfg)
    w.params["b"] = (np.random.default_rng(3).standard_normal(w.params["b"].shape) * 0.1).astype(np.float32)
    tr = steps.LSTMTrainer(w.params, w.bptt, w.batch, w.lr, lowp=True, fused_step=mode != "unfused", whole_sequence=mode == "sequence", whole_sequence_bwd=mode == "sequence")
    ids, tg = torch.from_numpy(w.ids).cuda(), torch.from_numpy(w.targets).cuda()
    loss = tr.step(ids, tg)
    assert tr.sequence_complete() and tr.whole_sequence == tr.whole_sequence_bwd == (mode == "sequence")
    r = OS.lstm_lm_step(w.params, w.ids, w.targets, np.float32(w.lr), lowp=True)
    assert abs(float(loss.cpu()) - r["loss"]) <= 2e-2 * abs(r["loss"])
    assert tr.Hs.dtype == torch.bfloat16 and tr.dZ.dtype == torch.bfloat16 and tr.Z.dtype == torch.float32
    lr = np.float32(w.lr)
    for k in w.params:
        assert tr.g[k].dtype == torch.float32
        cmp(tr.g[k], r["grads"][k], 2e-2, "d" + k)
        # the update itself is fp32 arithmetic on the master weights
        check(host(tr.P[k]), O.sgd_update(w.params[k], host(tr.g[k]), lr), 1e-6,
              np.abs(w.params[k]) + lr * np.abs(host(tr.g[k])), "update " + k)
    # the working copies follow the masters (nearest-even rounding of the updated value)
    for k in ("E", "W", "U", "W_out"):
        assert np.array_equal(host(tr._unpadded(tr._Pl)[k]), O.round_bf16(host(tr.P[k]))), k
    # second step reads the refreshed copies
    r1 = OS.lstm_lm_step(w.params, w.ids, w.targets, np.float32(w.lr), lowp=True)
    l2 = float(tr.step(ids, tg).cpu())
    r2 = OS.lstm_lm_step(r1["params"], w.ids, w.targets, np.float32(w.lr), lowp=True)
    assert abs(l2 - r2["loss"]) <= 2e-2 * abs(r2["loss"])


def test_graph_replay_equals_eager():
    # a captured step must reproduce the eager step bit for bit, on every replay, with eager work and
    # synchronisations in between
    w = W.config1()
    xd, td = torch.from_numpy(w.xs[0]).cuda(), torch.from_numpy(w.ts[0]).cuda()
    a = steps.MLPTrainer(w.params, w.batch, w.act, 0.1, False)
    b = steps.MLPTrainer(w.params, w.batch, w.act, 0.1, False)
    # the first graph step executes the program twice (eager warm-up, then the replay; the capture
    # pass itself executes nothing); mirror that on the eager side
    b.step(xd, td, graph=True)
    for _ in range(2):
        a.step(xd, td)
    for k in range(4):
        la = float(a.step(xd, td).cpu())
        lb = float(b.step(xd, td, graph=True).cpu())
        torch.cuda.synchronize()
        assert la == lb, (k, la, lb)
        for p, q in zip(a.W + a.b + a.dW + a.db, b.W + b.b + b.dW + b.db):
            assert torch.equal(p, q)
    wl = W.config4(vocab=200, embed=40, hidden=40, batch=8, bptt=3)
    ids, tg = torch.from_numpy(wl.ids).cuda(), torch.from_numpy(wl.targets).cuda()
    a = steps.LSTMTrainer(wl.params, wl.bptt, wl.batch, 0.1)
    b = steps.LSTMTrainer(wl.params, wl.bptt, wl.batch, 0.1)
    b.step(ids, tg, graph=True)
    for _ in range(2):
        a.step(ids, tg)
    for k in range(3):
        la, lb = float(a.step(ids, tg).cpu()), float(b.step(ids, tg, graph=True).cpu())
        assert la == lb, (k, la, lb)
        for name in a.P:
            assert torch.equal(a.P[name], b.P[name]) and torch.equal(a.g[name], b.g[name])


@pytest.mark.parametrize("lowp", [False, True])
def test_mlp_step_with_update_fused_into_the_weight_gradient_products(lowp):
    # the same step with W <- W - lr * dW applied in the epilogue of each dW product (and the bf16
    # working copies refreshed there): parameters, loss and logits must match the oracle's step, and
    # the unfused trainer's parameters to fp32 rounding of the update
    w = W.config5(n_batches=1, scale=8)
    tol = 2e-2 if lowp else 1e-4
    x, t = w.xs[0], w.ts[0]
    if lowp:
        x = bf16r(x)
    xd = torch.from_numpy(x).cuda()
    xd = xd.to(torch.bfloat16) if lowp else xd
    td = torch.from_numpy(t).cuda()
    fused = steps.MLPTrainer(w.params, w.batch, w.act, w.lr, lowp, fused_update=True)
    plain = steps.MLPTrainer(w.params, w.batch, w.act, w.lr, lowp)
    lf, lp = float(fused.step(xd, td).cpu()), float(plain.step(xd, td).cpu())
    assert lf == lp                                    # the forward passes are the same calls
    r = OS.mlp_step(w.params, x, t, np.float32(w.lr), w.act, lowp)
    lr = np.float32(w.lr)
    for l, ((dW, db), (Wn, bn)) in enumerate(zip(r["grads"], r["params"])):
        W0 = w.params[l][0]
        g = host(plain.dW[l])
        bound = np.abs(W0) + lr * np.abs(g)
        check(host(fused.W[l]), host(plain.W[l]), 1e-6, bound, "fused vs separate update, layer %d" % l)
        check(host(fused.W[l]), Wn, 1e-6, np.abs(W0) + float(lr) * tol * float(np.max(np.abs(dW))) / 1e-6, "param %d" % l)
        assert torch.equal(fused.b[l], plain.b[l])
        if lowp:
            assert np.array_equal(host(fused.Wl[l]), O.round_bf16(host(fused.W[l])))
    # and the second step starts from the updated weights in both
    l2f, l2p = float(fused.step(xd, td).cpu()), float(plain.step(xd, td).cpu())
    assert abs(l2f - l2p) <= 1e-5 * max(1.0, abs(l2p)) and l2f < lf
    assert fused.n_launch_calls(xd, td) == plain.n_launch_calls(xd, td)
