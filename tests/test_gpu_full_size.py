"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot afford whole products at these sizes, so each call is checked teacher-forced (the
oracle gets the GPU call's own inputs) on outputs it can compute one by one: sampled GEMM entries as
fp64 dot products, sampled rows / columns of the array primitives, and full tensors for the cheap
calls (softmax cross-entropy, bias gradients, LSTM cell, embedding, SGD)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_1908_00213_amd import binding as B, steps, workloads as W
from tests.util import TOL_BF16, TOL_EW, TOL_SUM, check, host

pytestmark = pytest.mark.gpu
RNG = np.random.default_rng(8192)


def sample_gemm(A, Bm, n=256):
    """fp64 reference and term-magnitude sum for n random entries of A @ B (NumPy views)."""
    ms, ns = RNG.integers(0, A.shape[0], n), RNG.integers(0, Bm.shape[1], n)
    return ms, ns, O.gemm_entries(A, Bm, ms, ns), O.gemm_entries(np.abs(A), np.abs(Bm), ms, ns)


def h32(t):
    return host(t).astype(np.float32) if t.dtype != torch.float32 else t.cpu().numpy()


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_config2_full_size_array_primitives(dt):
    n = 8192
    w = W.config2(n)
    tdt = torch.float32 if dt == "f32" else torch.bfloat16
    a, b, c = (torch.from_numpy(x).cuda().to(tdt) for x in (w.a, w.b, w.c))
    ah, bh, ch = h32(a), h32(b), h32(c)                       # the values the kernels actually read
    tol = TOL_EW if dt == "f32" else TOL_BF16
    rows = np.sort(RNG.choice(n, 48, replace=False))
    y = B.elementwise_broadcast("mad_relu", [a, b, c], torch.empty(n, n, dtype=tdt, device="cuda"))
    yh = h32(y)
    ref = O.elementwise("mad_relu", [ah[rows], bh[rows], ch])
    check(yh[rows].astype(np.float64), ref, tol, O.elementwise("mad", [np.abs(ah[rows]), np.abs(bh[rows]), np.abs(ch)]), "mad_relu rows")
    at = a.t().contiguous().t()                                # same values, transposed storage
    assert at.stride() == (1, n)
    yt = B.elementwise_broadcast("mad_relu", [at, b, c], torch.empty(n, n, dtype=tdt, device="cuda"))
    assert torch.equal(y.view(torch.int16 if dt == "bf16" else torch.int32), yt.view(torch.int16 if dt == "bf16" else torch.int32))
    ws = torch.empty(B.reduce_axis_workspace_bytes(y, 0), dtype=torch.uint8, device="cuda")
    s0 = host(B.reduce_axis("sum", y, 0, torch.empty(n, device="cuda"), ws=ws))
    s1 = host(B.reduce_axis("sum", y, 1, torch.empty(n, device="cuda")))
    cols = np.sort(RNG.choice(n, 48, replace=False))
    tol_s = TOL_SUM if dt == "f32" else TOL_BF16
    check(s0[cols], O.reduce_axis("sum", yh[:, cols], 0), tol_s, O.reduce_axis("sum", np.abs(yh[:, cols]), 0), "sum axis 0")
    check(s1[rows], O.reduce_axis("sum", yh[rows], 1), tol_s, O.reduce_axis("sum", np.abs(yh[rows]), 1), "sum axis 1")
    # transposed views: the two kernels swap roles, the sums are the same sums
    ytv = y.t()
    wt = torch.empty(max(256, B.reduce_axis_workspace_bytes(ytv, 1)), dtype=torch.uint8, device="cuda")
    t0 = host(B.reduce_axis("sum", ytv, 0, torch.empty(n, device="cuda"), ws=wt))
    t1 = host(B.reduce_axis("sum", ytv, 1, torch.empty(n, device="cuda"), ws=wt))
    check(t0[rows], O.reduce_axis("sum", yh[rows], 1), tol_s, O.reduce_axis("sum", np.abs(yh[rows]), 1), "sum T axis 0")
    check(t1[cols], O.reduce_axis("sum", yh[:, cols], 0), tol_s, O.reduce_axis("sum", np.abs(yh[:, cols]), 0), "sum T axis 1")
    assert abs(s0.sum() - s1.sum()) <= 1e-5 * np.abs(yh).sum(dtype=np.float64)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_config2_full_size_user_defined_kernels(dt):
    """The benchmark's user-kernel lines: the figure's multiply-add with type parameter T, its
    ReLU variant with a row operand, and a user-written sum over either axis and over everything."""
    from oracle import user_kernel as OU
    n = 8192
    w = W.config2(n)
    tdt = torch.float32 if dt == "f32" else torch.bfloat16
    a, b, c = (torch.from_numpy(x).cuda().to(tdt) for x in (w.a, w.b, w.c))
    ah, bh, ch = h32(a), h32(b), h32(c)
    tol = TOL_EW if dt == "f32" else TOL_BF16
    tol_s = TOL_SUM if dt == "f32" else TOL_BF16
    rows = np.sort(RNG.choice(n, 48, replace=False))
    cols = np.sort(RNG.choice(n, 48, replace=False))
    mad = ("T x, T y, T z", "T w", "w = x * y + z", "my_mad")
    y = B.ElementwiseKernel(*mad)(a, b, a)
    check(host(y)[rows], OU.ElementwiseKernel(*mad)(ah[rows], bh[rows], ah[rows]), tol,
          np.abs(ah[rows] * bh[rows]) + np.abs(ah[rows]), "my_mad rows")
    mr = ("T x, T y, T z", "T w", "w = fmax(x * y + z, (T)0)", "my_mad_relu")
    y = B.ElementwiseKernel(*mr)(a, b, c)
    yh = h32(y)
    check(yh[rows].astype(np.float64), OU.ElementwiseKernel(*mr)(ah[rows], bh[rows], ch), tol,
          np.abs(ah[rows] * bh[rows]) + np.abs(ch), "my_mad_relu rows")
    sm = ("T x", "float32 y", "x", "a + b", "y = a", "0", "my_sum")
    k, ko = B.ReductionKernel(*sm), OU.ReductionKernel(*sm)
    s0, s1, sa = host(k(y, axis=0)), host(k(y, axis=1)), float(k(y, axis=None).cpu())
    check(s0[cols], ko(yh[:, cols], axis=0), tol_s, np.abs(yh[:, cols]).sum(axis=0, dtype=np.float64), "user sum axis 0")
    check(s1[rows], ko(yh[rows], axis=1), tol_s, np.abs(yh[rows]).sum(axis=1, dtype=np.float64), "user sum axis 1")
    total = float(ko(yh, axis=None))
    assert abs(sa - total) <= tol_s * float(np.abs(yh).sum(dtype=np.float64))


def test_config5_full_size_step_sampled():
    w = W.config5(n_batches=1)
    x = W.bf16_exact(w.xs[0])
    t = w.ts[0]
    tr = steps.MLPTrainer(w.params, w.batch, w.act, w.lr, lowp=True)
    W0 = [h32(m) for m in tr.W]                               # masters before the step
    Wl0 = [h32(m) for m in tr.Wl]                             # bf16 working copies the GEMMs read
    xd, td = torch.from_numpy(x).cuda().to(torch.bfloat16), torch.from_numpy(t).cuda()
    loss = float(tr.step(xd, td).cpu())
    torch.cuda.synchronize()
    n = len(tr.W)
    hs = [x] + [h32(hh) for hh in tr.h[1:]]
    zs = [None] + [h32(z) for z in tr.z[1:]]
    dvs = [None] + [h32(d) for d in tr.dv[1:]]
    bias = [b.cpu().numpy() for b in tr.b]                    # biases after the update; recover the old ones
    db = [d.cpu().numpy() for d in tr.db]
    b_old = [p[1] for p in w.params]
    # forward layers
    for l in range(n):
        ms, ns, ref, S = sample_gemm(hs[l], Wl0[l].T)
        v = ref + b_old[l][ns]
        if l < n - 1:
            check(zs[l + 1][ms, ns].astype(np.float64), v, TOL_BF16, S, "z%d" % l)
            check(hs[l + 1][ms, ns].astype(np.float64), O.elementwise("gelu", [v]), TOL_BF16, S, "h%d" % l)
        else:
            logits = tr.logits.cpu().numpy()
            check(logits[ms, ns].astype(np.float64), v, TOL_SUM, S, "logits")      # fp32 out of exact bf16 inputs
    rl, _, _, nv = O.softmax_ce_fwd(logits, t)
    assert abs(loss - rl) <= TOL_SUM * abs(rl) and nv == w.batch
    check(dvs[n].astype(np.float64), O.softmax_ce_bwd(logits, t), TOL_BF16, 1.0 / w.batch, "dlogits")
    # backward layers, teacher-forced on the GPU's own bf16 gradients
    for l in range(n - 1, -1, -1):
        dv = dvs[l + 1]
        ms, ns, ref, S = sample_gemm(dv.T, hs[l])
        check(tr.dW[l].cpu().numpy()[ms, ns].astype(np.float64), ref, TOL_SUM, S, "dW%d" % l)
        check(db[l].astype(np.float64), O.reduce_axis("sum", dv, 0), TOL_SUM, O.reduce_axis("sum", np.abs(dv), 0), "db%d" % l)
        if l > 0:
            ms, ns, ref, S = sample_gemm(dv, Wl0[l])
            g = O.elementwise("gelu_bwd", [ref, zs[l][ms, ns]])
            check(dvs[l][ms, ns].astype(np.float64), g, TOL_BF16, S * 1.2, "dx%d" % l)
    # optimiser: new master = old - lr * (the GPU's gradient), working copy = RNE of the new master
    lr = np.float32(w.lr)
    for l in (0, n - 1):
        gW = tr.dW[l].cpu().numpy()
        newW = tr.W[l].cpu().numpy()
        check(newW.astype(np.float64), O.sgd_update(W0[l], gW, lr), 1e-6, np.abs(W0[l]) + lr * np.abs(gW), "W%d" % l)
        assert np.array_equal(h32(tr.Wl[l]).astype(np.float64), O.round_bf16(newW))
        check(bias[l].astype(np.float64), O.sgd_update(b_old[l], db[l], lr), 1e-6, np.abs(b_old[l]) + lr * np.abs(db[l]), "b%d" % l)


def test_config5_full_size_step_as_benchmarked_update_in_the_weight_gradient_products():
    """The trainer exactly as bench.py runs it: the weight-gradient products apply the SGD update in
    their epilogue and refresh the bf16 working copies, the hidden layers' bias gradients come from
    the row-block column sums.  Teacher-forced on the step's own activations and gradients: sampled
    entries of every updated weight matrix, every working copy, every bias."""
    w = W.config5(n_batches=1)
    x = W.bf16_exact(w.xs[0])
    tr = steps.MLPTrainer(w.params, w.batch, w.act, w.lr, lowp=True, fused_update=True)
    assert sorted(tr.rowsums) == [1, 2, 3]
    W0 = [m.clone() for m in tr.W]
    xd, td = torch.from_numpy(x).cuda().to(torch.bfloat16), torch.from_numpy(w.ts[0]).cuda()
    loss = float(tr.step(xd, td).cpu())
    torch.cuda.synchronize()
    assert np.isfinite(loss)
    n = len(tr.W)
    hs = [x] + [h32(hh) for hh in tr.h[1:]]
    lr = np.float32(w.lr)
    for l in range(n):
        dv = h32(tr.dv[l + 1])
        ms, ns, ref, S = sample_gemm(dv.T, hs[l])
        old = W0[l].cpu().numpy()[ms, ns].astype(np.float64)
        new = tr.W[l].cpu().numpy()
        check(new[ms, ns].astype(np.float64), old - float(lr) * ref, TOL_SUM, np.abs(old) + float(lr) * S, "W%d" % l)
        assert np.array_equal(h32(tr.Wl[l]).astype(np.float64), O.round_bf16(new)), "working copy %d" % l
        db = tr.db[l].cpu().numpy()
        check(db.astype(np.float64), O.reduce_axis("sum", dv, 0), TOL_SUM, O.reduce_axis("sum", np.abs(dv), 0), "db%d" % l)
        b_old = w.params[l][1]
        check(tr.b[l].cpu().numpy().astype(np.float64), O.sgd_update(b_old, db, lr), 1e-6, np.abs(b_old) + lr * np.abs(db), "b%d" % l)


def test_config4_full_size_step_sampled():
    w = W.config4()
    T, Bn, H, V = w.bptt, w.batch, w.hidden, w.vocab
    tr = steps.LSTMTrainer(w.params, T, Bn, w.lr)
    ids, tg = torch.from_numpy(w.ids).cuda(), torch.from_numpy(w.targets).cuda()
    prog = tr._build(ids, tg)
    L = B.lib()
    P0 = {k: v.copy() for k, v in w.params.items()}
    # run the recorded calls one by one; keep the logits before the gradient overwrites them in place
    logits = None
    for fn, args in prog.calls:
        if fn is L.chn_softmax_ce_fwd_bwd and logits is None:
            logits = tr.logits.cpu().numpy()
        B._check(fn(*args, None))
    torch.cuda.synchronize()
    idf, tgf = w.ids.reshape(-1), w.targets.reshape(-1)
    X = tr.X.cpu().numpy()
    assert np.array_equal(X, P0["E"][idf])                                           # gather is a bit copy
    Hs, Cs, Z, G = (m.cpu().numpy() for m in (tr.Hs, tr.Cs, tr.Z, tr.G))
    Hprev, Hall = Hs[:T * Bn], Hs[Bn:]
    # gate pre-activations x W + h U, sampled
    # the configuration the benchmark times: Z holds x W only, one launch for the 35 forward steps, one for the 35 backward steps
    assert tr.fused_step and tr.whole_sequence and tr.whole_sequence_bwd and tr.sequence_complete()
    ms, ns = RNG.integers(0, T * Bn, 256), RNG.integers(0, 4 * H, 256)
    ref = O.gemm_entries(X, P0["W"], ms, ns)
    S = O.gemm_entries(np.abs(X), np.abs(P0["W"]), ms, ns)
    check(Z[ms, ns].astype(np.float64), ref, TOL_SUM, S, "input part of the gate pre-activations")
    # fused step (recurrent product + cell), whole steps, from the GPU's own inputs of that step
    for t in (0, 1, T // 2, T - 1):
        sl = slice(t * Bn, (t + 1) * Bn)
        z = O.gemm(Hprev[sl], P0["U"], Z[sl], 1.0, 1.0)
        Sz = O.gemm(np.abs(Hprev[sl]), np.abs(P0["U"])) + np.abs(Z[sl]) + np.abs(P0["b"])
        c, h, g = O.lstm_fwd(z, P0["b"], Cs[sl])
        check(G[sl].astype(np.float64), g, TOL_SUM, Sz, "gates %d" % t)
        Sc = np.abs(g[:, H:2 * H] * Cs[sl]) + np.abs(g[:, :H] * g[:, 2 * H:3 * H]) + Sz[:, :H] + Sz[:, H:2 * H] * np.abs(Cs[sl]) + Sz[:, 2 * H:3 * H]
        check(Cs[t * Bn + Bn:(t + 2) * Bn].astype(np.float64), c, TOL_SUM, Sc, "c %d" % t)
        check(Hall[sl].astype(np.float64), h, TOL_SUM, Sc + Sz[:, 3 * H:], "h %d" % t)
    ms, ns, ref, S = sample_gemm(Hall, P0["W_out"].T)
    check(logits[ms, ns].astype(np.float64), ref + P0["b_out"][ns], TOL_SUM, S, "logits")
    rl, _, _, nv = O.softmax_ce_fwd(logits, tgf)
    assert abs(float(tr.loss.cpu()) - rl) <= TOL_SUM * rl and nv == T * Bn
    dlog = tr.logits.cpu().numpy()
    check(dlog.astype(np.float64), O.softmax_ce_bwd(logits, tgf), TOL_EW * 10, 1.0 / nv, "dlogits")
    g = {k: v.cpu().numpy() for k, v in tr.g.items()}
    ms, ns, ref, S = sample_gemm(dlog.T, Hall)
    check(g["W_out"][ms, ns].astype(np.float64), ref, TOL_SUM, S, "dW_out")
    check(g["b_out"].astype(np.float64), O.reduce_axis("sum", dlog, 0), TOL_SUM, O.reduce_axis("sum", np.abs(dlog), 0), "db_out")
    # dHs holds the total dh_t (output layer + recurrence); the chain is replayed teacher-forced
    dHs, dZ = tr.dHs.cpu().numpy(), tr.dZ.cpu().numpy()
    t = T - 1
    ms, ns, ref, S = sample_gemm(dlog[t * Bn:], P0["W_out"])
    check(dHs[t * Bn:][ms % Bn, ns].astype(np.float64), O.gemm_entries(dlog[t * Bn:], P0["W_out"], ms % Bn, ns), TOL_SUM,
          O.gemm_entries(np.abs(dlog[t * Bn:]), np.abs(P0["W_out"]), ms % Bn, ns), "dh last step")
    dc = None
    for t in range(T - 1, -1, -1):
        sl = slice(t * Bn, (t + 1) * Bn)
        dz, dc = O.lstm_bwd(G[sl], Cs[sl], Cs[t * Bn + Bn:(t + 2) * Bn], dHs[sl], dc)
        if t in (T - 1, T - 2, 0):
            Sdc = np.abs(dc) + np.abs(dHs[sl])
            check(dZ[sl].astype(np.float64), dz, TOL_EW * 10, np.concatenate([Sdc, Sdc * np.abs(Cs[sl]) + Sdc, Sdc, np.abs(dHs[sl])], axis=1), "dz %d" % t)
        if t > 0:      # dh_{t-1} = (output-layer part) + dz_t U^T: check the recurrent part on samples
            ms, ns = RNG.integers(0, Bn, 16), RNG.integers(0, H, 16)
            rec = O.gemm_entries(dZ[sl], P0["U"].T, ms, ns)
            out = O.gemm_entries(dlog[(t - 1) * Bn:t * Bn], P0["W_out"], ms, ns)
            S = O.gemm_entries(np.abs(dZ[sl]), np.abs(P0["U"].T), ms, ns) + O.gemm_entries(np.abs(dlog[(t - 1) * Bn:t * Bn]), np.abs(P0["W_out"]), ms, ns)
            check(dHs[(t - 1) * Bn:t * Bn][ms, ns].astype(np.float64), rec + out, TOL_SUM, S, "dh %d" % (t - 1))
    for name, A, Bm in (("U", Hprev.T, dZ), ("W", X.T, dZ)):
        ms, ns, ref, S = sample_gemm(A, Bm)
        check(g[name][ms, ns].astype(np.float64), ref, TOL_SUM, S, "d" + name)
    check(g["b"].astype(np.float64), O.reduce_axis("sum", dZ, 0), TOL_SUM, O.reduce_axis("sum", np.abs(dZ), 0), "db")
    dX = tr.dX.cpu().numpy()
    ms, ns, ref, S = sample_gemm(dZ, P0["W"].T)
    check(dX[ms, ns].astype(np.float64), ref, TOL_SUM, S, "dX")
    check(g["E"].astype(np.float64), O.embed_bwd(idf, dX, V), TOL_SUM, O.embed_bwd(idf, np.abs(dX), V), "dE")
    lr = np.float32(w.lr)
    for k in P0:
        check(tr.P[k].cpu().numpy().astype(np.float64), O.sgd_update(P0[k], g[k], lr), 1e-6, np.abs(P0[k]) + lr * np.abs(g[k]), "update " + k)


def test_config4_full_size_mixed_precision_sampled():
    """Workload 4 in mixed precision at full size: every product checked on sampled entries against
    fp64 dot products of the very bf16 operands it read (so the bar is the fp32-accumulation one),
    every bf16 store against the bf16 bar."""
    w = W.config4()
    T, Bn, H, V = w.bptt, w.batch, w.hidden, w.vocab
    tr = steps.LSTMTrainer(w.params, T, Bn, w.lr, lowp=True)
    ids, tg = torch.from_numpy(w.ids).cuda(), torch.from_numpy(w.targets).cuda()
    Pl0 = {k: host(v) for k, v in tr._unpadded(tr._Pl).items()}          # the working copies the step reads
    P0 = {k: host(v) for k, v in tr.P.items()}
    for k in ("E", "W", "U", "W_out"):
        assert np.array_equal(Pl0[k], O.round_bf16(P0[k]))
    tr.step(ids, tg)
    torch.cuda.synchronize()
    idf, tgf = w.ids.reshape(-1), w.targets.reshape(-1)
    X, Hs, Cs, Z, G = (host(m) for m in (tr.X, tr.Hs, tr.Cs, tr.Z, tr.G))
    assert np.array_equal(X, Pl0["E"][idf])
    Hprev, Hall = Hs[:T * Bn], Hs[Bn:]
    assert tr.fused_step and tr.whole_sequence and tr.sequence_complete()
    ms, ns = RNG.integers(0, T * Bn, 256), RNG.integers(0, 4 * H, 256)
    ref = O.gemm_entries(X, Pl0["W"], ms, ns)
    S = O.gemm_entries(np.abs(X), np.abs(Pl0["W"]), ms, ns)
    check(Z[ms, ns], ref, TOL_SUM, S, "input part of the gate pre-activations")
    for t in (0, T // 2, T - 1):
        sl = slice(t * Bn, (t + 1) * Bn)
        z = O.gemm(Hprev[sl], Pl0["U"], Z[sl], 1.0, 1.0)
        Sz = O.gemm(np.abs(Hprev[sl]), np.abs(Pl0["U"])) + np.abs(Z[sl]) + np.abs(P0["b"])
        c, h, g = O.lstm_fwd(z, P0["b"], Cs[sl])
        check(G[sl], g, TOL_SUM, Sz, "gates %d" % t)
        Sc = np.abs(g[:, H:2 * H] * Cs[sl]) + np.abs(g[:, :H] * g[:, 2 * H:3 * H]) + Sz[:, :H] + Sz[:, H:2 * H] * np.abs(Cs[sl]) + Sz[:, 2 * H:3 * H]
        check(Cs[t * Bn + Bn:(t + 2) * Bn], c, TOL_SUM, Sc, "c %d" % t)
        check(Hall[sl], h, TOL_BF16, Sc + Sz[:, 3 * H:], "h %d" % t)
    logits = host(tr.logits)
    ms, ns, ref, S = sample_gemm(Hall, Pl0["W_out"].T)
    check(logits[ms, ns], ref + P0["b_out"][ns], TOL_SUM, S, "logits")
    rl, _, _, nv = O.softmax_ce_fwd(logits, tgf)
    assert abs(float(tr.loss.cpu()) - rl) <= TOL_SUM * rl
    dlog = host(tr._dlogits)
    rows = np.sort(RNG.choice(T * Bn, 64, replace=False))
    check(dlog[rows], O.softmax_ce_bwd(logits, tgf)[rows], TOL_BF16, 1.0 / nv, "dlogits")
    g = {k: host(v) for k, v in tr.g.items()}
    ms, ns, ref, S = sample_gemm(dlog.T, Hall)
    check(g["W_out"][ms, ns], ref, TOL_SUM, S, "dW_out")
    check(g["b_out"], O.reduce_axis("sum", dlog, 0), TOL_SUM, O.reduce_axis("sum", np.abs(dlog), 0), "db_out")
    dHs, dZ, dX = host(tr.dHs), host(tr.dZ), host(tr.dX)
    t = T - 1
    ms, ns = RNG.integers(0, Bn, 128), RNG.integers(0, H, 128)
    check(dHs[t * Bn:][ms, ns], O.gemm_entries(dlog[t * Bn:], Pl0["W_out"], ms, ns), TOL_BF16,
          O.gemm_entries(np.abs(dlog[t * Bn:]), np.abs(Pl0["W_out"]), ms, ns), "dh last step")
    dz, _ = O.lstm_bwd(G[t * Bn:(t + 1) * Bn], Cs[t * Bn:(t + 1) * Bn], Cs[(t + 1) * Bn:(t + 2) * Bn], dHs[t * Bn:], None)
    Sd = np.abs(dHs[t * Bn:])
    check(dZ[t * Bn:], dz, TOL_BF16, np.concatenate([Sd, Sd * (1 + np.abs(Cs[t * Bn:(t + 1) * Bn])), Sd, Sd], axis=1), "dz last step")
    for name, A, Bm in (("U", Hprev.T, dZ), ("W", X.T, dZ)):
        ms, ns, ref, S = sample_gemm(A, Bm)
        check(g[name][ms, ns], ref, TOL_SUM, S, "d" + name)
    check(g["b"], O.reduce_axis("sum", dZ, 0), TOL_SUM, O.reduce_axis("sum", np.abs(dZ), 0), "db")
    ms, ns, ref, S = sample_gemm(dZ, Pl0["W"].T)
    check(dX[ms, ns], ref, TOL_SUM, S, "dX")
    check(g["E"], O.embed_bwd(idf, dX, V), TOL_SUM, O.embed_bwd(idf, np.abs(dX), V), "dE")
    lr = np.float32(w.lr)
    for k in P0:
        new = host(tr.P[k])
        check(new, O.sgd_update(P0[k], g[k], lr), 1e-6, np.abs(P0[k]) + lr * np.abs(g[k]), "update " + k)
        if k in ("E", "W", "U", "W_out"):
            assert np.array_equal(host(tr._unpadded(tr._Pl)[k]), O.round_bf16(new)), k


# ---- every tile of the benchmarked launches, bit for bit --------------------------------------------------------
# Operands are small integers (|v| <= 3): every partial sum is an integer below 2^24, so the product is exact
# in fp32 in any summation order and the WHOLE output must equal the exact product bit for bit.  The exact
# product is NumPy's fp64 matmul, tied to the oracle on a stratified sample: in every 256 x 256 tile of the
# output its four corner entries and one random interior entry (so every tile and every tile-edge row and
# column is looked at), plus the matrix's last rows and columns.
def _int_operand(shape, transposed_storage):
    """bf16 tensor of small integers with the given logical shape; stored transposed when asked."""
    v = RNG.integers(-3, 4, size=shape).astype(np.float32)
    if transposed_storage:
        t = torch.from_numpy(np.ascontiguousarray(v.T)).cuda().to(torch.bfloat16).t()
    else:
        t = torch.from_numpy(v).cuda().to(torch.bfloat16)
    return v, t


def _tie_to_oracle(A, Bm, ref):
    M, N = ref.shape
    ms, ns = [], []
    for tm in range(0, M, 256):
        for tn in range(0, N, 256):
            r1, c1 = min(tm + 255, M - 1), min(tn + 255, N - 1)
            ms += [tm, tm, r1, r1, int(RNG.integers(tm, r1 + 1))]
            ns += [tn, c1, tn, c1, int(RNG.integers(tn, c1 + 1))]
    got = O.gemm_entries(A, Bm, ms, ns)
    assert np.array_equal(got, ref[ms, ns])


@pytest.fixture(params=["planned", "four waves", "eight waves"])
def direct_kernel(request):
    """The headline products run on the 256x256 direct-copy path, which has two kernels; the planner picks
    one per call.  Every whole-output test runs as planned and with each kernel forced."""
    B.gemm_plan_override(direct_copy={"planned": -1, "four waves": 2, "eight waves": 3}[request.param])
    yield request.param
    B.gemm_plan_override()


# the three layouts of a hidden layer of workload 5 (forward x W^T, input gradient dY W, weight gradient dY^T X)
# and of its 1000-class output layer
HEADLINE_PRODUCTS = [
    ("fwd hidden", 8192, 4096, 4096, False, True),      # A (M,K) row-major, B = W^T: W (N,K) row-major
    ("dx hidden", 8192, 4096, 4096, False, False),      # B = W (K,N) row-major
    ("dW hidden", 4096, 4096, 8192, True, False),       # A = dY^T: dY (K,M) row-major
    ("fwd classes", 8192, 1000, 4096, False, True),
    ("dx classes", 8192, 4096, 1000, False, False),
    ("dW classes", 1000, 4096, 8192, True, False),
]


@pytest.mark.parametrize("name,M,N,K,a_t,b_t", HEADLINE_PRODUCTS)
def test_headline_products_whole_output_bit_exact(name, M, N, K, a_t, b_t, direct_kernel):
    A, Ad = _int_operand((M, K), a_t)
    Bm, Bd = _int_operand((K, N), b_t)
    ref = A.astype(np.float64) @ Bm.astype(np.float64)
    _tie_to_oracle(A, Bm, ref)
    Cd = torch.empty(M, N, dtype=torch.float32, device="cuda")
    need = B.gemm_workspace_bytes(Ad, Bd, Cd)
    ws = torch.empty(max(256, need), dtype=torch.uint8, device="cuda")
    B.gemm(Ad, Bd, Cd, ws=ws)
    out = Cd.cpu().numpy()
    bad = np.argwhere(out != ref)
    assert bad.size == 0, "%s: %d entries differ, first at %s (tile %s)" % (name, len(bad), bad[0], bad[0] // 256)


def test_headline_forward_epilogue_whole_output(direct_kernel):
    """The benchmarked forward launch itself: bias + GELU, bf16 output and bf16 pre-activation.  With integer
    operands and an integer bias v = acc + bias is exact, so the stored pre-activation must be the
    nearest-even bf16 of the exact value everywhere; the activation is compared within the bf16 bar."""
    M, N, K = 8192, 4096, 4096
    A, Ad = _int_operand((M, K), False)
    Bm, Bd = _int_operand((K, N), True)
    bias = RNG.integers(-5, 6, size=N).astype(np.float32)
    ref = A.astype(np.float64) @ Bm.astype(np.float64)
    _tie_to_oracle(A, Bm, ref)
    v = ref + bias
    out = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    pre = torch.empty_like(out)
    B.gemm(Ad, Bd, out, epilogue="bias_gelu", bias=torch.from_numpy(bias).cuda(), preact_out=pre)
    got_pre = pre.float().cpu().numpy()
    rows = np.sort(RNG.choice(M, 64, replace=False))
    assert np.array_equal(O.round_bf16(v[rows]), W.bf16_exact(v[rows].astype(np.float32)))    # host rounding helper tied to the oracle's
    assert np.array_equal(got_pre, W.bf16_exact(v.astype(np.float32)))                         # v is an integer below 2^24: the cast is exact
    got = out.float().cpu().numpy().astype(np.float64)
    gref = O.elementwise("gelu", [v[rows]])
    check(got[rows], gref, TOL_BF16, np.abs(v[rows]), "gelu rows")
    # everywhere: SciPy's erf form over the whole output (tied to the oracle's gelu on the sampled rows above)
    import scipy.special as sps
    full = 0.5 * v * (1.0 + sps.erf(v / np.sqrt(2.0)))
    assert np.max(np.abs(full[rows] - gref)) <= 1e-12 * np.max(np.abs(v))
    check(got, full, TOL_BF16, np.abs(v), "gelu everywhere")


def test_headline_input_gradient_epilogue_and_row_block_sums_whole_output(direct_kernel):
    """dx of a hidden layer as benchmarked: the activation-gradient epilogue with the per-128-row column sums.
    With the ReLU gradient and integer data everything is exact: C = RNE_bf16(acc * [aux > 0]) and the row-block
    sums are sums of those stored integers (below 2^24), so both outputs are compared bit for bit; the GELU
    gradient form (the one the benchmark runs) is compared within the bf16 bar on sampled rows and its row-block
    sums against the sums of what it stored."""
    M, N, K = 8192, 4096, 4096
    A, Ad = _int_operand((M, K), False)
    Bm, Bd = _int_operand((K, N), False)
    aux = RNG.integers(-2, 3, size=(M, N)).astype(np.float32)
    auxd = torch.from_numpy(aux).cuda().to(torch.bfloat16)
    ref = A.astype(np.float64) @ Bm.astype(np.float64)
    _tie_to_oracle(A, Bm, ref)
    out = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    sums = torch.empty(M // 128, N, dtype=torch.float32, device="cuda")
    B.gemm(Ad, Bd, out, epilogue="relu_bwd", aux=auxd, preact_out=sums)
    want = W.bf16_exact((ref * (aux > 0)).astype(np.float32)).astype(np.float64)
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.array_equal(got, want)
    assert np.array_equal(sums.cpu().numpy().astype(np.float64), want.reshape(M // 128, 128, N).sum(axis=1))
    rows = np.sort(RNG.choice(M, 48, replace=False))
    assert np.array_equal(O.elementwise("relu_bwd", [ref[rows], aux[rows]]), ref[rows] * (aux[rows] > 0))
    B.gemm(Ad, Bd, out, epilogue="gelu_bwd", aux=auxd, preact_out=sums)
    got = out.float().cpu().numpy().astype(np.float64)
    check(got[rows], O.elementwise("gelu_bwd", [ref[rows], aux[rows]]), TOL_BF16, np.abs(ref[rows]), "gelu_bwd rows")
    blk = got.reshape(M // 128, 128, N)
    check(sums.cpu().numpy().astype(np.float64), blk.sum(axis=1), TOL_SUM, np.abs(blk).sum(axis=1), "row-block sums")


def test_headline_weight_gradient_with_fused_update_whole_output(direct_kernel):
    """dW of a hidden layer as benchmarked: alpha = -lr, beta = 1 on the fp32 master weights, bf16 copy written in
    the same pass.  lr = 2^-7 and masters on a 2^-4 grid keep v = W - lr * dW exact in fp32, so the masters are
    compared bit for bit and the working copy is the nearest-even bf16 of them."""
    M, N, K = 4096, 4096, 8192
    A, Ad = _int_operand((M, K), True)
    Bm, Bd = _int_operand((K, N), False)
    W0 = (RNG.integers(-32, 33, size=(M, N)) / 16.0).astype(np.float32)
    ref = A.astype(np.float64) @ Bm.astype(np.float64)
    _tie_to_oracle(A, Bm, ref)
    lr = 2.0 ** -7
    Wd = torch.from_numpy(W0.copy()).cuda()
    Wl = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    B.gemm(Ad, Bd, Wd, alpha=-lr, beta=1.0, epilogue="bf16_copy", preact_out=Wl)
    want = W0.astype(np.float64) - lr * ref
    rows = np.sort(RNG.choice(M, 16, replace=False))
    assert np.array_equal(O.sgd_update(W0[rows], ref[rows], lr), want[rows])
    assert np.array_equal(Wd.cpu().numpy().astype(np.float64), want)
    assert np.array_equal(Wl.float().cpu().numpy(), W.bf16_exact(want.astype(np.float32)))
