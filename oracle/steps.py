"""Whole training steps written as a sequence of oracle calls (TEST INFRASTRUCTURE).

A define-by-run step (Section "On Demand Graph Construction") is: run the forward computation
operation by operation, backtrack the recorded operations in reverse order calling each backward
once, then let the optimiser update every parameter once ("Background and Motivation": forward /
backward computation, then updating).  The functions below write that order out by hand for the two
model families the benchmark workloads use:

* the multilayer perceptron of the model-definition figure: Linear layers ``y = x @ W.T + b`` with
  ``W`` of shape (n_out, n_in), an activation between layers, softmax cross-entropy on top;
* a single-layer LSTM language model: embedding, gates ``x W + h U + b``, textbook LSTM cell,
  output Linear layer, softmax cross-entropy over all (time, batch) tokens, full back-propagation
  through the T-step window (no gradient into the zero initial state).

``lowp=True`` inserts a round-to-nearest-even bfloat16 rounding at every point where the mixed
precision scheme stores a bfloat16 array (working copies of weights, activations, activation
gradients); all arithmetic in between stays float64.  Weight/bias gradients, logits, the loss and the
master parameters are never rounded.
"""
import numpy as np

from . import oracle as O


ROUND = O.round_bf16     # the storage rounding (a pin replaces it by the identity: see the tests of this module)


def _st(x, lowp):
    return ROUND(x) if lowp else x


def mlp_step(params, x, t, lr, act="relu", lowp=False):
    """One forward + backward + SGD step of an MLP.

    params: list of (W (n_out,n_in), b (n_out,)) master parameters.
    Returns dict(loss, logits, grads=[(dW, db)...], params=[(W', b')...], acts=[...], stored=...).
    ``stored`` names every array the mixed-precision scheme keeps in bfloat16 (rounded when lowp):
    working copies of the weights ``Wc``, activations ``acts``, pre-activations kept for the GELU
    backward ``zs``, and the activation gradients ``dvs`` (index l: gradient of layer l's
    pre-activation; the last one is the logit gradient); ``dhs`` are the unrounded input gradients.
    """
    L = len(params)
    Ws = [_st(np.asarray(W, dtype=np.float64), lowp) for W, _ in params]
    hs = [np.asarray(x, dtype=np.float64)]
    zs = []                                   # stored pre-activations (GELU backward needs them)
    for l, (W, b) in enumerate(params):
        v = O.elementwise("add", [O.gemm(hs[-1], Ws[l].T), np.asarray(b, dtype=np.float64)])
        if l == L - 1:
            logits = v
            break
        zs.append(_st(v, lowp))
        hs.append(_st(O.elementwise(act, [v]), lowp))
    loss, _, _, _ = O.softmax_ce_fwd(logits, t)
    dv = _st(O.softmax_ce_bwd(logits, t), lowp)
    grads = [None] * L
    dvs, dhs = [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        dvs[l] = dv
        dW = O.gemm(dv.T, hs[l])
        db = O.reduce_axis("sum", dv, 0)
        grads[l] = (dW, db)
        if l > 0:
            dh = O.gemm(dv, Ws[l])
            dhs[l] = dh
            if act == "relu":
                dv = O.elementwise("relu_bwd", [dh, hs[l]])
            else:
                dv = O.elementwise("gelu_bwd", [dh, zs[l - 1]])
            dv = _st(dv, lowp)
    new = [(O.sgd_update(W, dW, lr), O.sgd_update(b, db, lr))
           for (W, b), (dW, db) in zip(params, grads)]
    return dict(loss=loss, logits=logits, grads=grads, params=new, acts=hs[1:],
                stored=dict(Wc=Ws, acts=hs[1:], zs=zs, dvs=dvs), dhs=dhs)


def mlp_loss(params, x, t, act="relu"):
    """Forward only (float64, no storage rounding): the scalar the finite-difference pins perturb."""
    h = np.asarray(x, dtype=np.float64)
    for l, (W, b) in enumerate(params):
        v = O.elementwise("add", [O.gemm(h, np.asarray(W, dtype=np.float64).T), b])
        h = v if l == len(params) - 1 else O.elementwise(act, [v])
    return O.softmax_ce_fwd(h, t)[0]


def lstm_lm_forward(P, ids, targets, lowp=False):
    """Forward of the LSTM language model.  P: dict(E, W, U, b, W_out, b_out); ids, targets (T,B).

    W (E_dim,4H) and U (H,4H) are stored so that the gates are x W + h U + b; W_out (V,H) follows the
    Linear convention y = h @ W_out.T + b_out.

    ``lowp``: the arrays that feed matrix products are stored in bfloat16 -- working copies of E, W, U
    and W_out, and every h; gate pre-activations, activated gates, the cell state, logits and the loss
    stay unrounded.
    """
    T, B = ids.shape
    H = P["U"].shape[0]
    Pl = {k: _st(np.asarray(P[k], dtype=np.float64), lowp) if k in ("E", "W", "U", "W_out") else np.asarray(P[k], dtype=np.float64)
          for k in P}
    X = O.embed_fwd(Pl["E"], ids.reshape(-1))                 # (T*B, E_dim), time-major
    Zx = O.gemm(X, Pl["W"])                                   # (T*B, 4H)
    h = np.zeros((B, H))
    c = np.zeros((B, H))
    Hs, Cs, Gs, Cprev, Hprev = [], [], [], [], []
    for t in range(T):
        z = O.gemm(h, Pl["U"], Zx[t * B:(t + 1) * B], 1.0, 1.0)
        Cprev.append(c)
        Hprev.append(h)
        c, h, g = O.lstm_fwd(z, P["b"], c)
        h = _st(h, lowp)
        Hs.append(h); Cs.append(c); Gs.append(g)
    Hall = np.concatenate(Hs, axis=0)                         # (T*B, H)
    logits = O.elementwise("add", [O.gemm(Hall, Pl["W_out"].T), P["b_out"]])
    loss = O.softmax_ce_fwd(logits, targets.reshape(-1))[0]
    return dict(loss=loss, logits=logits, X=X, Zx=Zx, Hall=Hall, Cs=Cs, Gs=Gs, Cprev=Cprev, Hprev=Hprev, Pl=Pl)


def lstm_lm_step(P, ids, targets, lr, lowp=False):
    """One forward + full BPTT + SGD step.  Returns dict(loss, grads{name}, params{name}, logits,
    stored{...}, unrounded{...}): ``stored`` holds the arrays kept in bfloat16 when lowp (working
    copies, embeddings X, hidden states Hall, dlogits, dHall, the per-step total hidden-state
    gradients dH and the gate gradients dZ), ``unrounded`` those that stay wide (Zx, gates, cell
    states, cell-state gradients dC, the embedding-output gradient dX).

    ``lowp`` additionally stores the activation gradients that feed matrix products in bfloat16:
    the logit gradients, the gradient of every h (rounded again after the recurrent term has been
    added into it) and the gate gradients; parameter gradients, the cell-state gradient, the
    embedding-output gradient and the master parameters are never rounded."""
    T, B = ids.shape
    H = P["U"].shape[0]
    V = P["E"].shape[0]
    F = lstm_lm_forward(P, ids, targets, lowp)
    Pl = F["Pl"]
    dlogits = _st(O.softmax_ce_bwd(F["logits"], targets.reshape(-1)), lowp)
    g = {}
    g["W_out"] = O.gemm(dlogits.T, F["Hall"])
    g["b_out"] = O.reduce_axis("sum", dlogits, 0)
    dHall = _st(O.gemm(dlogits, Pl["W_out"]), lowp)          # (T*B, H)
    dZ = np.zeros((T * B, 4 * H))
    dH_tot, dC = [None] * T, [None] * T
    dh_rec = None
    dc = None
    for t in range(T - 1, -1, -1):
        dh = dHall[t * B:(t + 1) * B]
        if dh_rec is not None:
            dh = _st(O.elementwise("add", [dh, dh_rec]), lowp)
        dH_tot[t] = dh
        dz, dc = O.lstm_bwd(F["Gs"][t], F["Cprev"][t], F["Cs"][t], dh, dc)
        dC[t] = dc
        dz = _st(dz, lowp)
        dZ[t * B:(t + 1) * B] = dz
        dh_rec = O.gemm(dz, Pl["U"].T)
    Hprev_all = np.concatenate(F["Hprev"], axis=0)
    g["U"] = O.gemm(Hprev_all.T, dZ)
    g["W"] = O.gemm(F["X"].T, dZ)
    g["b"] = O.reduce_axis("sum", dZ, 0)
    dX = O.gemm(dZ, Pl["W"].T)
    g["E"] = O.embed_bwd(ids.reshape(-1), dX, V)
    new = {k: O.sgd_update(P[k], g[k], lr) for k in g}
    return dict(loss=F["loss"], grads=g, params=new, logits=F["logits"],
                stored=dict(Wc={k: Pl[k] for k in ("E", "W", "U", "W_out")}, X=F["X"], Hall=F["Hall"], dlogits=dlogits,
                            dHall=dHall, dH=dH_tot, dZ=dZ),
                unrounded=dict(Zx=F["Zx"], Gs=F["Gs"], Cs=F["Cs"], dC=dC, dX=dX))
