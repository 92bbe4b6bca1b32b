"""A tape backend whose kernels are the CPU oracle's functions (float64 NumPy arrays).

It lets the host logic of the define-by-run tape -- recording, ordering, accumulation, release --
be tested where no GPU exists, and compared with the hand-written oracle steps.  Fresh arrays are
filled with NaN so that a function reading a buffer nobody wrote shows up in the result.
"""
import numpy as np

from oracle import oracle as O


class OracleBackend:
    def __init__(self):
        self.calls = []                       # (name, detail) per kernel call, in issue order
        self.live_bytes = 0

    def empty(self, shape, dtype="f32"):
        if dtype in ("i64", "i32"):
            return np.zeros(tuple(shape), dtype=np.int64)
        return np.full(tuple(shape), np.nan, dtype=np.float64)

    def dtype(self, a):
        return "i64" if np.issubdtype(a.dtype, np.integer) else "f32"

    def from_numpy(self, a, dtype=None):
        a = np.asarray(a)
        return a.astype(np.int64) if np.issubdtype(a.dtype, np.integer) else a.astype(np.float64)

    def to_numpy(self, a):
        return np.asarray(a)

    def gemm(self, A, Bm, Cm, alpha=1.0, beta=0.0, epilogue="none", bias=None, aux=None, preact_out=None):
        self.calls.append(("gemm", epilogue))
        v = O.gemm(A, Bm, Cm if beta != 0.0 else None, alpha, beta)
        if epilogue in ("bias", "bias_relu", "bias_gelu"):
            v = O.elementwise("add", [v, bias])
            if preact_out is not None:
                preact_out[...] = v
            if epilogue != "bias":
                v = O.elementwise(epilogue[5:], [v])
        elif epilogue in ("relu_bwd", "gelu_bwd"):
            v = O.elementwise(epilogue, [v, aux])
        elif epilogue != "none":
            raise ValueError(epilogue)
        Cm[...] = v
        return Cm

    def elementwise_broadcast(self, op, inputs, out, scalars=()):
        self.calls.append(("elementwise", op))
        out[...] = O.elementwise(op, list(inputs), out.shape, scalars)
        return out

    def reduce_axis(self, op, x, axis, out):
        self.calls.append(("reduce", op))
        out[...] = O.reduce_axis(op, x, axis)
        return out

    def lstm_fwd(self, z, bias, c_prev, c, h, gates):
        self.calls.append(("lstm_fwd", None))
        c[...], h[...], gates[...] = O.lstm_fwd(z, bias, c_prev)

    fuse_lstm_step = False                    # tests switch it on to walk the fused-step code path

    def fuses_lstm_step(self, hidden):
        return self.fuse_lstm_step

    def lstm_step_fwd(self, zx, h_prev, Ut, bias, c_prev, c, h, gates):
        self.calls.append(("lstm_step_fwd", None))
        z = O.gemm(h_prev, Ut.T, zx, 1.0, 1.0)
        c[...], h[...], gates[...] = O.lstm_fwd(z, bias, c_prev)

    def lstm_steps_fwd(self, zx, Hs, Ut, bias, Cs, gates, n_steps):
        Bn = zx.shape[0] // n_steps
        blk = lambda a, t: a[t * Bn:(t + 1) * Bn]
        for t in range(n_steps):
            self.lstm_step_fwd(blk(zx, t), blk(Hs, t), Ut, bias, blk(Cs, t), blk(Cs, t + 1), blk(Hs, t + 1), blk(gates, t))

    def lstm_steps_bwd(self, dZ, U, dHs, gates, Cs, dc_last, dc, n_steps):
        Bn = dZ.shape[0] // n_steps
        blk = lambda a, t: a[t * Bn:(t + 1) * Bn]
        dc_next = dc_last
        for t in range(n_steps - 1, -1, -1):
            self.lstm_step_bwd(None if t == n_steps - 1 else blk(dZ, t + 1), U, blk(dHs, t), blk(gates, t), blk(Cs, t), blk(Cs, t + 1),
                               dc_next, blk(dZ, t), dc[t & 1])
            dc_next = dc[t & 1]

    def lstm_step_bwd(self, dz_next, U, dh, gates, c_prev, c, dc_next, dz, dc_prev):
        self.calls.append(("lstm_step_bwd", None))
        if dz_next is not None:
            dh[...] = O.gemm(dz_next, U.T, dh, 1.0, 1.0)
        dz[...], dc_prev[...] = O.lstm_bwd(gates, c_prev, c, dh, dc_next)

    def lstm_bwd(self, gates, c_prev, c, dh, dc_next, dz, dc_prev):
        self.calls.append(("lstm_bwd", None))
        dz[...], dc_prev[...] = O.lstm_bwd(gates, c_prev, c, dh, dc_next)

    def softmax_ce_fwd(self, logits, labels, loss_mean, lse, ignore_label):
        self.calls.append(("softmax_ce_fwd", None))
        loss, _, l, _ = O.softmax_ce_fwd(logits, labels, ignore_label)
        loss_mean[...] = loss
        lse[...] = l

    def softmax_ce_bwd(self, logits, labels, dlogits, lse, upstream, ignore_label):
        self.calls.append(("softmax_ce_bwd", None))
        dlogits[...] = O.softmax_ce_bwd(logits, labels, ignore_label, upstream)

    def softmax_ce_bwd2(self, logits, labels, gg, dlogits, dupstream, lse, upstream, ignore_label):
        self.calls.append(("softmax_ce_bwd2", None))
        dz, du = O.softmax_ce_bwd2(logits, labels, gg, ignore_label, upstream)
        dlogits[...] = dz
        if dupstream is not None:
            dupstream[...] = du

    def embed_fwd(self, table, ids, out):
        self.calls.append(("embed_fwd", None))
        out[...] = O.embed_fwd(table, ids)

    def embed_bwd(self, ids, dout, dtable, accumulate):
        self.calls.append(("embed_bwd", accumulate))
        dtable[...] = O.embed_bwd(ids, dout, dtable.shape[0], dtable if accumulate else None)

    def sgd_update_multi(self, params, grads, lr, lowp_copies):
        self.calls.append(("sgd", len(params)))
        for p, g in zip(params, grads):
            p[...] = O.sgd_update(p, g, lr)

    def adam_update_multi(self, params, grads, ms, vs, lr, step, beta1, beta2, eps, lowp_copies):
        self.calls.append(("adam", len(params)))
        for p, g, m, v in zip(params, grads, ms, vs):
            p[...], m[...], v[...] = O.adam_update(p, g, m, v, lr, step, beta1, beta2, eps)
