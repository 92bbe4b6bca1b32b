"""Training steps as sequences of C-ABI calls: the hand-unrolled tape of a define-by-run step.

The paper's training step (Sections "On Demand Graph Construction" and "Background and Motivation")
runs the forward computation operation by operation, then each recorded operation's backward once in
reverse order, then the optimiser.  The classes below issue exactly that sequence for the two model
families of the benchmark workloads.  All arithmetic happens inside libchn's kernels; Python only
decides which call comes next.  Buffers are allocated once (PyTorch is the allocator), and the
descriptor/argument list of every call is built once per input batch and replayed, so a step costs
one foreign call per kernel launch and can be captured into a HIP graph.

Linear layers follow the model-definition figure: W is (n_out, n_in), y = x @ W.T + b.
Mixed precision (``lowp=True``): fp32 master weights with bf16 working copies refreshed by the SGD
kernel; activations and activation gradients in bf16; logits, weight/bias gradients and the loss in
fp32; every product accumulates in fp32.
"""
import ctypes as C

import numpy as np
import torch

from . import binding as B


def _dev(a, lowp=False):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return B.cast(t, torch.bfloat16) if lowp else t


class _Program:
    """A recorded list of foreign calls; every libchn entry point takes the stream last."""

    def __init__(self):
        self.calls = []
        self._keep = []
        # one workspace shared by all GEMMs of the program (they run in stream order); sized when
        # the program is complete, which is why the calls hold mutable ctypes objects
        self.gemm_ws = C.c_void_p(0)
        self.gemm_ws_bytes = C.c_size_t(0)
        self._gemm_need = 0

    def finish(self):
        if self._gemm_need:
            t = torch.empty(self._gemm_need, dtype=torch.uint8, device="cuda")
            self._keep.append(t)
            self.gemm_ws.value = t.data_ptr()
            self.gemm_ws_bytes.value = self._gemm_need
        return self

    def d(self, t):
        if t is None:
            return None
        a = B.desc(t)
        self._keep.append((a, t))
        return C.byref(a)

    def ptrs(self, tensors):
        ds = [None if t is None else B.desc(t) for t in tensors]
        arr = B._ptrs(ds)
        self._keep.append((ds, arr, tensors))
        return arr

    def ws(self, t):
        return (None, 0) if t is None else (C.c_void_p(t.data_ptr()), t.numel() * t.element_size())

    def add(self, fn, *args):
        self.calls.append((fn, args))

    def run(self, stream=None):
        s = B._stream() if stream is None else stream
        for fn, args in self.calls:
            st = fn(*args, s)
            if st != 0:
                B._check(st)

    def replay(self):
        """Run the program as one HIP graph launch (captured on first use, after an eager run has
        configured every kernel).  The library enqueues kernels only -- no memsets, no allocations --
        so the captured graph is exactly the eager launch sequence."""
        if getattr(self, "_graph", None) is None:
            self.run()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                self.run()
            self._graph = g
        self._graph.replay()


def _gemm(p, L, A, Bm, Cm, alpha=1.0, beta=0.0, epi="none", bias=None, aux=None, pre=None):
    a, b, c = p.d(A), p.d(Bm), p.d(Cm)
    p._gemm_need = max(p._gemm_need, L.chn_gemm_workspace_bytes(a, b, c))
    p.add(L.chn_gemm, a, b, c, C.c_float(alpha), C.c_float(beta), B.EPI[epi],
          p.d(bias), p.d(aux), p.d(pre), p.gemm_ws, p.gemm_ws_bytes)


class MLPTrainer:
    """Forward + backward + SGD for an MLP with softmax cross-entropy (workloads 1, 3 and 5)."""

    def __init__(self, params, batch, act="relu", lr=0.01, lowp=False, fused_update=False, fused_loss=True):
        """fused_update: the weight-gradient product of every layer applies the SGD update in its
        epilogue (alpha = -lr, beta = 1 on the fp32 weights, bf16 working copy refreshed in the same
        pass), so weight gradients never travel through memory and `dW` stays unwritten; the input
        gradient of a layer, which needs the weights of the forward pass, is then computed first."""
        self.L = B.lib()
        self.act, self.lr, self.lowp, self.batch = act, float(lr), lowp, batch
        self.fused_update = fused_update
        self.fused_loss = fused_loss      # loss and its gradient in one call (else the two separate calls)
        self.W = [_dev(W) for W, _ in params]
        self.b = [_dev(b) for _, b in params]
        self.Wl = [B.cast(w, torch.bfloat16) for w in self.W] if lowp else self.W
        adt = torch.bfloat16 if lowp else torch.float32
        n = len(params)
        self.sizes = [params[0][0].shape[1]] + [W.shape[0] for W, _ in params]
        mk = lambda *s, dt=torch.float32: torch.empty(*s, dtype=dt, device="cuda")
        self.h = [None] + [mk(batch, self.sizes[l + 1], dt=adt) for l in range(n - 1)]
        self.z = [None] + [mk(batch, self.sizes[l + 1], dt=adt) if act == "gelu" else None for l in range(n - 1)]
        self.logits = mk(batch, self.sizes[-1])
        # gradient wrt layer l's output; rows padded to 16 bytes, so that a narrow one (the logits') is still
        # read in 16-byte pieces where it is the transposed operand of the weight-gradient product
        epr = 8 if lowp else 4
        self.dv = [None] + [mk(batch, (self.sizes[l + 1] + epr - 1) // epr * epr, dt=adt)[:, :self.sizes[l + 1]] for l in range(n)]
        self.dW = [mk(*w.shape) for w in self.W]
        self.db = [mk(*b.shape) for b in self.b]
        self.loss = mk(())
        self.lse = mk(batch)
        self.ws_ce = torch.empty(B.softmax_ce_workspace_bytes(batch), dtype=torch.uint8, device="cuda")
        need = max([B.reduce_axis_workspace_bytes(d, 0) for d in self.dv[1:]] + [256])
        self.ws_red = torch.empty(need, dtype=torch.uint8, device="cuda")
        # Where a hidden layer's output gradient comes out of an activation-gradient product in whole
        # 256 x 256 tiles, that product also leaves its column sums per block of 128 rows, and the
        # bias gradient is the sum of those few rows instead of another pass over the gradient.
        self.rowsums = {l: mk(batch // 128, self.sizes[l]) for l in range(1, n)
                        if batch % 256 == 0 and self.sizes[l] % 256 == 0 and self.sizes[l + 1] % 8 == 0}
        self._progs = {}

    def _build(self, x, t):
        L, p, n = self.L, _Program(), len(self.W)
        fwd_epi = "bias_relu" if self.act == "relu" else "bias_gelu"
        bwd_epi = "relu_bwd" if self.act == "relu" else "gelu_bwd"
        hs = [x] + self.h[1:]
        # forward
        for l in range(n):
            last = l == n - 1
            _gemm(p, L, hs[l], self.Wl[l].t(), self.logits if last else hs[l + 1],
                  epi="bias" if last else fwd_epi, bias=self.b[l],
                  pre=None if last or self.act == "relu" else self.z[l + 1])
        wp, wn = p.ws(self.ws_ce)
        # loss and its gradient in one call (the logits are read once; one launch for the small models)
        if self.fused_loss:
            p.add(L.chn_softmax_ce_fwd_bwd, p.d(self.logits), p.d(t), -1, p.d(self.loss), p.d(self.lse), C.c_float(1.0), p.d(self.dv[n]), wp, wn)
        else:
            p.add(L.chn_softmax_ce_fwd, p.d(self.logits), p.d(t), -1, p.d(self.loss), None, p.d(self.lse), wp, wn)
            p.add(L.chn_softmax_ce_bwd, p.d(self.logits), p.d(t), -1, p.d(self.lse), C.c_float(1.0), p.d(self.dv[n]), wp, wn)
        # backward, reverse order
        rp, rn = p.ws(self.ws_red)
        for l in range(n - 1, -1, -1):
            dv = self.dv[l + 1]
            if not self.fused_update:
                _gemm(p, L, dv.t(), hs[l], self.dW[l])
            p.add(L.chn_reduce_axis, B.REDUCE["sum"], p.d(self.rowsums.get(l + 1, dv)), 0, 0, p.d(self.db[l]), rp, rn)
            if l > 0:
                _gemm(p, L, dv, self.Wl[l], self.dv[l], epi=bwd_epi,
                      aux=hs[l] if self.act == "relu" else self.z[l], pre=self.rowsums.get(l))
            if self.fused_update:     # after dx: that product still reads this layer's old weights
                _gemm(p, L, dv.t(), hs[l], self.W[l], alpha=-self.lr, beta=1.0,
                      epi="bf16_copy" if self.lowp else "none", pre=self.Wl[l] if self.lowp else None)
        # optimiser: every parameter once (with fused_update only the biases are left)
        if self.fused_update:
            params, grads, lows = self.b, self.db, None
        else:
            params = self.W + self.b
            grads = self.dW + self.db
            lows = (self.Wl + [None] * n) if self.lowp else None
        p.add(L.chn_sgd_update_multi, len(params), p.ptrs(params), p.ptrs(grads), C.c_float(self.lr),
              None if lows is None else p.ptrs(lows))
        return p.finish()

    def step(self, x, t, stream=None, graph=False):
        key = (x.data_ptr(), t.data_ptr())
        if key not in self._progs:
            self._progs[key] = self._build(x, t)
        if graph:
            self._progs[key].replay()
        else:
            self._progs[key].run(stream)
        return self.loss

    def n_launch_calls(self, x, t):
        self.step(x, t)
        return len(self._progs[(x.data_ptr(), t.data_ptr())].calls)


def _ceil32(n):
    return (n + 31) // 32 * 32


class LSTMTrainer:
    """Forward + full BPTT + SGD for the single-layer LSTM language model (workload 4), fp32.

    Time-major layout: row t*B + b of every (T*B, .) buffer belongs to step t, batch element b.
    W (E,4H) and U (H,4H) give the gates as x W + h U + b; W_out (V,H) is a Linear layer.

    Layout in HBM: the embedding width E and the hidden width H are rounded up to multiples of 32 and
    every parameter is embedded in a zero-padded array of the rounded shape (gate blocks of W, U and b
    stay gate blocks, now of the rounded width).  The added embedding columns and hidden units are
    inert: their weights, biases, activations, cell states and every gradient that touches them are
    exactly zero from the first step on and stay zero under SGD, so the real entries take the values
    they would take unpadded, bit for bit (the padding only adds exact zeros to sums) -- but every row of
    every operand now starts on a 16-byte boundary and every contraction length is a whole number of
    tile steps, which is what the fast GEMM paths need (650 floats per row would allow 8-byte pieces
    only).  `P`, `g` and the activation buffers are exposed without the padding.

    Mixed precision (``lowp=True``): everything that feeds a matrix product is stored in bf16 -- working
    copies of E, W, U and W_out (refreshed by the SGD kernel), the embeddings, every h, the logit
    gradients, the gradients of h and of the gate pre-activations; gate pre-activations, activated
    gates, cell state and its gradient, logits, loss, parameter gradients and master weights stay fp32;
    every product accumulates in fp32.
    """

    def __init__(self, P, T, Bn, lr=0.01, lowp=False, fused_step=True, whole_sequence=None, whole_sequence_bwd=None):
        """whole_sequence: the T forward steps are ONE launch (chn_lstm_seq_fwd: the grid stays on the device,
        each workgroup keeps its rows of the recurrent matrix in LDS and the workgroups exchange h through
        device memory between steps).  None = wherever the library takes the shape (fused_step only).
        Measured on workload 4: 12.9 us instead of 14.3 us per step in fp32, 6.7 instead of 8.0 us in
        mixed precision.  In fp32 the T backward steps are one launch too (chn_lstm_seq_bwd: 14.4 us per
        step instead of the 41 us of product, partial-sum kernel and cell kernel); in mixed precision the
        per-step fused call (11.6 us) is as fast as the resident grid's exchange of partial sums (11.9 us)
        and stays.  `whole_sequence_bwd` overrides that choice.  The kernels' waits are bounded;
        `sequence_complete()` tells whether one ran out (then the step's results and the parameters it
        updated are invalid).

        fused_step: a time step is one launch (chn_lstm_step_fwd / _bwd: recurrent product and cell
        together) instead of product, partial-sum kernel and cell kernel; `Z` then holds the input part
        x W only, and the transposed recurrent matrix the forward reads is refreshed by one copy at the
        start of the step.  Measured on workload 4: the fused forward step wins in both precisions, the
        fused backward step (a four times longer contraction on a quarter of the tiles) only in mixed
        precision, so the fp32 backward keeps the three separate calls."""
        self.L = B.lib()
        self.T, self.B, self.lr, self.lowp, self.fused_step = T, Bn, float(lr), lowp, fused_step
        V, E = P["E"].shape
        H = P["U"].shape[0]
        self.V, self.E, self.H = V, E, H
        Ep, Hp = _ceil32(E), _ceil32(H)
        self.Ep, self.Hp = Ep, Hp
        z = lambda *s: torch.zeros(*s, dtype=torch.float32, device="cuda")
        self._P = {"E": z(V, Ep), "W": z(Ep, 4 * Hp), "U": z(Hp, 4 * Hp), "b": z(4 * Hp), "W_out": z(V, Hp), "b_out": z(V)}
        for k in self._P:
            dst = self._real(self._P, k)
            dst.copy_(_dev(P[k]).reshape(dst.shape))
        n = T * Bn
        adt = torch.bfloat16 if lowp else torch.float32
        za = lambda *s: torch.zeros(*s, dtype=adt, device="cuda")
        # working copies the products read: bf16 in mixed precision, else the parameters themselves
        self._Pl = {k: (B.cast(v, torch.bfloat16) if lowp and k in ("E", "W", "U", "W_out") else v) for k, v in self._P.items()}
        # zero-initialised: the inert columns must hold zeros before the first step
        self._X, self._Z, self._G = za(n, Ep), z(n, 4 * Hp), z(n, 4 * Hp)
        self._Hs = za(n + Bn, Hp)  # block 0 = h_0 = 0
        self._Cs = z(n + Bn, Hp)   # block 0 = c_0 = 0
        self.logits = z(n, V)
        self._dlogits = za(n, V) if lowp else self.logits      # fp32: the gradient overwrites the logits
        self._dHs, self._dZ, self._dX = za(n, Hp), za(n, 4 * Hp), z(n, Ep)
        self._dc = [z(Bn, Hp), z(Bn, Hp)]
        self._Ut = za(4 * Hp, Hp) if fused_step else None
        fits = fused_step and B.lstm_seq_supported(Bn, Hp, adt)
        if whole_sequence and not fits:
            raise ValueError("LSTMTrainer: the whole-sequence kernel does not take batch %d, hidden %d: %s" % (Bn, Hp, B.lib().chn_last_error().decode()))
        self.whole_sequence = fits if whole_sequence is None else bool(whole_sequence)
        self.ws_seq = torch.zeros(B.lstm_seq_workspace_bytes(Bn), dtype=torch.uint8, device="cuda") if self.whole_sequence else None
        fits = fused_step and B.lstm_seq_bwd_supported(Bn, Hp, adt)
        if whole_sequence_bwd and not fits:
            raise ValueError("LSTMTrainer: the whole-sequence backward kernel does not take batch %d, hidden %d: %s" % (Bn, Hp, B.lib().chn_last_error().decode()))
        self.whole_sequence_bwd = (fits and not lowp and self.whole_sequence) if whole_sequence_bwd is None else bool(whole_sequence_bwd)
        self.ws_seq_bwd = torch.zeros(B.lstm_seq_bwd_workspace_bytes(Bn, Hp), dtype=torch.uint8, device="cuda") if self.whole_sequence_bwd else None
        # fp32: the two backward products of the output layer read one operand along its strided
        # dimension, which for fp32 goes through registers instead of straight to LDS; a transposed
        # copy of that operand (10-12 us each) saves 50-60 us per product
        self._WoT = None if lowp else z(Hp, V)
        self._HallT = None if lowp else z(Hp, n)
        self._g = {k: z(*v.shape) for k, v in self._P.items()}
        self.loss, self.lse = z(()), z(n)
        self.ws_ce = torch.empty(B.softmax_ce_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        need = max(B.reduce_axis_workspace_bytes(self._dlogits, 0), B.reduce_axis_workspace_bytes(self._dZ, 0), 256)
        self.ws_red = torch.empty(need, dtype=torch.uint8, device="cuda")
        self._progs = {}

    # ---- views without the padding (for callers and tests; the step itself never uses them) ----------
    def _real(self, d, k):
        E, H, Hp = self.E, self.H, self.Hp
        t = d[k]
        if k == "E":
            return t[:, :E]
        if k == "W":
            return t.view(self.Ep, 4, Hp)[:E, :, :H]
        if k == "U":
            return t.view(Hp, 4, Hp)[:H, :, :H]
        if k == "b":
            return t.view(4, Hp)[:, :H]
        if k == "W_out":
            return t[:, :H]
        return t

    def _unpadded(self, d):
        shapes = {"W": (self.E, 4 * self.H), "U": (self.H, 4 * self.H), "b": (4 * self.H,)}
        return {k: self._real(d, k).reshape(shapes[k]) if k in shapes else self._real(d, k) for k in d}

    def _gates(self, t):
        return t.view(t.shape[0], 4, self.Hp)[:, :, :self.H].reshape(t.shape[0], 4 * self.H)

    P = property(lambda self: self._unpadded(self._P))
    g = property(lambda self: self._unpadded(self._g))
    X = property(lambda self: self._X[:, :self.E])
    dX = property(lambda self: self._dX[:, :self.E])
    Hs = property(lambda self: self._Hs[:, :self.H])
    Cs = property(lambda self: self._Cs[:, :self.H])
    dHs = property(lambda self: self._dHs[:, :self.H])
    dc = property(lambda self: [t[:, :self.H] for t in self._dc])
    Z = property(lambda self: self._gates(self._Z))
    G = property(lambda self: self._gates(self._G))
    dZ = property(lambda self: self._gates(self._dZ))

    def _build(self, ids, targets):
        L, p, P, Pl, T, Bn = self.L, _Program(), self._P, self._Pl, self.T, self.B
        blk = lambda buf, t: buf[t * Bn:(t + 1) * Bn]
        ids_f, tg_f = ids.reshape(-1), targets.reshape(-1)
        dlog = self._dlogits
        # forward
        p.add(L.chn_embed_fwd, p.d(Pl["E"]), p.d(ids_f), p.d(self._X))
        _gemm(p, L, self._X, Pl["W"], self._Z)                                  # x W for all steps at once
        if self.fused_step:
            p.add(L.chn_elementwise_broadcast, B.OP["copy"], 1, p.ptrs([Pl["U"].t()]), p.d(self._Ut), None, 0)
        if self.whole_sequence:                                                 # all T steps, one resident grid
            sp, sn = p.ws(self.ws_seq)
            p.add(L.chn_lstm_seq_fwd, p.d(self._Z), p.d(self._Ut), p.d(P["b"]), p.d(self._Hs), p.d(self._Cs), p.d(self._G), T, sp, sn)
        for t in range(0 if self.whole_sequence else T):
            if self.fused_step:                                                 # (x W)_t + h_{t-1} U, then the cell
                p.add(L.chn_lstm_step_fwd, p.d(blk(self._Z, t)), p.d(blk(self._Hs, t)), p.d(self._Ut), p.d(P["b"]),
                      p.d(blk(self._Cs, t)), p.d(blk(self._Cs, t + 1)), p.d(blk(self._Hs, t + 1)), p.d(blk(self._G, t)))
                continue
            _gemm(p, L, blk(self._Hs, t), Pl["U"], blk(self._Z, t), beta=1.0)   # + h_{t-1} U
            p.add(L.chn_lstm_fwd, p.d(blk(self._Z, t)), p.d(P["b"]), p.d(blk(self._Cs, t)),
                  p.d(blk(self._Cs, t + 1)), p.d(blk(self._Hs, t + 1)), p.d(blk(self._G, t)))
        Hall, Hprev = self._Hs[Bn:], self._Hs[:T * Bn]
        _gemm(p, L, Hall, Pl["W_out"].t(), self.logits, epi="bias", bias=P["b_out"])
        wp, wn = p.ws(self.ws_ce)
        # loss and gradient in one visit of every row (in fp32 the logit gradients overwrite the logits)
        p.add(L.chn_softmax_ce_fwd_bwd, p.d(self.logits), p.d(tg_f), -1, p.d(self.loss), p.d(self.lse), C.c_float(1.0), p.d(dlog), wp, wn)
        rp, rn = p.ws(self.ws_red)
        if self.lowp:
            _gemm(p, L, dlog.t(), Hall, self._g["W_out"])
        else:
            p.add(L.chn_elementwise_broadcast, B.OP["copy"], 1, p.ptrs([Hall.t()]), p.d(self._HallT), None, 0)
            _gemm(p, L, dlog.t(), self._HallT.t(), self._g["W_out"])
        p.add(L.chn_reduce_axis, B.REDUCE["sum"], p.d(dlog), 0, 0, p.d(self._g["b_out"]), rp, rn)
        if self.lowp:
            _gemm(p, L, dlog, Pl["W_out"], self._dHs)
        else:
            p.add(L.chn_elementwise_broadcast, B.OP["copy"], 1, p.ptrs([Pl["W_out"].t()]), p.d(self._WoT), None, 0)
            _gemm(p, L, dlog, self._WoT.t(), self._dHs)
        if self.whole_sequence_bwd:                                             # all T steps, one resident grid
            sp, sn = p.ws(self.ws_seq_bwd)
            p.add(L.chn_lstm_seq_bwd, p.d(Pl["U"]), p.d(self._dHs), p.d(self._G), p.d(self._Cs), None, p.d(self._dZ), p.d(self._dc[0]), T, sp, sn)
        for t in range(-1 if self.whole_sequence_bwd else T - 1, -1, -1):
            dc_next = None if t == T - 1 else self._dc[(t + 1) & 1]
            if self.fused_step and self.lowp:                     # dh_t += dz_{t+1} U^T, then the cell backward
                dz_next = None if t == T - 1 else blk(self._dZ, t + 1)
                p.add(L.chn_lstm_step_bwd, p.d(dz_next), p.d(Pl["U"]), p.d(blk(self._dHs, t)), p.d(blk(self._G, t)),
                      p.d(blk(self._Cs, t)), p.d(blk(self._Cs, t + 1)), p.d(dc_next), p.d(blk(self._dZ, t)), p.d(self._dc[t & 1]))
                continue
            p.add(L.chn_lstm_bwd, p.d(blk(self._G, t)), p.d(blk(self._Cs, t)), p.d(blk(self._Cs, t + 1)),
                  p.d(blk(self._dHs, t)), p.d(dc_next), p.d(blk(self._dZ, t)), p.d(self._dc[t & 1]))
            if t > 0:
                _gemm(p, L, blk(self._dZ, t), Pl["U"].t(), blk(self._dHs, t - 1), beta=1.0)
        _gemm(p, L, Hprev.t(), self._dZ, self._g["U"])
        _gemm(p, L, self._X.t(), self._dZ, self._g["W"])
        p.add(L.chn_reduce_axis, B.REDUCE["sum"], p.d(self._dZ), 0, 0, p.d(self._g["b"]), rp, rn)
        _gemm(p, L, self._dZ, Pl["W"].t(), self._dX)
        p.add(L.chn_embed_bwd, p.d(ids_f), p.d(self._dX), p.d(self._g["E"]), 0)
        names = list(P.keys())
        lows = p.ptrs([Pl[k] if Pl[k] is not P[k] else None for k in names]) if self.lowp else None
        p.add(L.chn_sgd_update_multi, len(names), p.ptrs([P[k] for k in names]),
              p.ptrs([self._g[k] for k in names]), C.c_float(self.lr), lows)
        return p.finish()

    def step(self, ids, targets, stream=None, graph=False):
        key = (ids.data_ptr(), targets.data_ptr())
        if key not in self._progs:
            self._progs[key] = self._build(ids, targets)
        if graph:
            self._progs[key].replay()
        else:
            self._progs[key].run(stream)
        return self.loss

    def sequence_complete(self):
        """Synchronises; False if a bounded wait of the whole-sequence kernel ran out in the last step."""
        return all(w is None or B.lstm_seq_status(w) == 0 for w in (self.ws_seq, self.ws_seq_bwd))

    def n_launch_calls(self, ids, targets):
        self.step(ids, targets)
        return len(self._progs[(ids.data_ptr(), targets.data_ptr())].calls)
