"""Define-by-run tape: the backtracking graph is recorded while the forward code runs.

Section "On Demand Graph Construction": every differentiable operation applied to variables records
a *function node* that references the *variable nodes* of its inputs; each output's variable node
references the function node that made it.  The graph says nothing about the forward computation
(plain Python does that, so control flow may change from one iteration to the next); it only tells
``backward`` how to walk back: function nodes are visited once each in reverse topological order.

Memory (Sections "Global Memory Usage Reduction" and "Function-wise Local Memory Usage Reduction"):

* the user-facing :class:`Variable` owns its array; the :class:`VariableNode` in the graph refers to
  the array only while some function has declared that its backward needs it (``retain_inputs`` /
  ``retain_outputs``).  A function that can differentiate from its outputs (ReLU, the LSTM cell)
  retains those and lets its inputs go; one that needs nothing (addition) retains nothing;
* ``backward`` cuts every function node out of the graph right after calling its backward, so plain
  reference counting returns the buffers of everything behind it at once -- no collector pass;
* gradients of intermediate variables are dropped as soon as they have been consumed.

All arithmetic happens in the library behind the C ABI: each function's forward and backward is a
handful of calls on a *backend* object whose methods carry the names of the entry points
(``gemm``, ``elementwise_broadcast``, ``reduce_axis``, ``lstm_fwd`` ...).  :class:`GpuBackend` routes
them to the binding (PyTorch is the allocator, nothing more) and refuses to work without the built
library.  Host-logic tests drive the same tape with a backend of their own.
"""
import heapq
import itertools
import weakref

__all__ = ["Variable", "Parameter", "VariableNode", "FunctionNode", "GpuBackend", "using_backend",
           "no_backprop_mode", "linear", "matmul", "relu", "gelu", "add", "softmax_cross_entropy",
           "embed_id", "lstm", "split_rows", "concat_rows", "Linear", "SGD", "Adam", "live_function_nodes",
           "grad", "mul", "sub", "scale", "tanh", "sum_all", "sum_rows", "broadcast_to", "broadcast_rows", "transpose",
           "relu_grad", "user_elementwise",
           "MLP", "LSTMLanguageModel"]


# ---- backend ----------------------------------------------------------------------------------------
class GpuBackend:
    """Routes the tape's kernel calls to libchn through the binding; arrays are CUDA tensors."""

    def __init__(self):
        import torch
        from . import binding
        binding.lib()                       # fails loudly when the library has not been built
        self.torch, self.B = torch, binding
        self._dt = {"f32": torch.float32, "bf16": torch.bfloat16, "i64": torch.int64, "i32": torch.int32}
        self._name = {v: k for k, v in self._dt.items()}
        self._gemm_ws = None
        self._seq_ws = []          # workspaces of whole-sequence recurrent launches whose status word is unread
        self._dev = torch.device("cuda", torch.cuda.current_device())

    # allocation (PyTorch's caching allocator; freed by reference count, reused in stream order)
    def empty(self, shape, dtype="f32"):
        return self.torch.empty(tuple(shape), dtype=self._dt[dtype], device=self._dev)

    def dtype(self, a):
        return self._name[a.dtype]

    def from_numpy(self, a, dtype=None):
        import numpy as np
        t = self.torch.from_numpy(np.ascontiguousarray(a)).cuda()
        return t if dtype is None else self.B.cast(t, self._dt[dtype])

    def to_numpy(self, a):
        if self._seq_ws:
            self.check_sequences()
        return a.detach().to(self.torch.float64 if a.is_floating_point() else a.dtype).cpu().numpy()

    def _bytes(self, n):
        return None if n == 0 else self.torch.empty(n, dtype=self.torch.uint8, device="cuda")

    # kernels: same names and argument order as the binding
    def gemm(self, A, Bm, Cm, alpha=1.0, beta=0.0, epilogue="none", bias=None, aux=None, preact_out=None):
        A, Bm, Cm = self.B.desc(A), self.B.desc(Bm), self.B.desc(Cm)     # marshalled once for both calls
        need = self.B.gemm_workspace_bytes(A, Bm, Cm)
        if need and (self._gemm_ws is None or self._gemm_ws.numel() < need):
            self._gemm_ws = self._bytes(need)   # the old one stays valid for launches already queued
        return self.B.gemm(A, Bm, Cm, alpha, beta, epilogue, bias, aux, preact_out,
                           ws=self._gemm_ws if need else None)

    def elementwise_broadcast(self, op, inputs, out, scalars=()):
        return self.B.elementwise_broadcast(op, inputs, out, scalars)

    def reduce_axis(self, op, x, axis, out):
        return self.B.reduce_axis(op, x, axis, out, ws=self._bytes(self.B.reduce_axis_workspace_bytes(x, axis)))

    def lstm_fwd(self, z, bias, c_prev, c, h, gates):
        self.B.lstm_fwd(z, bias, c_prev, c, h, gates)

    def lstm_bwd(self, gates, c_prev, c, dh, dc_next, dz, dc_prev):
        self.B.lstm_bwd(gates, c_prev, c, dh, dc_next, dz, dc_prev)

    def fuses_lstm_step(self, hidden):
        """Whether lstm_step_fwd (recurrent product and cell in one launch) takes this hidden width."""
        return hidden % 32 == 0

    def lstm_step_fwd(self, zx, h_prev, Ut, bias, c_prev, c, h, gates):
        self.B.lstm_step_fwd(zx, h_prev, Ut, bias, c_prev, c, h, gates)

    def lstm_step_bwd(self, dz_next, U, dh, gates, c_prev, c, dc_next, dz, dc_prev):
        self.B.lstm_step_bwd(dz_next, U, dh, gates, c_prev, c, dc_next, dz, dc_prev)

    # A whole sequence of fused steps over time-major buffers: one launch for all steps where the library's
    # resident-grid kernels take the shape (forward: both precisions; backward: fp32, in mixed precision the
    # per-step call is as fast), else one launch per step (the marshalling is done once).  The resident
    # kernels' waits are bounded; whether one ran out shows in a status word that `check_sequences` reads.
    def lstm_steps_fwd(self, zx, Hs, Ut, bias, Cs, gates, n_steps):
        Bn = zx.shape[0] // max(1, n_steps)
        if n_steps > 0 and self.B.lstm_seq_supported(Bn, Hs.shape[1], Hs.dtype):
            ws = self._bytes(self.B.lstm_seq_workspace_bytes(Bn))
            self.B.lstm_seq_fwd(zx, Ut, bias, Hs, Cs, gates, n_steps, ws)
            self._pending(ws)
        else:
            self.B.lstm_step_fwd_seq(zx, Hs, Ut, bias, Cs, gates, n_steps)

    def lstm_steps_bwd(self, dZ, U, dHs, gates, Cs, dc_last, dc, n_steps):
        Bn = dZ.shape[0] // max(1, n_steps)
        if n_steps > 0 and dHs.dtype == self.torch.float32 and self.B.lstm_seq_bwd_supported(Bn, dHs.shape[1], dHs.dtype):
            ws = self._bytes(self.B.lstm_seq_bwd_workspace_bytes(Bn, dHs.shape[1]))
            self.B.lstm_seq_bwd(U, dHs, gates, Cs, dc_last, dZ, dc[0], n_steps, ws)
            self._pending(ws)
        else:
            self.B.lstm_step_bwd_seq(dZ, U, dHs, gates, Cs, dc_last, dc, n_steps)

    def _pending(self, ws):
        self._seq_ws.append(ws)
        if len(self._seq_ws) >= 256:
            self.check_sequences()

    def check_sequences(self):
        """Synchronises and raises if a wait of a whole-sequence recurrent kernel ran out since the last check
        (its outputs, and whatever was computed from them, are then invalid)."""
        pending, self._seq_ws = self._seq_ws, []
        if any(self.B.lstm_seq_status(w) != 0 for w in pending):
            raise RuntimeError("a whole-sequence recurrent kernel gave up waiting for its grid (the device was shared); "
                               "results since the last check are invalid")

    def softmax_ce_fwd(self, logits, labels, loss_mean, lse, ignore_label):
        ws = self._bytes(self.B.softmax_ce_workspace_bytes(logits.shape[0]))
        self.B.softmax_ce_fwd(logits, labels, loss_mean, None, lse, ignore_label, ws)

    def softmax_ce_bwd(self, logits, labels, dlogits, lse, upstream, ignore_label):
        ws = self._bytes(self.B.softmax_ce_workspace_bytes(logits.shape[0]))
        self.B.softmax_ce_bwd(logits, labels, dlogits, lse, upstream, ignore_label, ws)

    def softmax_ce_bwd2(self, logits, labels, gg, dlogits, dupstream, lse, upstream, ignore_label):
        ws = self._bytes(self.B.softmax_ce_workspace_bytes(logits.shape[0]))
        self.B.softmax_ce_bwd2(logits, labels, gg, dlogits, dupstream, lse, upstream, ignore_label, ws)

    def embed_fwd(self, table, ids, out):
        self.B.embed_fwd(table, ids, out)

    def embed_bwd(self, ids, dout, dtable, accumulate):
        self.B.embed_bwd(ids, dout, dtable, accumulate)

    def sgd_update_multi(self, params, grads, lr, lowp_copies):
        self.B.sgd_update_multi(params, grads, lr, lowp_copies)

    def adam_update_multi(self, params, grads, ms, vs, lr, step, beta1, beta2, eps, lowp_copies):
        self.B.adam_update_multi(params, grads, ms, vs, lr, step, beta1, beta2, eps, lowp_copies)


_backend = None


def backend():
    global _backend
    if _backend is None:
        _backend = GpuBackend()
    return _backend


class using_backend:
    """``with using_backend(b):`` -- run the tape on another backend (tests of the host logic)."""

    def __init__(self, b):
        self.b = b

    def __enter__(self):
        global _backend
        self.prev, _backend = _backend, self.b
        return self.b

    def __exit__(self, *exc):
        global _backend
        _backend = self.prev


_record = True


class no_backprop_mode:
    """Inside the block no function node is recorded (pure forward evaluation)."""

    def __enter__(self):
        global _record
        self.prev, _record = _record, False

    def __exit__(self, *exc):
        global _record
        _record = self.prev


# ---- graph objects ----------------------------------------------------------------------------------
class VariableNode:
    """A variable's place in the backtracking graph.

    Holds the creator function node, the topological rank, and -- only while a function has asked
    for it -- the array (Section "Function-wise Local Memory Usage Reduction").  `grad` is a slot
    used while a backward pass is running; when the pass ends the gradient moves to the user's
    :class:`Variable` (Section "Interface to Access the Resulting Gradients": the reference from a
    variable to its gradient is not part of the graph; kept on the node it would close a cycle
    through the graph of a differentiable backward pass).  The node knows its variable weakly.
    """
    __slots__ = ("creator", "rank", "requires_grad", "data", "grad", "_grad_owned", "_retainers", "name",
                 "_variable", "__weakref__")

    def __init__(self, requires_grad, name=None):
        self._variable = None
        self.creator = None
        self.rank = 0
        self.requires_grad = requires_grad
        self.data = None
        self.grad = None
        self._grad_owned = False
        self._retainers = 0
        self.name = name

    def _retain(self, array):
        self.data = array
        self._retainers += 1

    def _release(self):
        self._retainers -= 1
        if self._retainers <= 0:
            self._retainers = 0
            self.data = None


class Variable:
    """User handle: owns the array, points at its node (Section "Global Memory Usage Reduction":
    the array of an intermediate result is returned as soon as the handle is dropped unless a
    function retained it)."""

    def __init__(self, array, requires_grad=True, name=None):
        self.array = array
        self.node = VariableNode(requires_grad, name)
        self.node._variable = weakref.ref(self)
        self._grad, self._grad_owned, self.grad_var = None, False, None

    @classmethod
    def _of(cls, node, array):
        """Another handle on an existing node (what a function's backward sees of a retained value)."""
        v = cls.__new__(cls)
        v.array, v.node = array, node
        v._grad, v._grad_owned, v.grad_var = None, False, None
        return v

    shape = property(lambda self: self.array.shape)
    creator = property(lambda self: self.node.creator)
    requires_grad = property(lambda self: self.node.requires_grad)

    @property
    def grad(self):
        """The gradient array of the last backward pass(es); `grad_var` is the same gradient as a
        variable with its own history after ``backward(enable_double_backprop=True)``."""
        return self._grad

    @grad.setter
    def grad(self, g):
        self._grad, self._grad_owned, self.grad_var = g, False, None

    def cleargrad(self):
        self.grad = None

    def unchain(self):
        """Forget how this variable was computed (truncates back-propagation here)."""
        self.node.creator = None
        self.node.rank = 0

    def backward(self, retain_grad=False, enable_double_backprop=False):
        """Gradients of this variable with respect to everything it was computed from, stored in
        the `grad` of each variable.  With `enable_double_backprop` the backward computation is
        itself recorded (Section "Double Backpropagation"): the graph is kept, `grad_var` carries
        the history, and what was computed from the gradients can be differentiated again."""
        if enable_double_backprop:
            _backward_vars([self], [None if self._grad is None else Variable(self._grad, False)], None, True, retain_grad)
        else:
            _backward(self, retain_grad)


class Parameter(Variable):
    """A leaf variable that persists across iterations: fp32 master array, optionally a bf16
    working copy (``lowp``) that the optimiser refreshes and that products read instead."""

    def __init__(self, array, lowp=None, name=None):
        super().__init__(array, True, name)
        self.lowp = lowp

    @property
    def compute_array(self):
        return self.array if self.lowp is None else self.lowp


_live = weakref.WeakSet()


def live_function_nodes():
    """Number of function nodes still chained into some graph (0 after a full backward)."""
    return sum(1 for f in _live if f.inputs is not None)


class FunctionNode:
    """One applied operation.  Subclasses give ``forward(xs) -> tuple of arrays`` and
    ``backward(indexes, gys) -> tuple of arrays or None, one per index``; inside ``forward`` they
    declare what backward will need with ``retain_inputs`` / ``retain_outputs`` -- everything else
    is let go when the forward returns.

    ``fresh``: positions of inputs whose gradient, as returned by ``backward``, is always a newly
    allocated array nobody else refers to (the tape may then accumulate into it in place).
    """
    fresh = ()

    def __init__(self):
        self.inputs = None            # tuple of VariableNode (strong references)
        self.outputs = None           # tuple of weak references to VariableNode
        self.rank = 0
        self._retain_in = ()
        self._retain_out = ()
        self._out_data = None

    # -- declarations made inside forward
    def retain_inputs(self, indexes):
        self._retain_in = tuple(indexes)

    def retain_outputs(self, indexes):
        self._retain_out = tuple(indexes)

    # -- what backward may look at
    def get_retained_inputs(self):
        return tuple(self.inputs[i].data for i in self._retain_in)

    def get_retained_outputs(self):
        return self._out_data

    def get_retained_input_vars(self):
        return tuple(Variable._of(self.inputs[i], self.inputs[i].data) for i in self._retain_in)

    def get_retained_output_vars(self):
        """Retained outputs as variables for a differentiable backward.  The function knows its
        outputs only weakly (a strong reference would close a cycle), so an output node may be gone
        by now: then nobody else refers to it, and a fresh node is connected in its place around the
        array kept as a backup (Section "Output Retention for Double Backpropagation")."""
        outs = []
        for k, i in enumerate(self._retain_out):
            node = self.outputs[i]()
            if node is None:
                node = VariableNode(True)
                node.creator, node.rank = self, self.rank + 1
                refs = list(self.outputs)
                refs[i] = weakref.ref(node)
                self.outputs = tuple(refs)
            outs.append(Variable._of(node, self._out_data[k]))
        return tuple(outs)

    def apply(self, inputs):
        """Run forward on the inputs' arrays, wrap the results, and record this node if any
        input takes part in back-propagation."""
        inputs = tuple(x if isinstance(x, Variable) else Variable(x, requires_grad=False) for x in inputs)
        self.in_vars = inputs                # compute_array lookups inside forward; dropped below
        outs = self.forward(tuple(x.array for x in inputs))
        self.in_vars = None
        record = _record and any(x.node.requires_grad for x in inputs)
        ys = tuple(Variable(a, requires_grad=record) for a in outs)
        if record:
            self.inputs = tuple(x.node for x in inputs)
            self.rank = max(n.rank for n in self.inputs)
            for y in ys:
                y.node.creator = self
                y.node.rank = self.rank + 1
            self.outputs = tuple(weakref.ref(y.node) for y in ys)
            for i in self._retain_in:
                inputs[i].node._retain(self._input_array(inputs[i]))
            self._out_data = tuple(outs[i] for i in self._retain_out)
            _live.add(self)
        else:
            self._retain_in, self._retain_out = (), ()
            self.release_locals()
        return ys

    def _input_array(self, var):
        return var.array

    def release_locals(self):
        """Drop arrays the subclass stashed for its backward (called when the node is cut out)."""

    def unchain(self):
        """Cut this node out of the graph: outputs forget their creator, inputs lose the reference
        that kept them alive, retained arrays are let go."""
        if self.inputs is None:
            return
        for ref in self.outputs:
            n = ref()
            if n is not None and n.creator is self:
                n.creator = None
        for i in self._retain_in:
            self.inputs[i]._release()
        self.inputs = None
        self.outputs = None
        self._out_data = None
        self.release_locals()

    def forward(self, xs):
        raise NotImplementedError

    # A function gives `backward` (arrays in, arrays out: kernels called directly), or
    # `backward_vars` (variables in, variables out, written with differentiable functions: Section
    # "Double Backpropagation"), or both; each default is derived from the other.
    def backward(self, indexes, gys):
        if type(self).backward_vars is FunctionNode.backward_vars:
            raise NotImplementedError
        with no_backprop_mode():
            gxs = self.backward_vars(indexes, tuple(None if g is None else Variable(g, False) for g in gys))
        return tuple(None if g is None else g.array for g in gxs)

    def backward_vars(self, indexes, gys):
        if type(self).backward is FunctionNode.backward:
            raise NotImplementedError
        if _record:
            raise NotImplementedError("%s has no differentiable backward: double backprop cannot pass through it"
                                      % type(self).__name__)
        self.grad_slots, self.unit_seed = (None,) * len(indexes), False
        gxs = self.backward(indexes, tuple(None if g is None else g.array for g in gys))
        self.grad_slots = None
        return tuple(None if g is None else Variable(g, False) for g in gxs)


def _settle(nodes):
    """End of a backward pass: gradients move from the nodes' slots to the users' variables."""
    for n in nodes:
        v = None if n._variable is None else n._variable()
        if v is not None and n.grad is not None:
            v._grad, v._grad_owned, v.grad_var = n.grad, n._grad_owned, None
        n.grad, n._grad_owned = None, False


def _accumulate(node, g, fresh):
    """node.grad += g; in place only into an array the tape itself owns."""
    if node.grad is None:
        node.grad, node._grad_owned = g, fresh
        return
    F = backend()
    if node._grad_owned:
        F.elementwise_broadcast("add", [node.grad, g], node.grad)
    elif fresh:
        F.elementwise_broadcast("add", [g, node.grad], g)
        node.grad, node._grad_owned = g, True
    else:
        out = F.empty(g.shape, F.dtype(g))
        F.elementwise_broadcast("add", [node.grad, g], out)
        node.grad, node._grad_owned = out, True


def _backward(root, retain_grad):
    """Backtrack from `root` (Section "On Demand Graph Construction"): function nodes in order of
    decreasing rank, each exactly once; each is cut out of the graph as soon as it has run
    (Section "Global Memory Usage Reduction"), and gradients of intermediate variables are dropped
    once consumed unless `retain_grad`."""
    F = backend()
    rn = root.node
    touched = {}                          # every node whose slot this pass uses, by identity

    def touch(n):
        if id(n) not in touched:
            touched[id(n)] = n
            v = None if n._variable is None else n._variable()
            if v is not None and v._grad is not None:      # gradients accumulate until cleared
                n.grad, n._grad_owned = v._grad, v._grad_owned
        return n

    touch(rn)
    if rn.grad is None:
        n = 1
        for s in root.shape:
            n *= s
        if n != 1:
            raise ValueError("backward() from a non-scalar needs its .grad set first")
        one = F.empty(root.shape, F.dtype(root.array))
        F.elementwise_broadcast("fill", [], one, (1.0,))
        rn.grad, rn._grad_owned = one, True
        rn_unit = True
    else:
        rn_unit = False
    if rn.creator is None:
        _settle(touched.values())
        return
    tie = itertools.count()
    heap, waiting = [], {}

    def push(node):
        # the entry holds the node: once its consumers are cut out nothing else would keep an
        # intermediate result's node -- and the gradient stored on it -- alive
        f = node.creator
        held = waiting.get(id(f))
        if held is None:
            waiting[id(f)] = [node]
            heapq.heappush(heap, (-f.rank, next(tie), f))
        else:
            held.append(node)

    push(rn)
    while heap:
        _, _, f = heapq.heappop(heap)
        held = waiting[id(f)]            # stays registered while f runs: f is visited once
        outs = [ref() for ref in f.outputs]
        gys = tuple(None if o is None else o.grad for o in outs)
        f.unit_seed = rn_unit and len(outs) == 1 and outs[0] is rn
        if not retain_grad:
            for o in outs:
                if o is not None and o is not rn:
                    o.grad, o._grad_owned = None, False
        indexes = tuple(i for i, n in enumerate(f.inputs) if n.requires_grad)
        for i in indexes:
            touch(f.inputs[i])
        # slots a function may accumulate into directly (a product can add into its output)
        slots = f.grad_slots = tuple(f.inputs[i].grad if f.inputs[i]._grad_owned else None for i in indexes)
        gxs = f.backward(indexes, gys)
        f.grad_slots = None
        if len(gxs) != len(indexes):
            raise RuntimeError("%s.backward returned %d gradients for %d inputs"
                               % (type(f).__name__, len(gxs), len(indexes)))
        for i, gx, slot in zip(indexes, gxs, slots):
            if gx is None:
                continue
            n = f.inputs[i]
            if slot is None or gx is not slot:      # else: the function added into the slot itself
                _accumulate(n, gx, i in f.fresh)
            if n.creator is not None:
                push(n)
        del gys, gxs, outs, held
        waiting[id(f)] = None
        f.unchain()
    _settle(touched.values())


def _backward_vars(roots, seeds, targets, store, retain_grad=False):
    """The same walk with gradients that are variables and backward computations that are function
    applications (Section "Double Backpropagation").  Whether those applications are recorded is
    the caller's business (`no_backprop_mode`).  Nothing is cut out of the graph: the gradients'
    own history refers to it.  Returns {id(node): gradient variable} for the nodes in `targets`
    (all leaves when None); with `store` the gradients also go to the users' variables."""
    F = backend()
    gvars, keep = {}, {}
    for r, seed in zip(roots, seeds):
        if seed is None:
            n = 1
            for d in r.shape:
                n *= d
            if n != 1:
                raise ValueError("a non-scalar output needs a gradient to start from")
            one = F.empty(r.shape, F.dtype(r.array))
            F.elementwise_broadcast("fill", [], one, (1.0,))
            seed = Variable(one, False)
        gvars[id(r.node)] = seed
        keep[id(r.node)] = r.node
    want = None if targets is None else {id(t.node) for t in targets}
    result = {}
    tie = itertools.count()
    heap, queued = [], set()

    def push(node):
        f = node.creator
        if f is not None and id(f) not in queued:
            queued.add(id(f))
            heapq.heappush(heap, (-f.rank, next(tie), f))

    for r in roots:
        push(r.node)
    while heap:
        _, _, f = heapq.heappop(heap)
        outs = [ref() for ref in f.outputs]
        gys = []
        for o in outs:
            g = None if o is None else gvars.get(id(o))
            gys.append(g)
            if g is not None and ((want is not None and id(o) in want) or retain_grad):
                result[id(o)] = g
            if o is not None and not any(o is r.node for r in roots):
                gvars.pop(id(o), None)
        indexes = tuple(i for i, n in enumerate(f.inputs) if n.requires_grad)
        gxs = f.backward_vars(indexes, tuple(gys))
        if len(gxs) != len(indexes):
            raise RuntimeError("%s.backward_vars returned %d gradients for %d inputs" % (type(f).__name__, len(gxs), len(indexes)))
        for i, gx in zip(indexes, gxs):
            if gx is None:
                continue
            n = f.inputs[i]
            keep[id(n)] = n
            old = gvars.get(id(n))
            gvars[id(n)] = gx if old is None else add(old, gx)
            push(n)
    for k, g in gvars.items():            # what is left belongs to leaves (and the roots)
        if want is None or k in want:
            result[k] = g
    if store:
        for k, g in result.items():
            n = keep[k]
            v = None if n._variable is None else n._variable()
            if v is None:
                continue
            if v._grad is not None and not any(n is r.node for r in roots):   # accumulate until cleared
                base = v.grad_var if v.grad_var is not None else Variable(v._grad, False)
                g = add(base, g)
            v._grad, v._grad_owned, v.grad_var = g.array, False, g
    return result


def grad(outputs, inputs, grad_outputs=None, enable_double_backprop=False):
    """Gradients of `outputs` with respect to `inputs`, returned (one variable or None per input)
    instead of stored: the interface that adds no reference between the objects involved (Section
    "Interface to Access the Resulting Gradients").  With `enable_double_backprop` the returned
    variables carry the history of the backward computation."""
    seeds = list(grad_outputs) if grad_outputs is not None else [None] * len(outputs)
    seeds = [s if (s is None or isinstance(s, Variable)) else Variable(s, False) for s in seeds]
    if enable_double_backprop:
        res = _backward_vars(list(outputs), seeds, list(inputs), False)
    else:
        with no_backprop_mode():
            res = _backward_vars(list(outputs), seeds, list(inputs), False)
    return [res.get(id(x.node)) for x in inputs]


# ---- functions ----------------------------------------------------------------------------------------
def _t(a):
    return a.T


class LinearFunction(FunctionNode):
    """y = act(x @ W.T + b), W of shape (n_out, n_in) as in the model-definition figure (Section
    "API Design"); bias and activation run in the product's epilogue.  Retains x and W; ReLU is
    differentiated from the retained *output*, GELU from the pre-activation the epilogue stores."""
    fresh = (0, 1, 2)

    def __init__(self, act=None, out_dtype=None):
        super().__init__()
        self.act, self.out_dtype, self.z = act, out_dtype, None

    def _input_array(self, var):
        return var.compute_array if isinstance(var, Parameter) else var.array

    def forward(self, xs):
        F = backend()
        x, _, b = xs
        W = self._input_array(self.in_vars[1])
        dt = self.out_dtype or F.dtype(x)
        y = F.empty((x.shape[0], W.shape[0]), dt)
        if self.act == "gelu":
            self.z = F.empty(y.shape, dt)
        epi = {None: "bias", "relu": "bias_relu", "gelu": "bias_gelu"}[self.act]
        F.gemm(x, _t(W), y, epilogue=epi, bias=b, preact_out=self.z)
        self.retain_inputs((0, 1, 2) if self.act == "gelu" else (0, 1))   # (the bias: a differentiable backward rebuilds z)
        if self.act == "relu":
            self.retain_outputs((0,))
        return (y,)

    def release_locals(self):
        self.z = None

    def backward(self, indexes, gys):
        F = backend()
        x, W = self.get_retained_inputs()[:2]
        gy, = gys
        if self.act is not None:
            ref = self.get_retained_outputs()[0] if self.act == "relu" else self.z
            gz = F.empty(gy.shape, F.dtype(gy))
            F.elementwise_broadcast(self.act + "_bwd", [gy, ref], gz)
            gy = gz
        out = []
        for k, i in enumerate(indexes):
            if i == 0:
                gx = F.empty(x.shape, F.dtype(x))
                F.gemm(gy, W, gx)
            elif i == 1:
                gx = self.grad_slots[k]
                if gx is None:
                    gx = F.empty(W.shape, "f32")
                    F.gemm(_t(gy), x, gx)
                else:
                    F.gemm(_t(gy), x, gx, beta=1.0)
            else:
                gx = F.empty((gy.shape[1],), "f32")
                F.reduce_axis("sum", gy, 0, gx)
            out.append(gx)
        return tuple(out)


    def backward_vars(self, indexes, gys):
        x, W = self.get_retained_input_vars()[:2]
        if self.act == "gelu":
            # the pre-activation the epilogue stored is an array without history: as a function of x, W and
            # b it is computed once more, by a recorded linear function
            z = linear(x, W, self.get_retained_input_vars()[2])
            gz = gelu_grad(gys[0], z)
        else:
            gz = gys[0] if self.act is None else relu_grad(gys[0], self.get_retained_output_vars()[0])
        grads = {0: lambda: matmul(gz, W), 1: lambda: matmul(transpose(gz), x), 2: lambda: sum_rows(gz)}
        return tuple(grads[i]() for i in indexes)


class MatMul(FunctionNode):
    """y = x @ W (both 2-d); retains both inputs.  ``out_dtype`` / ``gx_dtype``: storage type of the
    result and of the gradient with respect to x (default: x's)."""
    fresh = (0, 1)

    def __init__(self, out_dtype=None, gx_dtype=None):
        super().__init__()
        self.out_dtype, self.gx_dtype = out_dtype, gx_dtype

    def _input_array(self, var):
        return var.compute_array if isinstance(var, Parameter) else var.array

    def forward(self, xs):
        F = backend()
        x = xs[0]
        W = self._input_array(self.in_vars[1])
        y = F.empty((x.shape[0], W.shape[1]), self.out_dtype or F.dtype(x))
        F.gemm(x, W, y)
        self.retain_inputs((0, 1))
        return (y,)

    def backward(self, indexes, gys):
        F = backend()
        x, W = self.get_retained_inputs()
        gy, = gys
        out = []
        for k, i in enumerate(indexes):
            if i == 0:
                gx = F.empty(x.shape, self.gx_dtype or F.dtype(x))
                F.gemm(gy, _t(W), gx)
            else:
                gx = self.grad_slots[k]
                if gx is None:
                    gx = F.empty(W.shape, "f32")
                    F.gemm(_t(x), gy, gx)
                else:
                    F.gemm(_t(x), gy, gx, beta=1.0)
            out.append(gx)
        return tuple(out)


    def backward_vars(self, indexes, gys):
        x, W = self.get_retained_input_vars()
        grads = {0: lambda: matmul(gys[0], transpose(W)), 1: lambda: matmul(transpose(x), gys[0])}
        return tuple(grads[i]() for i in indexes)


class _Activation(FunctionNode):
    fresh = (0,)
    op = None

    def backward(self, indexes, gys):
        F = backend()
        ref = self.saved()
        gx = F.empty(ref.shape, F.dtype(gys[0]))
        F.elementwise_broadcast(self.op + "_bwd", [gys[0], ref], gx)
        return (gx,)


class ReLU(_Activation):
    """Differentiated from its output: the input is not retained (Section "Function-wise Local
    Memory Usage Reduction")."""
    op = "relu"

    def forward(self, xs):
        F = backend()
        y = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("relu", [xs[0]], y)
        self.retain_outputs((0,))
        return (y,)

    def saved(self):
        return self.get_retained_outputs()[0]

    def backward_vars(self, indexes, gys):
        return (relu_grad(gys[0], self.get_retained_output_vars()[0]),)


class GELU(_Activation):
    """x * Phi(x); its derivative needs the input, so that is what it retains."""
    op = "gelu"

    def forward(self, xs):
        F = backend()
        y = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("gelu", [xs[0]], y)
        self.retain_inputs((0,))
        return (y,)

    def saved(self):
        return self.get_retained_inputs()[0]

    def backward_vars(self, indexes, gys):
        return (gelu_grad(gys[0], self.get_retained_input_vars()[0]),)


class GELUGrad(FunctionNode):
    """gy * gelu'(z): the backward of GELU as a function of both its operands.  Its own derivative with
    respect to z needs gelu''(z) = phi(z) (2 - z^2)."""

    def forward(self, xs):
        F = backend()
        out = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("gelu_bwd", [xs[0], xs[1]], out)
        self.retain_inputs((0, 1))
        return (out,)

    def backward_vars(self, indexes, gys):
        gy, z = self.get_retained_input_vars()
        return tuple(gelu_grad(gys[0], z) if i == 0 else gelu_grad2(mul(gys[0], gy), z) for i in indexes)


class GELUGrad2(FunctionNode):
    """a * gelu''(z).  Linear in a; the derivative with respect to z (a third derivative of GELU) is not
    provided."""

    def forward(self, xs):
        F = backend()
        out = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("gelu_bwd2", [xs[0], xs[1]], out)
        self.retain_inputs((1,))
        return (out,)

    def backward_vars(self, indexes, gys):
        z, = self.get_retained_input_vars()
        if 1 in indexes and z.node.requires_grad:
            raise NotImplementedError("the third derivative of gelu is not provided")
        return tuple(gelu_grad2(gys[0], z) if i == 0 else None for i in indexes)


class Sigmoid(FunctionNode):
    """1 / (1 + exp(-x)); differentiated from its output: gx = gy y (1 - y)."""

    def forward(self, xs):
        F = backend()
        out = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("sigmoid", [xs[0]], out)
        self.retain_outputs((0,))
        return (out,)

    def backward_vars(self, indexes, gys):
        y, = self.get_retained_output_vars()
        gyy = mul(gys[0], y)
        return (sub(gyy, mul(gyy, y)),)


class SliceCols(FunctionNode):
    """Columns lo .. hi - 1 of a 2-d array, as a VIEW (the kernels take any strides); the backward places
    the gradient into a zero array of the full width."""

    def __init__(self, lo, hi):
        super().__init__()
        self.lo, self.hi = lo, hi

    def forward(self, xs):
        self.width = xs[0].shape[1]
        return (xs[0][:, self.lo:self.hi],)

    def backward_vars(self, indexes, gys):
        return (PadCols(self.lo, self.width).apply((gys[0],))[0],)


class PadCols(FunctionNode):
    """(n, w) -> (n, width): the array placed at column `lo` of zeros; the backward slices it out again."""

    def __init__(self, lo, width):
        super().__init__()
        self.lo, self.width = lo, width

    def forward(self, xs):
        F = backend()
        x = xs[0]
        out = F.empty((x.shape[0], self.width), F.dtype(x))
        F.elementwise_broadcast("fill", [], out, (0.0,))
        F.elementwise_broadcast("copy", [x], out[:, self.lo:self.lo + x.shape[1]])
        self.w = x.shape[1]
        return (out,)

    def backward_vars(self, indexes, gys):
        return (slice_cols(gys[0], self.lo, self.lo + self.w),)


class Add(FunctionNode):
    """x + y with NumPy broadcasting of y's leading axes (a bias); retains nothing."""

    def forward(self, xs):
        F = backend()
        x, y = xs
        self.bias_like = tuple(y.shape) != tuple(x.shape)
        if self.bias_like and (len(y.shape) != 1 or y.shape[0] != x.shape[-1] or len(x.shape) != 2):
            raise ValueError("add: second operand must match the first or be its row-shaped bias")
        out = F.empty(x.shape, F.dtype(x))
        F.elementwise_broadcast("add", [x, y], out)
        return (out,)

    def backward(self, indexes, gys):
        F = backend()
        out = []
        for i in indexes:
            if i == 1 and self.bias_like:
                g = F.empty((gys[0].shape[1],), "f32")
                F.reduce_axis("sum", gys[0], 0, g)
                out.append(g)
            else:
                out.append(gys[0])
        return tuple(out)


    def backward_vars(self, indexes, gys):
        return tuple(sum_rows(gys[0]) if i == 1 and self.bias_like else gys[0] for i in indexes)


# ---- functions whose backward is written with functions (all of them differentiable any number of times)
class ReLUGrad(FunctionNode):
    """gy * [y > 0]: the backward of ReLU as a function of gy.  As a function of y it is constant
    almost everywhere, so y receives no gradient."""

    def forward(self, xs):
        F = backend()
        out = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("relu_bwd", [xs[0], xs[1]], out)
        self.retain_inputs((1,))
        return (out,)

    def backward_vars(self, indexes, gys):
        y, = self.get_retained_input_vars()
        return tuple(relu_grad(gys[0], y) if i == 0 else None for i in indexes)


class Mul(FunctionNode):
    """x * y, same shape; each factor's gradient is gy times the other factor."""

    def forward(self, xs):
        F = backend()
        out = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("mul", [xs[0], xs[1]], out)
        self.retain_inputs((0, 1))
        return (out,)

    def backward_vars(self, indexes, gys):
        x, y = self.get_retained_input_vars()
        return tuple(mul(gys[0], y if i == 0 else x) for i in indexes)


class Sub(FunctionNode):
    """x - y, same shape; retains nothing."""

    def forward(self, xs):
        F = backend()
        out = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("sub", [xs[0], xs[1]], out)
        return (out,)

    def backward_vars(self, indexes, gys):
        return tuple(gys[0] if i == 0 else scale(gys[0], -1.0) for i in indexes)


class Scale(FunctionNode):
    """s * x for a constant s."""

    def __init__(self, s):
        super().__init__()
        self.s = float(s)

    def forward(self, xs):
        F = backend()
        out = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("scale", [xs[0]], out, (self.s,))
        return (out,)

    def backward_vars(self, indexes, gys):
        return (scale(gys[0], self.s),)


class Tanh(FunctionNode):
    """tanh(x); differentiated from its output, gx = gy * (1 - y^2) (Section "Function-wise Local
    Memory Usage Reduction"), and since that is written with functions of y, any number of times."""

    def forward(self, xs):
        F = backend()
        out = F.empty(xs[0].shape, F.dtype(xs[0]))
        F.elementwise_broadcast("tanh", [xs[0]], out)
        self.retain_outputs((0,))
        return (out,)

    def backward_vars(self, indexes, gys):
        y, = self.get_retained_output_vars()
        return (sub(gys[0], mul(gys[0], mul(y, y))),)


class SumAll(FunctionNode):
    """Sum of every element, a 0-d result (fixed-order reduction over the flattened array)."""

    def forward(self, xs):
        F = backend()
        x = xs[0]
        self.shape, self.dt = tuple(x.shape), F.dtype(x)
        out = F.empty((1,), "f32")
        if len(x.shape) == 2:                 # any strides: rows first, then the row sums
            rows = F.empty((x.shape[0],), "f32")
            F.reduce_axis("sum", x, 1, rows)
            x = rows
        F.reduce_axis("sum", x.reshape(1, -1), 1, out)
        return (out.reshape(()),)

    def backward_vars(self, indexes, gys):
        return (broadcast_to(gys[0], self.shape),)


class BroadcastTo(FunctionNode):
    """A 0-d value repeated into `shape`; its backward is the sum of everything."""

    def __init__(self, shape):
        super().__init__()
        self.shape = tuple(shape)

    def forward(self, xs):
        F = backend()
        out = F.empty(self.shape, F.dtype(xs[0]))
        F.elementwise_broadcast("copy", [xs[0]], out)
        return (out,)

    def backward_vars(self, indexes, gys):
        return (sum_all(gys[0]),)


class SumRows(FunctionNode):
    """(n, d) -> (d,): the sum over the rows (a bias gradient); backward repeats the row."""

    def forward(self, xs):
        F = backend()
        self.n = xs[0].shape[0]
        out = F.empty((xs[0].shape[1],), "f32")
        F.reduce_axis("sum", xs[0], 0, out)
        return (out,)

    def backward_vars(self, indexes, gys):
        return (broadcast_rows(gys[0], self.n),)


class BroadcastRows(FunctionNode):
    """(d,) -> (n, d): the row repeated n times; backward sums the rows."""

    def __init__(self, n):
        super().__init__()
        self.n = n

    def forward(self, xs):
        F = backend()
        out = F.empty((self.n, xs[0].shape[0]), F.dtype(xs[0]))
        F.elementwise_broadcast("copy", [xs[0]], out)
        return (out,)

    def backward_vars(self, indexes, gys):
        return (sum_rows(gys[0]),)


class Transpose(FunctionNode):
    """The transposed VIEW of a 2-d array (no copy: the kernels take any strides)."""

    def forward(self, xs):
        return (_t(xs[0]),)

    def backward_vars(self, indexes, gys):
        return (transpose(gys[0]),)


class UserElementwise(FunctionNode):
    """A differentiable element-wise operation written as two user-defined kernels (Section "Custom
    CUDA Kernels": users extend the array layer with kernels of their own): `forward_kernel`
    maps the inputs to one output, `backward_kernel` maps (inputs..., gy) to one gradient per
    input.  Both are kernel objects called with arrays (the binding's ElementwiseKernel, or
    anything with the same call signature); all operands share one shape.  Retains its inputs."""

    def __init__(self, forward_kernel, backward_kernel):
        super().__init__()
        self.fk, self.bk = forward_kernel, backward_kernel

    def forward(self, xs):
        self.retain_inputs(tuple(range(len(xs))))
        return (self.fk(*xs),)

    def backward(self, indexes, gys):
        xs = self.get_retained_inputs()
        gxs = self.bk(*xs, gys[0])
        if not isinstance(gxs, tuple):
            gxs = (gxs,)
        if len(gxs) != len(xs):
            raise RuntimeError("the backward kernel must have one output per input")
        return tuple(gxs[i] for i in indexes)


def user_elementwise(forward_kernel, backward_kernel):
    """``softplus = user_elementwise(fk, bk); y = softplus(x)``: a function of variables made from
    two element-wise kernels."""
    def apply(*xs):
        return UserElementwise(forward_kernel, backward_kernel).apply(xs)[0]
    return apply


class SoftmaxCrossEntropy(FunctionNode):
    """Mean softmax cross-entropy of (N,C) logits against integer labels.  Retains the logits and
    keeps the per-row log-sum-exp the forward kernel produced, so the backward is one pass."""
    fresh = (0,)

    def __init__(self, ignore_label=-1, grad_dtype=None):
        super().__init__()
        self.ignore_label, self.grad_dtype, self.lse, self.labels = ignore_label, grad_dtype, None, None

    def forward(self, xs):
        F = backend()
        logits, labels = xs
        loss = F.empty((), "f32")
        self.lse = F.empty((logits.shape[0],), "f32")
        self.labels = labels
        F.softmax_ce_fwd(logits, labels, loss, self.lse, self.ignore_label)
        self.retain_inputs((0,))
        return (loss,)

    def release_locals(self):
        self.lse = self.labels = None

    def backward(self, indexes, gys):
        F = backend()
        logits, = self.get_retained_inputs()
        g = F.empty(logits.shape, self.grad_dtype or F.dtype(logits))
        F.softmax_ce_bwd(logits, self.labels, g, self.lse, 1.0, self.ignore_label)
        if not self.unit_seed:                 # an upstream factor other than the implicit 1
            F.elementwise_broadcast("mul", [g, gys[0]], g)
        return tuple(g if i == 0 else None for i in indexes)

    def backward_vars(self, indexes, gys):
        if not _record:
            return FunctionNode.backward_vars(self, indexes, gys)
        logits, = self.get_retained_input_vars()
        g = SoftmaxCEGrad(self.labels, self.lse, self.ignore_label).apply((logits, gys[0]))[0]
        return tuple(g if i == 0 else None for i in indexes)


class SoftmaxCEGrad(FunctionNode):
    """(logits, gy) -> gy * (softmax(logits) - onehot) / N_valid: the backward of the mean softmax
    cross-entropy as a function, so that it can be differentiated in turn (gradient penalties on a
    classifier's loss).  Its own backward is one kernel (the softmax Jacobian applied to the incoming
    gradient); a third derivative is not provided.  fp32."""

    def __init__(self, labels, lse, ignore_label):
        super().__init__()
        self.labels, self.lse, self.ignore_label = labels, lse, ignore_label

    def forward(self, xs):
        F = backend()
        logits, gy = xs
        g = F.empty(logits.shape, "f32")
        F.softmax_ce_bwd(logits, self.labels, g, self.lse, 1.0, self.ignore_label)
        F.elementwise_broadcast("mul", [g, gy], g)
        self.retain_inputs((0, 1))
        return (g,)

    def release_locals(self):
        self.labels = self.lse = None

    def backward(self, indexes, gys):
        F = backend()
        logits, gy = self.get_retained_inputs()
        dz = F.empty(logits.shape, "f32")
        dup = F.empty((), "f32")
        F.softmax_ce_bwd2(logits, self.labels, gys[0], dz, dup, self.lse, 1.0, self.ignore_label)
        out = []
        for i in indexes:
            if i == 0:
                F.elementwise_broadcast("mul", [dz, gy], dz)
                out.append(dz)
            else:
                out.append(dup.reshape(gy.shape))
        return tuple(out)


class EmbedID(FunctionNode):
    """out[n] = table[ids[n]]; the backward scatters rows back (a dense gradient of the table,
    summed in a fixed order).  Retains nothing but the ids."""
    fresh = (1,)

    def forward(self, xs):
        F = backend()
        ids = xs[0]
        var = self.in_vars[1]
        table = var.compute_array if isinstance(var, Parameter) else var.array   # (the bf16 working copy, if any)
        self.ids, self.table_shape = ids, tuple(table.shape)
        out = F.empty((ids.shape[0], table.shape[1]), F.dtype(table))
        F.embed_fwd(table, ids, out)
        return (out,)

    def release_locals(self):
        self.ids = None

    def backward(self, indexes, gys):
        F = backend()
        out = []
        for k, i in enumerate(indexes):
            if i != 1:
                out.append(None)
                continue
            g = self.grad_slots[k]
            if g is None:
                g = F.empty(self.table_shape, "f32")
                F.embed_bwd(self.ids, gys[0], g, False)
            else:
                F.embed_bwd(self.ids, gys[0], g, True)
            out.append(g)
        return tuple(out)

    def backward_vars(self, indexes, gys):
        if not _record:
            return FunctionNode.backward_vars(self, indexes, gys)
        return tuple(EmbedGrad(self.ids, self.table_shape).apply((gys[0],))[0] if i == 1 else None for i in indexes)


class EmbedGrad(FunctionNode):
    """dout (N, D) -> dtable (V, D): rows summed into the table rows their ids name (the backward of the
    lookup as a function).  Linear, so its own backward is the lookup again."""

    def __init__(self, ids, table_shape):
        super().__init__()
        self.ids, self.table_shape = ids, table_shape

    def forward(self, xs):
        F = backend()
        g = F.empty(self.table_shape, "f32")
        F.embed_bwd(self.ids, xs[0], g, False)
        return (g,)

    def backward_vars(self, indexes, gys):
        return (embed_id(self.ids, gys[0]),)


class LSTM(FunctionNode):
    """(c_prev, z[, bias]) -> (c, h): the cell of the recurrent language model; z holds the four
    gate pre-activations.  Backward works from retained outputs: the activated gates the forward
    kernel stored, c_prev and c."""
    fresh = (0, 1, 2)

    def __init__(self, twice_differentiable=False):
        """twice_differentiable: also retain the gate pre-activations z (and the bias), which the fused
        backward does not need but a differentiable backward does: it rebuilds the cell from element-wise
        functions of c_prev and z and differentiates that."""
        super().__init__()
        self.twice = twice_differentiable

    def forward(self, xs):
        F = backend()
        c_prev, z = xs[0], xs[1]
        bias = xs[2] if len(xs) > 2 else None
        c = F.empty(c_prev.shape, "f32")
        h = F.empty(c_prev.shape, "f32")
        self.gates = F.empty(z.shape, "f32")
        F.lstm_fwd(z, bias, c_prev, c, h, self.gates)
        self.retain_inputs(tuple(range(len(xs))) if self.twice else (0,))
        self.retain_outputs((0,))
        return (c, h)

    def backward_vars(self, indexes, gys):
        if not _record:
            return FunctionNode.backward_vars(self, indexes, gys)
        if not self.twice:
            raise NotImplementedError("lstm(..., twice_differentiable=True) is needed for a differentiable backward "
                                      "(the fused cell does not retain its pre-activations)")
        ins = self.get_retained_input_vars()
        c_prev, z = ins[0], ins[1]
        H = c_prev.shape[1]
        zb = z if len(ins) < 3 else add(z, ins[2])
        i, f, o = (sigmoid(slice_cols(zb, k * H, (k + 1) * H)) for k in (0, 1, 3))
        g = tanh(slice_cols(zb, 2 * H, 3 * H))
        c = add(mul(f, c_prev), mul(i, g))
        h = mul(o, tanh(c))
        pairs = [(y, gy) for y, gy in zip((c, h), gys) if gy is not None]
        res = _backward_vars([y for y, _ in pairs], [gy for _, gy in pairs], [ins[k] for k in indexes], False)
        return tuple(res.get(id(ins[k].node)) for k in indexes)

    def release_locals(self):
        self.gates = None

    def backward(self, indexes, gys):
        F = backend()
        c_prev = self.get_retained_inputs()[0]
        c, = self.get_retained_outputs()
        gc, gh = gys
        if gh is None:
            gh = F.empty(c.shape, "f32")
            F.elementwise_broadcast("fill", [], gh, (0.0,))
        dz = F.empty(self.gates.shape, "f32")
        dc_prev = F.empty(c.shape, "f32")
        F.lstm_bwd(self.gates, c_prev, c, gh, gc, dz, dc_prev)
        out = []
        for i in indexes:
            if i == 0:
                out.append(dc_prev)
            elif i == 1:
                out.append(dz)
            else:
                gb = F.empty((dz.shape[1],), "f32")
                F.reduce_axis("sum", dz, 0, gb)
                out.append(gb)
        return tuple(out)


class NStepLSTM(FunctionNode):
    """(c0, h0, zx, U, bias) -> (c_T, h_T, hs): all time steps of one LSTM layer in one function node.

    zx (T*B, 4H) holds the input part of the gate pre-activations of every step (time-major: rows
    t*B .. t*B + B - 1 belong to step t), U (H, 4H) the recurrent weights; hs (T*B, H) stacks the
    hidden states h_1 .. h_T the same way.  Step by step the tape would record a product, a sum and
    a cell per time step and, backwards, add T small weight-gradient products into U's gradient;
    here the forward is one launch per step where the backend fuses product and cell (two
    otherwise), and the backward computes U's gradient as one product over all steps once every
    step's gate gradient is known.  The arithmetic per element is that of the step-by-step graph;
    sums over time are taken in a different order.

    ``lowp``: what feeds a matrix product is stored in bfloat16 -- the hidden states, their gradients,
    the gate gradients, and U is read from its parameter's working copy; gates, cell states and
    parameter gradients stay fp32.  The backward step is then fused as well where the backend can."""
    fresh = (0, 1, 2, 3, 4)

    def __init__(self, n_steps, lowp=False):
        super().__init__()
        self.T, self.lowp = int(n_steps), lowp

    def _input_array(self, var):
        return var.compute_array if isinstance(var, Parameter) else var.array

    def forward(self, xs):
        F = backend()
        c0, h0, zx, _, bias = xs
        U = self._input_array(self.in_vars[3])
        T, Bn, H = self.T, c0.shape[0], c0.shape[1]
        if tuple(zx.shape) != (T * Bn, 4 * H) or tuple(U.shape) != (H, 4 * H) or tuple(h0.shape) != (Bn, H):
            raise ValueError("n_step_lstm: zx %s, U %s, c0 %s, h0 %s do not fit %d steps"
                             % (tuple(zx.shape), tuple(U.shape), tuple(c0.shape), tuple(h0.shape), T))
        adt = "bf16" if self.lowp else "f32"
        blk = lambda a, t: a[t * Bn:(t + 1) * Bn]
        Hs, Cs = F.empty(((T + 1) * Bn, H), adt), F.empty(((T + 1) * Bn, H), "f32")   # block 0 = initial state
        F.elementwise_broadcast("copy", [h0], blk(Hs, 0))
        F.elementwise_broadcast("copy", [c0], blk(Cs, 0))
        G = F.empty((T * Bn, 4 * H), "f32")
        self.fused = F.fuses_lstm_step(H)
        if self.fused:
            Ut = F.empty((4 * H, H), adt)
            F.elementwise_broadcast("copy", [_t(U)], Ut)
            F.lstm_steps_fwd(zx, Hs, Ut, bias, Cs, G, T)
        else:
            F.elementwise_broadcast("copy", [zx], G)                 # the pre-activations are completed in place
            for t in range(T):
                F.gemm(blk(Hs, t), U, blk(G, t), beta=1.0)
                F.lstm_fwd(blk(G, t), bias, blk(Cs, t), blk(Cs, t + 1), blk(Hs, t + 1), blk(G, t))
        self.Hs, self.Cs, self.G = Hs, Cs, G
        self.retain_inputs((3,))
        return (blk(Cs, T), blk(Hs, T), Hs[Bn:])

    def release_locals(self):
        self.Hs = self.Cs = self.G = None

    def backward(self, indexes, gys):
        F = backend()
        U, = self.get_retained_inputs()
        Hs, Cs, G, T = self.Hs, self.Cs, self.G, self.T
        Bn, H = Hs.shape[0] // (T + 1), Hs.shape[1]
        adt = "bf16" if self.lowp else "f32"
        blk = lambda a, t: a[t * Bn:(t + 1) * Bn]
        gc, gh, ghs = gys
        dHs = F.empty((T * Bn, H), adt)                              # gradient reaching h_1 .. h_T from outside
        if ghs is None:
            F.elementwise_broadcast("fill", [], dHs, (0.0,))
        else:
            F.elementwise_broadcast("copy", [ghs], dHs)
        if gh is not None:
            if F.dtype(gh) != F.dtype(dHs):
                g2 = F.empty((Bn, H), adt)
                F.elementwise_broadcast("copy", [gh], g2)
                gh = g2
            F.elementwise_broadcast("add", [blk(dHs, T - 1), gh], blk(dHs, T - 1))
        dZ = F.empty((T * Bn, 4 * H), adt)
        dc = [F.empty((Bn, H), "f32"), F.empty((Bn, H), "f32")]
        dh0 = F.empty((Bn, H), adt)
        dc_next = gc
        fused_bwd = self.lowp and self.fused       # (in fp32 the three separate calls are the faster ones)
        if fused_bwd:                              # per step: dh_t += dz_{t+1} U^T, then the cell
            F.lstm_steps_bwd(dZ, U, dHs, G, Cs, gc, dc, T)
        else:
            for t in range(T - 1, -1, -1):
                F.lstm_bwd(blk(G, t), blk(Cs, t), blk(Cs, t + 1), blk(dHs, t), dc_next, blk(dZ, t), dc[t & 1])
                if t > 0:
                    F.gemm(blk(dZ, t), _t(U), blk(dHs, t - 1), beta=1.0)
                dc_next = dc[t & 1]
        if 1 in indexes:
            F.gemm(blk(dZ, 0), _t(U), dh0)
        out = []
        for i in indexes:
            if i == 0:
                out.append(dc[0])
            elif i == 1:
                out.append(dh0)
            elif i == 2:
                out.append(dZ)
            elif i == 3:
                gU = F.empty(tuple(U.shape), "f32")
                F.gemm(_t(Hs[:T * Bn]), dZ, gU)
                out.append(gU)
            else:
                gb = F.empty((4 * H,), "f32")
                F.reduce_axis("sum", dZ, 0, gb)
                out.append(gb)
        return tuple(out)


class SplitRows(FunctionNode):
    """Cut a (n*r, d) array into n views of r rows (no copy; the views keep the buffer alive).
    The backward gathers the pieces' gradients into one array, zero where a piece was unused."""
    fresh = (0,)

    def __init__(self, n):
        super().__init__()
        self.n = n

    def forward(self, xs):
        x, = xs
        if x.shape[0] % self.n:
            raise ValueError("split_rows: %d rows do not divide into %d pieces" % (x.shape[0], self.n))
        r = x.shape[0] // self.n
        self.shape, self.dt = tuple(x.shape), backend().dtype(x)
        return tuple(x[k * r:(k + 1) * r] for k in range(self.n))

    def backward(self, indexes, gys):
        F = backend()
        g = F.empty(self.shape, self.dt)
        r = self.shape[0] // self.n
        for k, gy in enumerate(gys):
            blk = g[k * r:(k + 1) * r]
            if gy is None:
                F.elementwise_broadcast("fill", [], blk, (0.0,))
            else:
                F.elementwise_broadcast("copy", [gy], blk)
        return (g,)


class ConcatRows(FunctionNode):
    """Stack equally shaped (r, d) arrays along the rows; the backward hands out views."""

    def forward(self, xs):
        F = backend()
        r = xs[0].shape[0]
        out = F.empty((r * len(xs),) + tuple(xs[0].shape[1:]), F.dtype(xs[0]))
        for k, x in enumerate(xs):
            if tuple(x.shape) != tuple(xs[0].shape):
                raise ValueError("concat_rows: pieces differ in shape")
            F.elementwise_broadcast("copy", [x], out[k * r:(k + 1) * r])
        self.r = r
        return (out,)

    def backward(self, indexes, gys):
        return tuple(gys[0][i * self.r:(i + 1) * self.r] for i in indexes)


def linear(x, W, b, act=None, out_dtype=None):
    return LinearFunction(act, out_dtype).apply((x, W, b))[0]


def matmul(x, W, out_dtype=None, gx_dtype=None):
    return MatMul(out_dtype, gx_dtype).apply((x, W))[0]


def relu(x):
    return ReLU().apply((x,))[0]


def gelu(x):
    return GELU().apply((x,))[0]


def gelu_grad(gy, z):
    return GELUGrad().apply((gy, z))[0]


def gelu_grad2(a, z):
    return GELUGrad2().apply((a, z))[0]


def sigmoid(x):
    return Sigmoid().apply((x,))[0]


def slice_cols(x, lo, hi):
    return SliceCols(lo, hi).apply((x,))[0]


def add(x, y):
    return Add().apply((x, y))[0]


def relu_grad(gy, y):
    return ReLUGrad().apply((gy, y))[0]


def mul(x, y):
    return Mul().apply((x, y))[0]


def sub(x, y):
    return Sub().apply((x, y))[0]


def scale(x, s):
    return Scale(s).apply((x,))[0]


def tanh(x):
    return Tanh().apply((x,))[0]


def sum_all(x):
    return SumAll().apply((x,))[0]


def broadcast_to(x, shape):
    return BroadcastTo(shape).apply((x,))[0]


def sum_rows(x):
    return SumRows().apply((x,))[0]


def broadcast_rows(x, n):
    return BroadcastRows(n).apply((x,))[0]


def transpose(x):
    return Transpose().apply((x,))[0]


def softmax_cross_entropy(logits, labels, ignore_label=-1, grad_dtype=None):
    return SoftmaxCrossEntropy(ignore_label, grad_dtype).apply((logits, labels))[0]


def embed_id(ids, table):
    return EmbedID().apply((ids, table))[0]


def lstm(c_prev, z, bias=None, twice_differentiable=False):
    """Returns (c, h)."""
    return LSTM(twice_differentiable).apply((c_prev, z) if bias is None else (c_prev, z, bias))


def n_step_lstm(c0, h0, zx, U, bias, n_steps, lowp=False):
    """All n_steps time steps of an LSTM layer; returns (c_T, h_T, hs) with hs (n_steps*B, H)."""
    return NStepLSTM(n_steps, lowp).apply((c0, h0, zx, U, bias))


def split_rows(x, n):
    return SplitRows(n).apply((x,))


def concat_rows(xs):
    return ConcatRows().apply(tuple(xs))[0]


# ---- links and optimiser -------------------------------------------------------------------------------
class Linear:
    """The Linear link of the model-definition figure: parameters W (n_out, n_in) and b (n_out,)
    bound to the forward code ``y = x W^T + b``."""

    def __init__(self, W, b, lowp=None):
        self.W = Parameter(W, lowp, "W")
        self.b = Parameter(b, None, "b")

    def params(self):
        return [self.W, self.b]

    def __call__(self, x, act=None, out_dtype=None):
        return linear(x, self.W, self.b, act, out_dtype)


class SGD:
    """param <- param - lr * grad for every parameter that received a gradient, in one call for the
    whole set (Section "Background and Motivation": the update ends each iteration)."""

    def __init__(self, params, lr):
        self.params, self.lr = list(params), float(lr)

    def cleargrads(self):
        for p in self.params:
            p.cleargrad()

    def update(self):
        ps = [p for p in self.params if p.grad is not None]
        if not ps:
            return
        lows = [p.lowp for p in ps]
        backend().sgd_update_multi([p.array for p in ps], [p.grad for p in ps], self.lr,
                                   lows if any(l is not None for l in lows) else None)


class Adam(SGD):
    """Adam (the optimiser of the paper's distributed-training code figure): first and second moment
    estimates per parameter, created zero on first use; one call updates the whole set."""

    def __init__(self, params, lr=0.001, beta1=0.9, beta2=0.999, eps=1e-8):
        super().__init__(params, lr)
        self.beta1, self.beta2, self.eps, self.t = beta1, beta2, eps, 0
        self._state = {}

    def update(self):
        ps = [p for p in self.params if p.grad is not None]
        if not ps:
            return
        F = backend()
        self.t += 1
        for p in ps:
            if id(p) not in self._state:
                m, v = F.empty(p.array.shape, "f32"), F.empty(p.array.shape, "f32")
                F.elementwise_broadcast("fill", [], m, (0.0,))
                F.elementwise_broadcast("fill", [], v, (0.0,))
                self._state[id(p)] = (m, v)
        lows = [p.lowp for p in ps]
        F.adam_update_multi([p.array for p in ps], [p.grad for p in ps], [self._state[id(p)][0] for p in ps],
                            [self._state[id(p)][1] for p in ps], self.lr, self.t, self.beta1, self.beta2, self.eps,
                            lows if any(l is not None for l in lows) else None)


# ---- the two model families of the benchmark workloads, written as define-by-run forward code ---------
class MLP:
    """``l_n(act(... act(l_1(x))))`` with softmax cross-entropy on top (the model-definition figure
    of Section "API Design", any depth).  ``params``: list of (W, b) backend arrays.

    ``lowp``: bf16 working copies of the weights, bf16 activations and activation gradients; fp32
    logits, loss, weight/bias gradients and master weights.  ``fused_activation=False`` applies the
    activation as a function node of its own instead of in the product's epilogue.
    """

    def __init__(self, params, act="relu", lowp=False, fused_activation=True):
        F = backend()
        self.act, self.lowp, self.fused = act, lowp, fused_activation
        self.layers = []
        for W, b in params:
            low = None
            if lowp:
                low = F.empty(W.shape, "bf16")
                F.elementwise_broadcast("copy", [W], low)
            self.layers.append(Linear(W, b, low))

    def params(self):
        return [p for l in self.layers for p in l.params()]

    def __call__(self, x):
        h = x
        for l in self.layers[:-1]:
            if self.fused:
                h = l(h, act=self.act)
            else:
                h = (relu if self.act == "relu" else gelu)(l(h))
        return self.layers[-1](h, out_dtype="f32")

    def loss(self, x, t):
        return softmax_cross_entropy(self(x), t, grad_dtype="bf16" if self.lowp else None)


class LSTMLanguageModel:
    """Embedding, one LSTM layer, output Linear layer, softmax cross-entropy over every (time,
    batch) token; time-major rows (row t*B + b).  ``P``: dict of backend arrays E (V,E), W (E,4H),
    U (H,4H), b (4H,), W_out (V,H), b_out (V,).  The forward code is ordinary Python: the number of
    time steps is whatever the batch at hand has.  ``n_step``: the recurrent layer is one
    ``n_step_lstm`` node instead of a product, a sum and a cell per time step."""

    def __init__(self, P, n_step=False, lowp=False):
        """lowp (with n_step): bf16 working copies of E, W, U and W_out feed the products, as do bf16
        embeddings, hidden states and their gradients; everything else stays fp32."""
        if lowp and not n_step:
            raise ValueError("LSTMLanguageModel: lowp needs n_step=True")
        F = backend()
        self.P = {}
        for k, v in P.items():
            low = None
            if lowp and k in ("E", "W", "U", "W_out"):
                low = F.empty(tuple(v.shape), "bf16")
                F.elementwise_broadcast("copy", [v], low)
            self.P[k] = Parameter(v, low, k)
        self.n_step, self.lowp = n_step, lowp

    def params(self):
        return list(self.P.values())

    def loss(self, ids, targets, n_steps, state=None):
        """ids, targets: flat (T*B,) integer arrays.  Returns (loss, (c, h)) so that a caller may
        carry the state into the next window (after ``unchain`` for truncated back-propagation)."""
        P, F = self.P, backend()
        X = embed_id(ids, P["E"])
        zx = matmul(X, P["W"], out_dtype="f32", gx_dtype="f32")
        if state is None:
            Bn, H = ids.shape[0] // n_steps, P["U"].shape[0]
            z0 = F.empty((Bn, H), "f32")
            F.elementwise_broadcast("fill", [], z0, (0.0,))
            c = h = Variable(z0, requires_grad=False)
        else:
            c, h = state
        if self.n_step:
            c, h, hs = n_step_lstm(c, h, zx, P["U"], P["b"], n_steps, self.lowp)
            logits = linear(hs, P["W_out"], P["b_out"], out_dtype="f32")
            return softmax_cross_entropy(logits, targets, grad_dtype="bf16" if self.lowp else None), (c, h)
        zs = split_rows(zx, n_steps)
        hs = []
        for t in range(n_steps):
            c, h = lstm(c, add(zs[t], matmul(h, P["U"])), P["b"])
            hs.append(h)
        logits = linear(concat_rows(hs), P["W_out"], P["b_out"])
        return softmax_cross_entropy(logits, targets), (c, h)
