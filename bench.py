#!/usr/bin/env python3
"""Benchmark of the training-step hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A "step" is one forward + backward + SGD pass of the wide MLP workload (4096-4096-4096-4096-1000,
GELU, batch 8192, bf16 storage with fp32 accumulation and fp32 master weights) issued call by call
through the C ABI; the printed JSON line reports train steps/s for it, the roofline figure of the
kernel that dominates it (the bf16 MFMA GEMM), the CPU oracle timed on a bounded sample of the same
workload, and -- under "workloads" -- the other benchmark configurations: the array microbenchmark
(element-wise / reduction GB/s against the HBM peak), the fp32/bf16 MLP and the LSTM language-model
step.  All inputs are seeded synthetic tensors already resident in HBM when timing starts.
Protocol of the headline: W warm-up steps of the very callable that is timed (the recorded step, no
instrumentation), then `--repeats` (5) regions of exactly K steps each between HIP events on the launch
stream; the median region is `value`, all regions are listed.  Per-product times (and the roofline
figure built from them) come from a separate pass afterwards in which every GEMM call sits between two
events created beforehand.
One GPU only: this build has no multi-GPU path, and --gpus N > 1 exits with a message.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
# HBM-side bytes per launch of the dominant kernel (L2 misses fetched + bytes written), from the two
# counter runs recorded in profiles/gemm_bf16_forward_8192x4096x4096_counters.txt (made with
# `bench.py --traffic-driver gemm` under rocprofv3 --pmc); 403.3 MB fetched + 134.2 MB written.
DOMINANT_KERNEL_TRAFFIC_BYTES = 537.5e6


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Timer:
    """HIP-event stopwatch on the stream the kernels are launched on (torch's current stream)."""

    def __init__(self, torch):
        self.torch = torch

    def time(self, fn, iters, warmup):
        t = self.torch
        for _ in range(warmup):
            fn()
        t.cuda.synchronize()
        e0, e1 = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        t.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / iters       # seconds per call

    def repeats(self, fn, iters, warmup, n):
        """`n` timed regions of exactly `iters` calls each (warm-up before the first only); seconds per
        call of every region, in run order."""
        return [self.time(fn, iters, warmup if r == 0 else 0) for r in range(n)]


def bench_array(torch, B, W, timer, quick):
    """Workload 2: y = relu(a*b + c) with a row-broadcast c, sums over both axes, transposed views."""
    n = 8192
    out = {}
    w = W.config2(n)
    for name, tdt, isz in (("f32", torch.float32, 4), ("bf16", torch.bfloat16, 2)):
        sets = 2 if name == "f32" else 4            # rotate buffers: defeat the 256 MB Infinity Cache
        a = [B.cast(torch.from_numpy(w.a).cuda(), tdt) for _ in range(sets)]
        b = [B.cast(torch.from_numpy(w.b).cuda(), tdt) for _ in range(sets)]
        c = B.cast(torch.from_numpy(w.c).cuda(), tdt)
        y = [torch.empty(n, n, dtype=tdt, device="cuda") for _ in range(4)]
        o = torch.empty(n, dtype=torch.float32, device="cuda")
        ws = torch.empty(max(256, B.reduce_axis_workspace_bytes(y[0], 0)), dtype=torch.uint8, device="cuda")
        k = [0]

        def rot(fn):
            def g():
                k[0] += 1
                fn(k[0])
            return g
        iters = 8 if quick else 40
        cases = {
            "mad_relu": (rot(lambda i: B.elementwise_broadcast("mad_relu", [a[i % sets], b[i % sets], c], y[i % 4])), 3 * n * n * isz + n * isz),
            "mad_relu_transposed_a": (rot(lambda i: B.elementwise_broadcast("mad_relu", [a[i % sets].t(), b[i % sets], c], y[i % 4])), 3 * n * n * isz + n * isz),
            "sum_axis0": (rot(lambda i: B.reduce_axis("sum", y[i % 4], 0, o, ws=ws)), n * n * isz + n * 4),
            "sum_axis1": (rot(lambda i: B.reduce_axis("sum", y[i % 4], 1, o, ws=ws)), n * n * isz + n * 4),
            "sum_axis0_transposed": (rot(lambda i: B.reduce_axis("sum", y[i % 4].t(), 0, o, ws=ws)), n * n * isz + n * 4),
            "sum_axis1_transposed": (rot(lambda i: B.reduce_axis("sum", y[i % 4].t(), 1, o, ws=ws)), n * n * isz + n * 4),
        }
        # the same work through user-defined kernels (snippets compiled at run time, generic type T)
        uk_mad = B.ElementwiseKernel("T x, T y, T z", "T w", "w = x * y + z", "my_mad")
        uk_mad_relu = B.ElementwiseKernel("T x, T y, T z", "T w", "w = fmaxf(x * y + z, 0.0f)", "my_mad_relu")
        uk_sum = B.ReductionKernel("T x", "float32 y", "x", "a + b", "y = a", "0", "my_sum")
        o0 = torch.empty((), dtype=torch.float32, device="cuda")
        uws = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")
        cases.update({
            "user_my_mad": (rot(lambda i: uk_mad(a[i % sets], b[i % sets], y[(i + 1) % 4], y[i % 4])), 4 * n * n * isz),
            "user_mad_relu_row_c": (rot(lambda i: uk_mad_relu(a[i % sets], b[i % sets], c, y[i % 4])), 3 * n * n * isz + n * isz),
            "user_sum_axis0": (rot(lambda i: uk_sum(y[i % 4], o, axis=0, ws=uws)), n * n * isz + n * 4),
            "user_sum_axis1": (rot(lambda i: uk_sum(y[i % 4], o, axis=1, ws=uws)), n * n * isz + n * 4),
            "user_sum_all": (rot(lambda i: uk_sum(y[i % 4], o0, axis=None, ws=uws)), n * n * isz + 4),
        })
        for cname, (fn, nbytes) in cases.items():
            s = timer.time(fn, iters, 4)
            gbs = nbytes / s / 1e9
            out["%s_%s" % (cname, name)] = {"us": round(s * 1e6, 2), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                                            "algorithmic_bytes": nbytes}
            log("  cfg2 %-28s %-5s %9.1f us  %8.1f GB/s  %.1f%% of HBM peak" % (cname, name, s * 1e6, gbs, 100 * gbs / HBM_PEAK_GBS))
        del a, b, y
        torch.cuda.empty_cache()
    return out


class GemmProbe:
    """Brackets every GEMM launch of a recorded step with HIP events (same stream) so that the time of
    each launch can be read back afterwards.  A measurement pass of its own, run after the timed
    region of the step benchmark: recording two events per product costs host and device time that
    the step itself does not have.  The events exist before the pass starts."""

    def __init__(self, torch, B, prog, slots):
        self.torch = torch
        self.fn = B.lib().chn_gemm
        self.prog = prog
        self.n = sum(1 for fn, _ in prog.calls if fn is self.fn)
        mk = lambda: torch.cuda.Event(enable_timing=True)
        self.events = [[(mk(), mk()) for _ in range(self.n)] for _ in range(slots)]
        self.used = set()

    def run(self, slot):
        import ctypes as C
        s = C.c_void_p(self.torch.cuda.current_stream().cuda_stream)
        ev = iter(self.events[slot])
        for fn, args in self.prog.calls:
            if fn is self.fn:
                e0, e1 = next(ev)
                e0.record()
                st = fn(*args, s)
                e1.record()
            else:
                st = fn(*args, s)
            if st != 0:
                raise RuntimeError("chn call failed with status %d" % st)
        self.used.add(slot)

    def empty_pair_seconds(self, n=40):
        """Median time between two events recorded back to back with nothing between them: what a bracket
        reads beyond the kernel it encloses (the kernel trace of the profiler does not contain it)."""
        t = self.torch
        pairs = [(t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)) for _ in range(n)]
        t.cuda.synchronize()
        for e0, e1 in pairs:
            e0.record()
            e1.record()
        t.cuda.synchronize()
        return sorted(e0.elapsed_time(e1) for e0, e1 in pairs)[n // 2] * 1e-3

    def per_call_seconds(self):
        tot = [0.0] * self.n
        for slot in self.used:
            for i, (e0, e1) in enumerate(self.events[slot]):
                tot[i] += e0.elapsed_time(e1) * 1e-3
        return [x / max(1, len(self.used)) for x in tot]


def gemm_shapes_mlp(sizes, batch, fused_update):
    """(label, M, N, K) of every GEMM of one MLP step in issue order (see steps.MLPTrainer)."""
    n = len(sizes) - 1
    out = [("fwd%d" % l, batch, sizes[l + 1], sizes[l]) for l in range(n)]
    for l in range(n - 1, -1, -1):
        dW = ("dW%d%s" % (l, "+sgd" if fused_update else ""), sizes[l + 1], sizes[l], batch)
        dx = [("dx%d" % l, batch, sizes[l], sizes[l + 1])] if l > 0 else []
        out += dx + [dW] if fused_update else [dW] + dx
    return out


def bench_mlp(torch, B, steps_mod, w, lowp, timer, steps, warmup, probe=False, graph=False, fused_update=False, repeats=1,
              probe_steps=20):
    """Times the recorded step (`repeats` regions of exactly `steps` steps after `warmup` steps of the same
    callable; the median region is reported, all regions are listed).
    fused_update: the SGD update of the weights runs in the epilogue of the weight-gradient products
    (same arithmetic, the gradients do not travel through memory); still one full
    forward + backward + update step.
    probe: afterwards, outside every timed region, `probe_steps` more steps run with each GEMM launch
    bracketed by HIP events (per-product times and rates)."""
    tr = steps_mod.MLPTrainer(w.params, w.batch, w.act, w.lr, lowp, fused_update=fused_update)
    xs = [torch.from_numpy(x).cuda() for x in w.xs]
    if lowp:
        xs = [B.cast(x, torch.bfloat16) for x in xs]
    ts = [torch.from_numpy(t).cuda() for t in w.ts]
    nb = len(xs)
    for i in range(nb):
        tr.step(xs[i], ts[i])                                   # builds the call lists
    res = {}
    k = [0]

    def fn():
        tr.step(xs[k[0] % nb], ts[k[0] % nb], graph=graph)
        k[0] += 1
    regions = timer.repeats(fn, steps, warmup, repeats)
    s = sorted(regions)[len(regions) // 2]
    if repeats > 1:
        res["ms_per_step_regions"] = [round(r * 1e3, 4) for r in regions]
        res["ms_per_step_spread"] = [round(min(regions) * 1e3, 4), round(max(regions) * 1e3, 4)]
    if probe:
        per_batch = (probe_steps + nb - 1) // nb
        probes = [GemmProbe(torch, B, tr._progs[(xs[i].data_ptr(), ts[i].data_ptr())], per_batch) for i in range(nb)]
        for i in range(nb):                                     # warm the instrumented path (events get re-recorded)
            probes[i].run(0)
        torch.cuda.synchronize()
        for slot in range(per_batch):
            for i in range(nb):
                probes[i].run(slot)
        torch.cuda.synchronize()
        per = [0.0] * probes[0].n
        for p in probes:
            for i, v in enumerate(p.per_call_seconds()):
                per[i] += v / len(probes)
        empty = probes[0].empty_pair_seconds()
        # "us": the event bracket as read; "us_net": minus what an empty bracket reads (the launch itself;
        # for a product of a few microseconds the bracket's own cost is a large part of "us")
        res["gemm_calls"] = [{"call": lab, "M": M, "N": N, "K": K, "us": round(t_ * 1e6, 1),
                              "TFLOP/s": round(2.0 * M * N * K / t_ / 1e12, 1),
                              "us_net": round(max(t_ - empty, 1e-7) * 1e6, 1),
                              "TFLOP/s_net": round(2.0 * M * N * K / max(t_ - empty, 1e-7) / 1e12, 1)}
                             for (lab, M, N, K), t_ in zip(gemm_shapes_mlp(w.sizes, w.batch, fused_update), per)]
        res["gemm_seconds_per_step"] = sum(per)
        res["gemm_flops_per_step"] = sum(2.0 * M * N * K for _, M, N, K in gemm_shapes_mlp(w.sizes, w.batch, fused_update))
        res["gemm_probe_steps"] = per_batch * nb
        res["event_pair_empty_us"] = round(empty * 1e6, 2)
    res.update({"ms_per_step": s * 1e3, "steps_per_s": 1.0 / s, "loss": float(tr.loss.cpu()),
                "TFLOP/s": w.flops_per_step() / s / 1e12, "launch_calls_per_step": tr.n_launch_calls(xs[0], ts[0])})
    return res


def bench_lstm(torch, B, steps_mod, w, timer, steps, warmup, graph=False, lowp=False):
    tr = steps_mod.LSTMTrainer(w.params, w.bptt, w.batch, w.lr, lowp=lowp)
    ids, tg = torch.from_numpy(w.ids).cuda(), torch.from_numpy(w.targets).cuda()
    s = timer.time(lambda: tr.step(ids, tg, graph=graph), steps, warmup)
    if not tr.sequence_complete():
        raise SystemExit("bench.py: a wait of the whole-sequence recurrent kernel ran out; the timing of workload 4 is void")
    return {"ms_per_step": s * 1e3, "steps_per_s": 1.0 / s, "tokens_per_s": w.bptt * w.batch / s, "loss": float(tr.loss.cpu()),
            "forward_steps_in_one_launch": bool(tr.whole_sequence), "backward_steps_in_one_launch": bool(tr.whole_sequence_bwd),
            "TFLOP/s": w.flops_per_step() / s / 1e12, "frac_mfma_peak_f32": w.flops_per_step() / s / 1e12 / MFMA_PEAK_TFLOPS["f32"],
            "launch_calls_per_step": tr.n_launch_calls(ids, tg)}


def bench_tape(torch, W, timer, quick):
    """The same training steps issued by the define-by-run tape instead of a recorded call list:
    graph recorded during the forward code, walked back, released, optimiser -- every iteration."""
    from paper_1908_00213_amd import tape as T
    F = T.backend()
    res = {}

    def mlp(w, lowp, steps, warmup):
        model = T.MLP([(F.from_numpy(Wm), F.from_numpy(b)) for Wm, b in w.params], w.act, lowp)
        opt = T.SGD(model.params(), w.lr)
        xs = [F.from_numpy(x, "bf16" if lowp else None) for x in w.xs]
        ts = [F.from_numpy(t) for t in w.ts]
        k, last = [0], [None]

        def fn():
            opt.cleargrads()
            loss = model.loss(xs[k[0] % len(xs)], ts[k[0] % len(xs)])
            loss.backward()
            opt.update()
            last[0] = loss.array
            k[0] += 1
        s = timer.time(fn, steps, warmup)
        return {"ms_per_step": s * 1e3, "steps_per_s": 1.0 / s, "loss": float(last[0].cpu()),
                "TFLOP/s": w.flops_per_step() / s / 1e12}

    res["cfg5_wide_mlp_bf16"] = mlp(W.config5(n_batches=4), True, 20, 3)
    torch.cuda.empty_cache()
    if quick:
        return res
    res["cfg3_mlp_f32"] = mlp(W.config3(), False, 100, 10)
    res["cfg3_mlp_bf16"] = mlp(W.config3(), True, 100, 10)
    res["cfg1_tiny_mlp_f32"] = mlp(W.config1(), False, 200, 20)
    w = W.config4()
    ids, tg = F.from_numpy(w.ids.reshape(-1)), F.from_numpy(w.targets.reshape(-1))
    # step by step (a product, a sum and a cell node per time step), the recurrent layer as one node,
    # and that with the hidden width rounded up to 672 by inert units (the width the fused step takes)
    padded = W.pad_lstm_params(w.params)
    for name, params, n_step, lowp in (("cfg4_lstm_lm_f32", w.params, False, False), ("cfg4_lstm_lm_f32_n_step", w.params, True, False),
                                       ("cfg4_lstm_lm_f32_n_step_padded", padded, True, False),
                                       ("cfg4_lstm_lm_bf16_n_step_padded", padded, True, True)):
        model = T.LSTMLanguageModel({k: F.from_numpy(v) for k, v in params.items()}, n_step=n_step, lowp=lowp)
        opt = T.SGD(model.params(), w.lr)
        last = [None]

        def fn():
            opt.cleargrads()
            loss, _ = model.loss(ids, tg, w.bptt)
            loss.backward()
            opt.update()
            last[0] = loss.array
        s = timer.time(fn, 10, 2)
        res[name] = {"ms_per_step": s * 1e3, "steps_per_s": 1.0 / s, "tokens_per_s": w.bptt * w.batch / s,
                     "loss": float(last[0].cpu())}
        del model, opt
    return res


def traffic_driver(torch, B, W, what):
    """What `rocprofv3 --pmc ...` is pointed at (counters in runs of their own).  Every variant alternates,
    three times, a 256 MiB fp32 copy through chn_elementwise_broadcast (the calibration launch: reads and
    writes exactly 268435456 bytes) with the launches under study, a 256 MiB scratch add after each to flush
    the caches.
    gemm:  the dominant launch of the headline workload, one hidden layer's forward product x @ W.T + b with
           the GELU epilogue that also writes the pre-activation (M=8192, N=4096, K=4096, bf16 in / bf16 out).
    array: every kernel of the array microbenchmark once (8192 x 8192, fp32 then bf16): multiply-add-ReLU
           with a row operand, the same with a transposed first operand, sums over axis 0 and axis 1."""
    src = torch.zeros(64 * 1024 * 1024, device="cuda", dtype=torch.float32)
    dst = torch.empty_like(src)
    scratch = torch.zeros(64 * 1024 * 1024, device="cuda", dtype=torch.float32)
    if what == "gemm":
        w = W.config5(n_batches=1)
        bf = torch.bfloat16
        x = B.cast(torch.from_numpy(w.xs[0]).cuda(), bf)
        Wm = B.cast(torch.from_numpy(w.params[0][0]).cuda(), bf)
        bias = torch.from_numpy(w.params[0][1]).cuda()
        out = torch.empty((w.batch, Wm.shape[0]), device="cuda", dtype=bf)
        pre = torch.empty_like(out)
        launches = [lambda: B.gemm(x, Wm.t(), out, epilogue="bias_gelu", bias=bias, preact_out=pre)]
    else:
        n = 8192
        w = W.config2(n)
        launches = []
        for tdt in (torch.float32, torch.bfloat16):
            a, b, c = (B.cast(torch.from_numpy(t).cuda(), tdt) for t in (w.a, w.b, w.c))
            y = torch.empty(n, n, dtype=tdt, device="cuda")
            o = torch.empty(n, dtype=torch.float32, device="cuda")
            ws = torch.empty(max(256, B.reduce_axis_workspace_bytes(y, 0)), dtype=torch.uint8, device="cuda")
            launches += [lambda a=a, b=b, c=c, y=y: B.elementwise_broadcast("mad_relu", [a, b, c], y),
                         lambda a=a, b=b, c=c, y=y: B.elementwise_broadcast("mad_relu", [a.t(), b, c], y),
                         lambda y=y, o=o, ws=ws: B.reduce_axis("sum", y, 0, o, ws=ws),
                         lambda y=y, o=o, ws=ws: B.reduce_axis("sum", y, 1, o, ws=ws)]
    for _ in range(3):
        B.elementwise_broadcast("copy", [src], dst)
        scratch.add_(1.0)
        for fn in launches:
            fn()
            scratch.add_(1.0)
    torch.cuda.synchronize()
    log("traffic driver (%s): 3 x (copy 256 MiB, flush, %d launches with a flush after each) done" % (what, len(launches)))


class _SysfsSampler:
    """Reads the driver's own gauges (shader clock as the starred line of pp_dpm_sclk, board power from
    hwmon) every 20 ms on a thread of its own while a measurement runs.  Read-only; where the files are
    missing or unreadable the probe reports no clock and power."""

    def __init__(self):
        import glob
        self.sclk = next(iter(sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))), None)
        self.power = next(iter(sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                                      glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))), None)

    def _read(self):
        mhz = watts = None
        try:
            for line in open(self.sclk):
                if line.rstrip().endswith("*"):
                    mhz = float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        except Exception:
            pass
        try:
            watts = float(open(self.power).read()) * 1e-6
        except Exception:
            pass
        return mhz, watts

    def run(self, fn):
        """fn() once (it synchronises itself); returns (its result, median MHz or None, median W or None)."""
        import threading
        stop, samples = threading.Event(), []

        def loop():
            while not stop.is_set():
                samples.append(self._read())
                stop.wait(0.02)
        th = threading.Thread(target=loop, daemon=True)
        th.start()
        try:
            out = fn()
        finally:
            stop.set()
            th.join()
        samples = samples[len(samples) // 4:]                # the first quarter: clock and power still ramping
        med = lambda xs: (sorted(xs)[len(xs) // 2] if xs else None)
        return out, med([m for m, _ in samples if m is not None]), med([w for _, w in samples if w is not None])


def power_probe(torch, B, W, timer):
    """The dominant product (8192 x 4096 x 4096, bf16, plain epilogue) on operands of different bit activity:
    the instruction stream is identical, only the data differs.  What the times show is how far the chip's
    power management, not the kernel's schedule, sets the rate on data that looks like a training step's;
    the shader clock and board power the driver reports while each loop runs are listed beside them."""
    M, N, K = 8192, 4096, 4096
    bf = torch.bfloat16
    rng = np.random.default_rng(190800213)
    out = torch.empty(M, N, dtype=bf, device="cuda")
    res = {}
    sampler = _SysfsSampler()
    kinds = {"zeros": lambda s: np.zeros(s, np.float32), "ones": lambda s: np.ones(s, np.float32),
             "small integers in [-3, 3]": lambda s: rng.integers(-3, 4, size=s).astype(np.float32),
             "standard normal": lambda s: rng.standard_normal(s, dtype=np.float32)}
    for rep in range(2):
        for kind, gen in kinds.items():
            a = B.cast(torch.from_numpy(gen((M, K))).cuda(), bf)
            wt = B.cast(torch.from_numpy(gen((N, K))).cuda(), bf)
            s, mhz, watts = sampler.run(lambda: timer.time(lambda: B.gemm(a, wt.t(), out), 2000, 5))   # about half a second
            r = res.setdefault(kind, {"us": [], "TFLOP/s": [], "sclk_MHz": [], "board_W": []})
            r["us"].append(round(s * 1e6, 1)); r["TFLOP/s"].append(round(2.0 * M * N * K / s / 1e12, 1))
            r["sclk_MHz"].append(mhz); r["board_W"].append(None if watts is None else round(watts))
            log("  power probe  %-28s %7.1f us  %7.1f TFLOP/s   sclk %s MHz   board %s W" % (
                kind, s * 1e6, 2.0 * M * N * K / s / 1e12, mhz, None if watts is None else round(watts)))
    return res


def cpu_baseline(W, rows=(32, 96)):
    """The CPU oracle, as it stands, on a bounded sample of the headline workload.  A full step would
    take the host about half an hour, so the figure is an EXTRAPOLATION and says so: the oracle's
    mixed-precision step (forward + backward + SGD through the full-width network) is timed on two
    small batches, the times are split into a part per batch row and a part that does not depend on
    the batch (rounding the working copies of 54 M weights, the SGD update), and the step at 8192
    rows is the fixed part once plus 8192 times the per-row part."""
    from oracle import oracle as O
    from oracle import steps as OS
    w = W.config5(n_batches=1)
    times = []
    for r in rows:
        x = W.bf16_exact(w.xs[0][:r])
        t0 = time.perf_counter()
        OS.mlp_step(w.params, x, w.ts[0][:r], np.float32(w.lr), w.act, lowp=True)
        times.append(time.perf_counter() - t0)
    per_row = (times[1] - times[0]) / (rows[1] - rows[0])
    fixed = max(0.0, times[0] - per_row * rows[0])
    full = fixed + per_row * w.batch
    return {"value": 1.0 / full, "unit": "steps/s", "cores": O.num_threads(), "kind": "oracle", "extrapolated": True,
            "rows_timed": list(rows), "seconds_timed": [round(t, 2) for t in times],
            "fit": {"fixed_s": round(fixed, 3), "per_row_s": round(per_row, 4), "batch": w.batch, "step_s": round(full, 1)},
            "sample": "oracle mixed-precision step (fp64 arithmetic, bf16 storage rounding) of the full 4096-4096-4096-4096-1000 "
                      "network timed at %d and %d of the %d batch rows (%.1f s and %.1f s); extrapolated linearly in the rows "
                      "to one full step = %.0f s" % (rows[0], rows[1], w.batch, times[0], times[1], full)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--repeats", type=int, default=5,
                    help="timed regions of --steps steps each for the headline workload; the median region is reported")
    ap.add_argument("--quick", action="store_true", help="headline workload only, fewer repetitions of the rest")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--workloads", default="1,2,3,4,tape",
                    help="which of the secondary workloads to run (comma list; `tape` = the steps driven by the define-by-run tape)")
    ap.add_argument("--separate-update", action="store_true",
                    help="headline workload: write the weight gradients and update in a separate SGD launch "
                         "instead of updating in the epilogue of the weight-gradient products (about 1 %% slower)")
    ap.add_argument("--traffic-driver", nargs="?", const="gemm", choices=["gemm", "array"],
                    help="run only a calibration copy + the dominant GEMM launch (gemm) or the array microbenchmark's "
                         "kernels (array), for rocprofv3 --pmc, and exit")
    ap.add_argument("--power-probe", action="store_true",
                    help="run only the dominant product on operands of different bit activity and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1908_00213_amd import binding as B, steps as steps_mod, workloads as W
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.lib()
    torch.cuda.set_device(0)
    timer = Timer(torch)
    extra = {}
    if args.traffic_driver:
        traffic_driver(torch, B, W, args.traffic_driver)
        return
    if args.power_probe:
        print(json.dumps({"power_probe": power_probe(torch, B, W, timer)}))
        return

    # ---- headline: workload 5, wide MLP, bf16 storage / fp32 accumulate
    log("workload 5: wide MLP 4096-4096-4096-4096-1000, GELU, batch 8192, bf16/fp32-accumulate")
    w5 = W.config5(n_batches=4)
    torch.cuda.synchronize()
    r5 = bench_mlp(torch, B, steps_mod, w5, True, timer, args.steps, args.warmup, probe=True,
                   fused_update=not args.separate_update, repeats=args.repeats)
    torch.cuda.synchronize()
    log("  %.3f ms/step (median of %d regions of %d steps: %s)  %.1f steps/s  %.1f TFLOP/s whole step; "
        "GEMMs (separate instrumented pass) %.3f ms/step = %.1f TFLOP/s" % (
        r5["ms_per_step"], args.repeats, args.steps, r5.get("ms_per_step_regions"), r5["steps_per_s"], r5["TFLOP/s"],
        r5["gemm_seconds_per_step"] * 1e3, r5["gemm_flops_per_step"] / r5["gemm_seconds_per_step"] / 1e12))
    # dominant kernel: the 256x256-tile eight-wave bf16 GEMM, forward layout (both operands unit-stride along K)
    dom = [c for c in r5["gemm_calls"] if c["call"] in ("fwd0", "fwd1", "fwd2")]
    # a bracket of two events reads `event_pair_empty_us` more than the kernel between them takes (what two events
    # with nothing between them read); the launch duration is the bracket minus that, which is also what the
    # profiler's kernel trace shows for these launches
    dom_bracket_s = sum(c["us"] for c in dom) * 1e-6 / len(dom)
    dom_s = dom_bracket_s - r5["event_pair_empty_us"] * 1e-6
    dom_flops = 2.0 * dom[0]["M"] * dom[0]["N"] * dom[0]["K"]
    roofline = {"bound": "mfma", "kernel": "gemm_kernel_w8<A and B unit-stride along K> (bf16, 256x256 tile, eight waves, direct global-to-LDS copies; "
                                           "hidden-layer forward x @ W.T + b with GELU, M=8192 N=4096 K=4096)",
                "achieved": dom_flops / dom_s / 1e12, "peak": MFMA_PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                "frac": dom_flops / dom_s / 1e12 / MFMA_PEAK_TFLOPS["bf16"], "traffic": DOMINANT_KERNEL_TRAFFIC_BYTES,
                "avg_launch_us": dom_s * 1e6, "avg_bracket_us": dom_bracket_s * 1e6, "event_pair_empty_us": r5["event_pair_empty_us"],
                "flops_per_launch": dom_flops,
                "all_gemms_achieved": r5["gemm_flops_per_step"] / r5["gemm_seconds_per_step"] / 1e12}
    extra["cfg5_wide_mlp_bf16"] = r5
    del w5
    torch.cuda.empty_cache()

    sel = set() if args.quick else set(x for x in args.workloads.split(",") if x)
    if "2" in sel:
        log("workload 2: array primitives (8192 x 8192)")
        extra["cfg2_array"] = bench_array(torch, B, W, timer, False)
    if "3" in sel:
        log("workload 3: MLP 784-1000-1000-10, batch 1024")
        w3 = W.config3()
        for lowp in (False, True):
            for graph in (False, True):
                r = bench_mlp(torch, B, steps_mod, w3, lowp, timer, 100, 10, graph=graph, probe=not graph)
                tag = ("bf16" if lowp else "f32") + ("_hipgraph" if graph else "")
                extra["cfg3_mlp_%s" % tag] = r
                log("  %s: %.1f us/step  %.0f steps/s  %.2f TFLOP/s  (%d launches/step)" % (
                    tag, r["ms_per_step"] * 1e3, r["steps_per_s"], r["TFLOP/s"], r["launch_calls_per_step"]))
                if "gemm_calls" in r:
                    log("    products (us, TFLOP/s; net of the event bracket): " + "  ".join(
                        "%s %.1f %.0f" % (c["call"], c["us_net"], c["TFLOP/s_net"]) for c in r["gemm_calls"]))
    if "1" in sel:
        log("workload 1: tiny MLP 784-100-100-10, batch 32")
        for graph in (False, True):
            r = bench_mlp(torch, B, steps_mod, W.config1(), False, timer, 200, 20, graph=graph)
            extra["cfg1_tiny_mlp_f32" + ("_hipgraph" if graph else "")] = r
            log("  %s%.1f us/step  %.0f steps/s" % ("HIP graph: " if graph else "", r["ms_per_step"] * 1e3, r["steps_per_s"]))
    if "4" in sel:
        log("workload 4: LSTM language model step (vocab 10000, 650 hidden, batch 128, BPTT 35), fp32")
        w4 = W.config4()
        for graph in (False, True):
            r = bench_lstm(torch, B, steps_mod, w4, timer, 20, 3, graph=graph)
            extra["cfg4_lstm_lm_f32" + ("_hipgraph" if graph else "")] = r
            log("  %s%.3f ms/step  %.1f steps/s  %.0f tokens/s  %.1f TFLOP/s (%.1f%% of fp32 MFMA peak; %d launches/step)" % (
                "HIP graph: " if graph else "", r["ms_per_step"], r["steps_per_s"], r["tokens_per_s"], r["TFLOP/s"],
                100 * r["frac_mfma_peak_f32"], r["launch_calls_per_step"]))
        r = bench_lstm(torch, B, steps_mod, w4, timer, 20, 3, lowp=True)
        r.pop("frac_mfma_peak_f32")
        extra["cfg4_lstm_lm_bf16"] = r
        log("  mixed precision (bf16 storage, fp32 accumulate): %.3f ms/step  %.1f steps/s  %.0f tokens/s  %.1f TFLOP/s" % (
            r["ms_per_step"], r["steps_per_s"], r["tokens_per_s"], r["TFLOP/s"]))

    if "tape" in sel:
        log("define-by-run tape driving the same steps")
        extra["tape"] = bench_tape(torch, W, timer, False)
        for k, r in extra["tape"].items():
            log("  %s: %.3f ms/step  %.1f steps/s" % (k, r["ms_per_step"], r["steps_per_s"]))

    cpu = None
    if not args.no_cpu:
        log("cpu baseline: oracle on a bounded sample of workload 5")
        cpu = cpu_baseline(W)
        log("  %.3g steps/s on %d host threads (%s)" % (cpu["value"], cpu["cores"], cpu["sample"]))

    line = {
        "metric": "train steps/s", "value": r5["steps_per_s"], "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": r5["ms_per_step"], "repeats": args.repeats,
        "ms_per_step_regions": r5.get("ms_per_step_regions"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "cfg5: wide MLP 4096-4096-4096-4096-1000, GELU, softmax cross-entropy, batch 8192, "
                               "bf16 storage / fp32 accumulate / fp32 master weights, forward+backward+SGD "
                               "(weight update applied in the epilogue of the weight-gradient products)",
                   "global_batch": 8192, "parallelism": "single GPU"},
        "roofline": roofline, "cpu_baseline": cpu, "workloads": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
