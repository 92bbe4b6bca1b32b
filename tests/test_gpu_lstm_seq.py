"""GPU parity of the whole-sequence recurrent forward (one launch for all time steps) against the CPU oracle,
step by step from the GPU's own previous state, and against the chain of per-step calls."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_1908_00213_amd import binding as B
from tests.util import TOL_BF16, TOL_EW, TOL_SUM, bf16r, check, dev, empty, host, ws

pytestmark = pytest.mark.gpu

CASES = [(128, 672, 35, "f32"), (128, 672, 35, "bf16"),      # the language-model workload: 84 x 2 workgroups
         (70, 40, 4, "f32"), (5, 8, 3, "f32"),               # ragged batch block, one partial chunk
         (33, 144, 6, "bf16"), (200, 256, 3, "f32"),         # four batch blocks, two chunks
         (64, 1536, 2, "bf16"), (128, 768, 2, "f32"),        # the widest rows: Ut in registers, five stages, six chunks
         (64, 640, 3, "f32"),                                # ... five chunks
         (64, 512, 3, "f32"), (40, 352, 3, "f32")]           # four chunks through three stages (one reused); three, the last one partial


def inputs(Bn, H, T, dt, seed):
    rng = np.random.default_rng(seed)
    q = (lambda a: a) if dt == "f32" else bf16r
    u = lambda shape, lo, hi: rng.uniform(lo, hi, size=shape).astype(np.float32)
    s = 1.5 / np.sqrt(H)
    return u((T * Bn, 4 * H), -2, 2), u((4 * H,), -1, 1), q(u((Bn, H), -1, 1)), u((Bn, H), -2, 2), q(u((H, 4 * H), -s, s))


def run(zx, bias, h0, c0, U, T, dt, Hs=None, Cs=None, gates=None, work=None):
    Bn, H = h0.shape
    Hs = empty(((T + 1) * Bn, H), dt) if Hs is None else Hs
    Cs = empty(((T + 1) * Bn, H)) if Cs is None else Cs
    gates = empty((T * Bn, 4 * H)) if gates is None else gates
    work = ws(B.lstm_seq_workspace_bytes(Bn)) if work is None else work
    Hs[:Bn].copy_(dev(h0, dt))
    Cs[:Bn].copy_(dev(c0))
    print("lstm_seq_fwd B=%d H=%d T=%d %s" % (Bn, H, T, dt), flush=True)
    B.lstm_seq_fwd(dev(zx), dev(np.ascontiguousarray(U.T), dt), None if bias is None else dev(bias), Hs, Cs, gates, T, work)
    torch.cuda.synchronize()
    return Hs, Cs, gates, work


def status_word(work):
    return int(work[:4].view(torch.int32).item())


def check_against_oracle(zx, bias, U, T, dt, Hs, Cs, gates):
    """Every step from the state the GPU itself left for it: one product and one cell of error per check."""
    Bn, H = Hs.shape[0] // (T + 1), Hs.shape[1]
    Hh, Ch, Gh = host(Hs), host(Cs), host(gates)
    tol = TOL_SUM if dt == "f32" else TOL_BF16
    for t in range(T):
        hp, cp, z0 = Hh[t * Bn:(t + 1) * Bn], Ch[t * Bn:(t + 1) * Bn], zx[t * Bn:(t + 1) * Bn]
        rc, rh, rg = O.lstm_fwd(O.gemm(hp, U, z0, 1.0, 1.0), bias, cp)
        Sz = O.gemm(np.abs(hp), np.abs(U)) + np.abs(z0) + (0 if bias is None else np.abs(bias))
        Sg = np.concatenate([0.25 * Sz[:, :H], 0.25 * Sz[:, H:2 * H], Sz[:, 2 * H:3 * H], 0.25 * Sz[:, 3 * H:]], axis=1)
        check(Gh[t * Bn:(t + 1) * Bn], rg, TOL_SUM, Sg + 1e-1, "gates of step %d" % t)
        Sc = np.abs(rg[:, H:2 * H] * cp) + np.abs(rg[:, :H] * rg[:, 2 * H:3 * H]) + Sg[:, :H] + Sg[:, H:2 * H] * np.abs(cp) + Sg[:, 2 * H:3 * H]
        check(Ch[(t + 1) * Bn:(t + 2) * Bn], rc, TOL_SUM, Sc, "c of step %d" % t)
        check(Hh[(t + 1) * Bn:(t + 2) * Bn], rh, tol, Sc + Sg[:, 3 * H:], "h of step %d" % t)


@pytest.mark.parametrize("Bn,H,T,dt", CASES)
def test_whole_sequence_forward(Bn, H, T, dt):
    zx, bias, h0, c0, U = inputs(Bn, H, T, dt, 7)
    Hs, Cs, gates, work = run(zx, bias, h0, c0, U, T, dt)
    assert status_word(work) == 0
    check_against_oracle(zx, bias, U, T, dt, Hs, Cs, gates)
    assert np.array_equal(host(Hs[:Bn]), h0.astype(np.float64)) and np.array_equal(host(Cs[:Bn]), c0.astype(np.float64))
    # the per-step calls on the same operands walk the same trajectory (another order of the fp32 sums)
    if H % 32 == 0:
        H2, C2, G2 = empty(((T + 1) * Bn, H), dt), empty(((T + 1) * Bn, H)), empty((T * Bn, 4 * H))
        H2[:Bn].copy_(dev(h0, dt)); C2[:Bn].copy_(dev(c0))
        B.lstm_step_fwd_seq(dev(zx), H2, dev(np.ascontiguousarray(U.T), dt), dev(bias), C2, G2, T)
        loose = (1e-4 if dt == "f32" else 4e-2) * max(1, T // 4)
        check(host(Cs), host(C2), loose, 1.0, "c whole sequence vs per step")
        check(host(Hs), host(H2), loose, 1.0, "h whole sequence vs per step")
    # the same buffers again with other inputs: nothing of the first call may be read back from a cache
    zx, bias, h0, c0, U = inputs(Bn, H, T, dt, 8)
    run(zx, None, h0, c0, U, T, dt, Hs, Cs, gates, work)
    assert status_word(work) == 0
    check_against_oracle(zx, None, U, T, dt, Hs, Cs, gates)


def test_whole_sequence_without_gates_and_pitched_buffers():
    Bn, H, T = 40, 64, 3
    zx, bias, h0, c0, U = inputs(Bn, H, T, "f32", 9)
    wide_z = dev(np.concatenate([zx, zx], axis=1))[:, :4 * H]
    wide_h = torch.zeros((T + 1) * Bn, 2 * H, device="cuda")[:, :H]
    Cs = empty(((T + 1) * Bn, H))
    wide_h[:Bn].copy_(dev(h0)); Cs[:Bn].copy_(dev(c0))
    work = ws(B.lstm_seq_workspace_bytes(Bn))
    B.lstm_seq_fwd(wide_z, dev(np.ascontiguousarray(U.T)), dev(bias), wide_h, Cs, None, T, work)
    Hs, C2, gates, _ = run(zx, bias, h0, c0, U, T, "f32")
    assert torch.equal(wide_h, Hs) and torch.equal(Cs, C2)


def test_whole_sequence_refusals():
    def call(Bn, H, T, dt="f32", work=None, hs_rows=None):
        tdt = torch.float32 if dt == "f32" else torch.bfloat16
        z = torch.zeros(T * Bn, 4 * H, device="cuda")
        Hs = torch.zeros((T + 1) * Bn if hs_rows is None else hs_rows, H, dtype=tdt, device="cuda")
        Cs = torch.zeros((T + 1) * Bn, H, device="cuda")
        B.lstm_seq_fwd(z, torch.zeros(4 * H, H, dtype=tdt, device="cuda"), None, Hs, Cs, None, T,
                       ws(B.lstm_seq_workspace_bytes(Bn)) if work is None else work)
    for args, status in [((4, 44, 2), -4),                     # hidden width not a multiple of 8
                         ((4, 40, 2, "bf16"), -4),             # ... of 16 for bfloat16
                         ((4, 776, 2), -4),                    # rows wider than the resident slice holds
                         ((256, 768, 2), -4),                  # 96 x 4 workgroups: more than compute units
                         ((4, 64, 2, "f32", None, 8), -4)]:    # Hs with too few rows
        with pytest.raises(B.ChnError) as e:
            call(*args)
        assert e.value.status == status, args
    with pytest.raises(B.ChnError):
        call(4, 64, 2, work=torch.empty(16, dtype=torch.uint8, device="cuda"))
    call(4, 64, 0)                                              # no steps: nothing to do
    torch.cuda.synchronize()


def test_a_wait_that_runs_out_ends_the_kernel_and_raises_the_status_word():
    """Spin limit 0: the first wait (before step 1) gives up without looking, in every workgroup.  The kernel
    ends after its first step with the status word set; the next call, with the default limit, is complete."""
    Bn, H, T, dt = 128, 672, 35, "f32"
    zx, bias, h0, c0, U = inputs(Bn, H, T, dt, 11)
    B.lstm_seq_spin_limit(0)
    try:
        Hs, Cs, gates, work = run(zx, bias, h0, c0, U, T, dt)
    finally:
        B.lstm_seq_spin_limit(1 << 20)
    assert status_word(work) == 1
    Hs, Cs, gates, work = run(zx, bias, h0, c0, U, T, dt, Hs, Cs, gates, work)
    assert status_word(work) == 0
    check_against_oracle(zx, bias, U, T, dt, Hs, Cs, gates)


# ------------------------------------------------------------------------------------ backward through time
BWD_CASES = [(128, 672, 35, "f32"), (128, 672, 35, "bf16"),  # the language-model workload: 42 x 4 workgroups
             (40, 48, 4, "f32"), (5, 16, 3, "f32"),          # ragged batch block, a partial 32-unit tile; one workgroup
             (33, 144, 5, "bf16"), (200, 256, 3, "f32"),
             (40, 96, 4, "bf16"), (250, 512, 2, "bf16"),     # ragged batch block; 32 x 8 = 256 workgroups, every compute unit
             (96, 768, 2, "f32"), (32, 1536, 2, "bf16")]     # the widest U the registers hold (bf16: two batches of partial sums)


def bwd_inputs(Bn, H, T, dt, seed):
    rng = np.random.default_rng(seed)
    q = (lambda a: a) if dt == "f32" else bf16r
    u = lambda shape, lo, hi: rng.uniform(lo, hi, size=shape).astype(np.float32)
    s = 1.5 / np.sqrt(H)
    gates = np.concatenate([u((T * Bn, 2 * H), 0.05, 0.95), u((T * Bn, H), -0.95, 0.95), u((T * Bn, H), 0.05, 0.95)], axis=1)
    return q(u((H, 4 * H), -s, s)), q(u((T * Bn, H), -1, 1)), gates, u(((T + 1) * Bn, H), -1.5, 1.5), u((Bn, H), -1, 1)


def run_bwd(U, dh_in, gates, Cs, dc_last, T, dt, bufs=None):
    Bn, H = Cs.shape[0] // (T + 1), Cs.shape[1]
    dHs, dZ, dc0, work = bufs or (empty((T * Bn, H), dt), empty((T * Bn, 4 * H), dt), empty((Bn, H)),
                                  ws(B.lstm_seq_bwd_workspace_bytes(Bn, H)))
    dHs.copy_(dev(dh_in, dt))
    print("lstm_seq_bwd B=%d H=%d T=%d %s" % (Bn, H, T, dt), flush=True)
    B.lstm_seq_bwd(dev(U, dt), dHs, dev(gates), dev(Cs), None if dc_last is None else dev(dc_last), dZ, dc0, T, work)
    torch.cuda.synchronize()
    return dHs, dZ, dc0, work


def check_bwd_against_oracle(U, dh_in, gates, Cs, dc_last, T, dt, dHs, dZ, dc0):
    """Last step first; the product of every step from the dz the GPU itself stored for the step after it, the
    cell from the dh the GPU stored; only dc is carried along by the oracle."""
    Bn, H = Cs.shape[0] // (T + 1), Cs.shape[1]
    dH, dz_gpu = host(dHs), host(dZ)
    tol = TOL_SUM if dt == "f32" else TOL_BF16
    dc = None if dc_last is None else dc_last.astype(np.float64)
    for t in range(T - 1, -1, -1):
        sl = slice(t * Bn, (t + 1) * Bn)
        if t == T - 1:
            assert np.array_equal(dH[sl], dh_in[sl].astype(np.float64))
        else:
            nx = slice((t + 1) * Bn, (t + 2) * Bn)
            check(dH[sl], O.gemm(dz_gpu[nx], U.T, dh_in[sl], 1.0, 1.0), tol, O.gemm(np.abs(dz_gpu[nx]), np.abs(U.T)) + np.abs(dh_in[sl]), "dh total %d" % t)
        cp, c = Cs[sl].astype(np.float64), Cs[(t + 1) * Bn:(t + 2) * Bn].astype(np.float64)
        rdz, dc = O.lstm_bwd(gates[sl], cp, c, dH[sl], dc)
        Sdc = np.abs(dc) + np.abs(dH[sl]) + 1e-3
        Sdz = np.concatenate([Sdc, Sdc * (1 + np.abs(cp)), Sdc, np.abs(dH[sl])], axis=1)
        check(dz_gpu[sl], rdz, TOL_EW * 10 * (T - t) if dt == "f32" else TOL_BF16, Sdz, "dz %d" % t)
    check(host(dc0), dc, TOL_EW * 10 * T, 1.0, "dc0")


@pytest.mark.parametrize("Bn,H,T,dt", BWD_CASES)
def test_whole_sequence_backward(Bn, H, T, dt):
    U, dh_in, gates, Cs, dc_last = bwd_inputs(Bn, H, T, dt, 21)
    dHs, dZ, dc0, work = run_bwd(U, dh_in, gates, Cs, dc_last, T, dt)
    assert status_word(work) == 0
    check_bwd_against_oracle(U, dh_in, gates, Cs, dc_last, T, dt, dHs, dZ, dc0)
    if H % 32 == 0:      # the chain of per-step calls walks the same trajectory
        d2, z2, dcs = dev(dh_in, dt), empty((T * Bn, 4 * H), dt), [empty((Bn, H)), empty((Bn, H))]
        B.lstm_step_bwd_seq(z2, dev(U, dt), d2, dev(gates), dev(Cs), dev(dc_last), dcs, T)
        loose = (1e-4 if dt == "f32" else 4e-2) * max(1, T // 4)
        check(host(dZ), host(z2), loose, 1.0, "dz whole sequence vs per step")
        check(host(dc0), host(dcs[0]), loose, 1.0, "dc0 whole sequence vs per step")
    # the same buffers and workspace again with other values, no gradient into the last cell state
    U, dh_in, gates, Cs, _ = bwd_inputs(Bn, H, T, dt, 22)
    run_bwd(U, dh_in, gates, Cs, None, T, dt, (dHs, dZ, dc0, work))
    assert status_word(work) == 0
    check_bwd_against_oracle(U, dh_in, gates, Cs, None, T, dt, dHs, dZ, dc0)


def test_whole_sequence_backward_refusals_and_give_up():
    def call(Bn, H, T, dt="f32", work=None):
        tdt = torch.float32 if dt == "f32" else torch.bfloat16
        z = lambda *s: torch.zeros(*s, device="cuda")
        B.lstm_seq_bwd(torch.zeros(H, 4 * H, dtype=tdt, device="cuda"), torch.zeros(T * Bn, H, dtype=tdt, device="cuda"), z(T * Bn, 4 * H),
                       z((T + 1) * Bn, H), None, torch.zeros(T * Bn, 4 * H, dtype=tdt, device="cuda"), z(Bn, H), T,
                       ws(B.lstm_seq_bwd_workspace_bytes(Bn, H)) if work is None else work)
    for args in [(4, 40, 2), (4, 784, 2), (4, 1552, 2, "bf16"), (288, 512, 2)]:      # width not a multiple of 16; too wide; 9 x 32 workgroups
        with pytest.raises(B.ChnError) as e:
            call(*args)
        assert e.value.status == -4, args
        assert not B.lstm_seq_bwd_supported(args[0], args[1], torch.float32 if len(args) < 4 else torch.bfloat16)
    with pytest.raises(B.ChnError):
        call(4, 64, 2, work=torch.empty(4096, dtype=torch.uint8, device="cuda"))
    call(4, 64, 0)
    torch.cuda.synchronize()
    # spin limit 0: the first exchange gives up without looking; the kernel ends, the status word says so
    Bn, H, T, dt = 128, 672, 35, "f32"
    U, dh_in, gates, Cs, dc_last = bwd_inputs(Bn, H, T, dt, 23)
    B.lstm_seq_spin_limit(0)
    try:
        bufs = run_bwd(U, dh_in, gates, Cs, dc_last, T, dt)
    finally:
        B.lstm_seq_spin_limit(1 << 20)
    assert status_word(bufs[3]) == 1
    dHs, dZ, dc0, work = run_bwd(U, dh_in, gates, Cs, dc_last, T, dt, bufs)
    assert status_word(work) == 0
    check_bwd_against_oracle(U, dh_in, gates, Cs, dc_last, T, dt, dHs, dZ, dc0)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_whole_sequence_kernels_are_reproducible_bit_for_bit(dt):
    """Every sum is taken in a fixed order (partial tiles in wave order, partial dh in sender order): two runs of
    the same launch agree in every bit, whatever order the workgroups arrive in."""
    Bn, H, T = 128, 672, 35
    zx, bias, h0, c0, U = inputs(Bn, H, T, dt, 31)
    first = [t.clone() for t in run(zx, bias, h0, c0, U, T, dt)[:3]]
    for _ in range(2):
        again = run(zx, bias, h0, c0, U, T, dt)[:3]
        assert all(torch.equal(a, b) for a, b in zip(first, again))
    Ub, dh_in, gates, Cs, dc_last = bwd_inputs(Bn, H, T, dt, 32)
    first = [t.clone() for t in run_bwd(Ub, dh_in, gates, Cs, dc_last, T, dt)[:3]]
    for _ in range(2):
        again = run_bwd(Ub, dh_in, gates, Cs, dc_last, T, dt)[:3]
        assert all(torch.equal(a, b) for a, b in zip(first, again))
