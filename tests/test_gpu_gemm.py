"""GPU parity of chn_gemm against the CPU oracle: all four operand layouts, both dtypes, the three
tile sizes, ragged edges in M, N and K, misaligned leading dimensions, alpha/beta and every epilogue.
Exact small-integer inputs must match bit for bit (fp32 accumulation of integers below 2^24 is exact
in any order)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_1908_00213_amd import binding as B
from tests.util import TOL_BF16, TOL_SUM, bf16r, check, dev, empty, host, ws

pytestmark = pytest.mark.gpu
RNG = np.random.default_rng(213_1908)


def rnd(shape, dt="f32", scale=1.0):
    a = (RNG.standard_normal(size=shape) * scale).astype(np.float32)
    return bf16r(a) if dt == "bf16" else a


def operands(M, N, K, layout, dt, gen=rnd):
    """Returns (A_np, B_np, A_dev, B_dev): A (M,K), B (K,N) views with the requested unit strides.
    layout[0]: 'n' A row-major (unit stride along K), 't' A stored transposed (unit stride along M);
    layout[1]: 'n' B row-major (unit stride along N), 't' B stored transposed (unit stride along K)."""
    if layout[0] == "n":
        a = gen((M, K), dt); A_np, A_dev = a, dev(a, dt)
    else:
        a = gen((K, M), dt); A_np, A_dev = a.T, dev(a, dt).t()
    if layout[1] == "n":
        b = gen((K, N), dt); B_np, B_dev = b, dev(b, dt)
    else:
        b = gen((N, K), dt); B_np, B_dev = b.T, dev(b, dt).t()
    return A_np, B_np, A_dev, B_dev


SHAPES = [(64, 64, 64), (100, 70, 50), (257, 129, 100), (130, 300, 650), (32, 10, 100), (10, 1000, 33),
          (600, 520, 96), (1, 1, 1), (5, 7, 3), (200, 64, 10), (72, 136, 6)]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("layout", ["nt", "nn", "tn", "tt"])
@pytest.mark.parametrize("shape", SHAPES)
def test_gemm_layouts(dt, layout, shape):
    M, N, K = shape
    A, Bm, Ad, Bd = operands(M, N, K, layout, dt)
    out = B.gemm(Ad, Bd, empty((M, N)))
    ref = O.gemm(A, Bm)
    S = O.gemm(np.abs(A), np.abs(Bm))
    check(host(out), ref, TOL_BF16 if dt == "bf16" else TOL_SUM, S, "gemm %s %s" % (layout, dt))
    if dt == "bf16":
        # bf16 inputs are exact, the accumulator is fp32: the fp32 result meets the fp32 bar too
        check(host(out), ref, TOL_SUM, S, "gemm bf16-in fp32-out")
        outb = B.gemm(Ad, Bd, empty((M, N), "bf16"))
        check(host(outb), ref, TOL_BF16, S, "gemm bf16 out")


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(10, 1000, 1024), (10, 37, 200), (77, 130, 96), (203, 5, 64), (1, 3, 40)])
def test_gemm_transposed_operands_with_padded_rows(dt, shape):
    """Operands whose unit stride runs along M / N, with rows padded to 16 bytes and an extent that is not
    a multiple of the load piece: the last piece of every row also brings the padding (NaN here), which
    must reach nothing that is stored.  (The weight-gradient product of a 10-class layer has this shape.)"""
    M, N, K = shape
    epr = 8 if dt == "bf16" else 4
    pm, pn = (M + epr - 1) // epr * epr, (N + epr - 1) // epr * epr + epr
    a, b = rnd((K, M), dt), rnd((K, N), dt)
    abuf = np.full((K, pm), np.nan, np.float32); abuf[:, :M] = a
    bbuf = np.full((K, pn), np.nan, np.float32); bbuf[:, :N] = b
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    Ad = torch.from_numpy(abuf).cuda().to(tdt)[:, :M].t()      # (NaN and bf16-exact values survive the cast)
    Bd = torch.from_numpy(bbuf).cuda().to(tdt)[:, :N]
    ref, S = O.gemm(a.T, b), O.gemm(np.abs(a.T), np.abs(b))
    tol = TOL_BF16 if dt == "bf16" else TOL_SUM
    for tile, splits in ((-1, -1), (-1, 2), (1, -1), (2, -1), (2, 2)):      # also on the larger register-staged tiles
        B.gemm_plan_override(tile, splits, 0)
        try:
            need = B.gemm_workspace_bytes(Ad, Bd, empty((M, N)))
            out = B.gemm(Ad, Bd, empty((M, N)), ws=ws(need) if need else None)
        finally:
            B.gemm_plan_override()
        check(host(out), ref, tol, S, "padded transposed operands %s %s tile %d splits %d" % (shape, dt, tile, splits))
    # the same buffer as the K-contiguous operand of another product (the input-gradient layout): along K
    # no piece may overhang, or the padding would be summed
    w = rnd((M, 24), dt)
    out = B.gemm(Ad.t(), dev(w, dt), empty((K, 24)))
    check(host(out), O.gemm(a, w), tol, O.gemm(np.abs(a), np.abs(w)), "padded rows along K %s %s" % (shape, dt))


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("layout", ["nt", "nn", "tn"])
@pytest.mark.parametrize("shape", [(3700, 3590, 130), (1500, 1400, 136), (300, 200, 4100)])
def test_gemm_big_tiles_exact_integers(dt, layout, shape):
    # sizes that select the 256x256 and 128x128 macro tiles, with ragged edges in every dimension
    M, N, K = shape
    gen = lambda s, d: RNG.integers(-3, 4, size=s).astype(np.float32)
    A, Bm, Ad, Bd = operands(M, N, K, layout, dt, gen)
    out = host(B.gemm(Ad, Bd, empty((M, N))))
    ref = A.astype(np.float64) @ Bm.astype(np.float64)       # exact in fp64; the oracle is pinned to it
    rows = RNG.integers(0, M, 24)
    assert np.array_equal(O.gemm(A[rows], Bm), ref[rows])
    assert np.array_equal(out, ref)


@pytest.fixture(params=["four waves", "eight waves"])
def direct_kernel(request):
    """Runs a test of the 256x256 direct-copy path once per kernel that can take a bf16 product there
    (fp32 products have the four-wave kernel only: the other parameter value then changes nothing)."""
    B.gemm_plan_override(direct_copy=2 if request.param == "four waves" else 3)
    yield request.param
    B.gemm_plan_override()


# The planner takes the 256x256 tile only when K is long enough to pay for its fixed cost; the short-K
# cases (one, two, three tile steps: where a pipeline's prologue and tail go wrong) force the tile
# through the library's test hook chn_gemm_plan_override.
DIRECT_COPY_CASES = [("bf16", s) for s in [(3704, 3592, 1024), (3720, 3592, 1000), (3704, 3592, 1088)]] + \
                    [("f32", s) for s in [(3704, 3592, 1000), (3720, 3592, 1024), (3704, 3592, 1056)]]
DIRECT_COPY_SHORT_K = [("bf16", s) for s in [(3704, 3592, 192), (3704, 3592, 64), (3720, 3592, 128), (3704, 3592, 200), (520, 264, 448)]] + \
                      [("f32", s) for s in [(3704, 3592, 32), (3720, 3592, 64), (1032, 520, 100)]]


def direct_copy_case(dt, layout, shape):
    # every unit-stride extent a multiple of 16 bytes: the 256x256 kernel that copies its operands
    # straight into LDS; odd and even numbers of tile steps, K with and without a ragged last step,
    # ragged last tiles in M and N; exact small integers, bit for bit
    M, N, K = shape
    gen = lambda s, d: RNG.integers(-3, 4, size=s).astype(np.float32)
    A, Bm, Ad, Bd = operands(M, N, K, layout, dt, gen)
    direct = not (dt == "f32" and layout == "tn")     # fp32 with both operands stored along M/N: register-staged
    assert B.gemm_plan(Ad, Bd, empty((M, N)))[:2] == (2, direct), (dt, layout, shape)
    out = host(B.gemm(Ad, Bd, empty((M, N))))
    ref = A.astype(np.float64) @ Bm.astype(np.float64)
    rows = RNG.integers(0, M, 24)
    assert np.array_equal(O.gemm(A[rows], Bm), ref[rows])
    assert np.array_equal(out, ref), (dt, layout, shape)


@pytest.mark.parametrize("layout", ["nt", "nn", "tn"])
@pytest.mark.parametrize("dt,shape", DIRECT_COPY_CASES)
def test_gemm_big_tiles_direct_copy(dt, layout, shape, direct_kernel):
    if dt == "f32" and direct_kernel == "eight waves":
        pytest.skip("fp32 products have the four-wave kernel only")
    direct_copy_case(dt, layout, shape)


@pytest.mark.parametrize("waves", [2, 3])
def test_gemm_big_tiles_direct_copy_short_k_forced_tile(waves):
    B.gemm_plan_override(tile=2, direct_copy=waves)
    try:
        for dt, shape in DIRECT_COPY_SHORT_K:
            if dt == "f32" and waves == 3:
                continue
            for layout in ("nt", "nn", "tn"):
                print(dt, layout, shape, flush=True)
                direct_copy_case(dt, layout, shape)
    finally:
        B.gemm_plan_override()


def test_gemm_direct_copy_odd_k_both_transposed(direct_kernel):
    # with both operands stored along M / N, K itself needs no alignment for the direct-copy kernel
    M, N, K = 3720, 3592, 1003
    gen = lambda s, d: RNG.integers(-3, 4, size=s).astype(np.float32)
    A, Bm, Ad, Bd = operands(M, N, K, "tn", "bf16", gen)
    assert B.gemm_plan(Ad, Bd, empty((M, N)))[:2] == (2, True)
    out = host(B.gemm(Ad, Bd, empty((M, N))))
    assert np.array_equal(out, A.astype(np.float64) @ Bm.astype(np.float64))


def test_gemm_plan_reports_the_direct_copy_kernel():
    M, N = 1024, 768
    for K, want in ((512, True), (2048, True), (4096, True)):        # bf16 products on the direct-copy path: eight waves
        _, _, Ad, Bd = operands(M, N, K, "nt", "bf16")
        B.gemm_plan_override(tile=2)
        try:
            assert B.gemm_plan(Ad, Bd, empty((M, N)))[:2] == (2, True)
            assert B.gemm_plan_eight_waves(Ad, Bd, empty((M, N))) == want
            B.gemm_plan_override(tile=2, direct_copy=2)
            assert not B.gemm_plan_eight_waves(Ad, Bd, empty((M, N)))
            B.gemm_plan_override(tile=2, direct_copy=3)
            assert B.gemm_plan_eight_waves(Ad, Bd, empty((M, N)))
        finally:
            B.gemm_plan_override()
    _, _, Ad, Bd = operands(M, N, 512, "nt", "f32")
    B.gemm_plan_override(tile=2, direct_copy=3)
    try:
        assert not B.gemm_plan_eight_waves(Ad, Bd, empty((M, N)))    # fp32: four waves only
    finally:
        B.gemm_plan_override()


def test_gemm_identity_and_ones():
    x = rnd((200, 96))
    assert np.array_equal(host(B.gemm(dev(x), dev(np.eye(96, dtype=np.float32)), empty((200, 96)))), x)
    o = host(B.gemm(dev(np.ones((70, 650), np.float32)), dev(np.ones((650, 90), np.float32)), empty((70, 90))))
    assert np.all(o == 650.0)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_gemm_alpha_beta_and_epilogues(dt):
    M, N, K = 150, 200, 90
    tol = TOL_BF16 if dt == "bf16" else TOL_SUM
    cdt = dt
    A, Bm, Ad, Bd = operands(M, N, K, "nt", dt)
    C0 = rnd((M, N), cdt)
    S = O.gemm(np.abs(A), np.abs(Bm))
    Cd = dev(C0, cdt)
    B.gemm(Ad, Bd, Cd, alpha=0.5, beta=-2.0)
    check(host(Cd), O.gemm(A, Bm, C0, 0.5, -2.0), tol, 0.5 * S + 2 * np.abs(C0), "alpha beta")
    bias = rnd((N,))
    v = O.elementwise("add", [O.gemm(A, Bm), bias])
    Sb = S + np.abs(bias)
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias", bias=dev(bias))
    check(host(out), v, tol, Sb, "bias")
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias_relu", bias=dev(bias))
    check(host(out), O.elementwise("relu", [v]), tol, Sb, "bias_relu")
    pre = empty((M, N), cdt)
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias_gelu", bias=dev(bias), preact_out=pre)
    check(host(pre), v, tol, Sb, "preact")
    check(host(out), O.elementwise("gelu", [v]), tol, Sb, "bias_gelu")
    out2 = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias_gelu", bias=dev(bias))
    assert torch.equal(out.view(torch.int16 if cdt == "bf16" else torch.int32), out2.view(torch.int16 if cdt == "bf16" else torch.int32))
    aux = rnd((M, N), cdt)
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="relu_bwd", aux=dev(aux, cdt))
    check(host(out), O.elementwise("relu_bwd", [O.gemm(A, Bm), aux]), tol, S, "relu_bwd")
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="gelu_bwd", aux=dev(aux, cdt))
    check(host(out), O.elementwise("gelu_bwd", [O.gemm(A, Bm), aux]), tol, S * 1.2, "gelu_bwd")
    # accumulate into a row block of a larger buffer (how the recurrent step adds h U to x W)
    big = rnd((3 * M, N))
    bd = dev(big)
    if dt == "f32":
        B.gemm(Ad, Bd, bd[M:2 * M], beta=1.0)
        want = big.astype(np.float64); want[M:2 * M] += O.gemm(A, Bm)
        check(host(bd), want, tol, np.concatenate([np.zeros((M, N)), S + np.abs(big[M:2 * M]), np.zeros((M, N))]), "beta=1 slice")


def test_gemm_misaligned_leading_dimensions():
    # K = 650 fp32: rows are 8-byte but not 16-byte aligned; K = 651: 4-byte only; bf16 K = 325: 2-byte
    for dt, K in (("f32", 650), ("f32", 651), ("bf16", 652), ("bf16", 325)):
        M, N = 140, 90
        for layout in ("nt", "nn", "tn"):
            A, Bm, Ad, Bd = operands(M, N, K, layout, dt)
            out = B.gemm(Ad, Bd, empty((M, N)))
            check(host(out), O.gemm(A, Bm), TOL_SUM, O.gemm(np.abs(A), np.abs(Bm)), "misaligned %s %d %s" % (dt, K, layout))
    # operands that are column slices of wider buffers (leading dimension > extent)
    a = rnd((100, 300)); b = rnd((80, 300))
    out = B.gemm(dev(a)[:, 4:204], dev(b)[:, 8:208].t(), empty((100, 80)))
    check(host(out), O.gemm(a[:, 4:204], b[:, 8:208].T), TOL_SUM, O.gemm(np.abs(a[:, 4:204]), np.abs(b[:, 8:208].T)), "sliced")
    # empty problems
    B.gemm(empty((0, 5)), empty((5, 7)), empty((0, 7)))
    z = B.gemm(empty((4, 0)), empty((0, 7)), dev(rnd((4, 7))))
    assert np.all(host(z) == 0)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("layout,shape", [("nt", (128, 650, 2600)), ("nn", (128, 2600, 650)), ("tn", (100, 70, 4099)), ("nt", (33, 10, 3000))])
def test_gemm_split_k(dt, layout, shape):
    # few output tiles and a long K: the product is cut along K when the caller provides the workspace
    M, N, K = shape
    A, Bm, Ad, Bd = operands(M, N, K, layout, dt)
    need = B.gemm_workspace_bytes(Ad, Bd, empty((M, N)))
    assert need > 0 or K < 2600          # the planner always splits these long-K shapes
    w = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    ref, S = O.gemm(A, Bm), O.gemm(np.abs(A), np.abs(Bm))
    out = B.gemm(Ad, Bd, empty((M, N)), ws=w)
    check(host(out), ref, TOL_SUM, S, "split-K")
    out2 = B.gemm(Ad, Bd, empty((M, N)), ws=w)
    assert torch.equal(out, out2)                                   # fixed order: bit-reproducible
    unsplit = B.gemm(Ad, Bd, empty((M, N)))                         # no workspace: same product, unsplit
    check(host(unsplit), ref, TOL_SUM, S, "unsplit")
    # epilogue and beta run in the finishing kernel
    bias, C0 = rnd((N,)), rnd((M, N))
    Cd = dev(C0)
    B.gemm(Ad, Bd, Cd, alpha=0.5, beta=1.0, epilogue="bias_relu", bias=dev(bias), ws=w)
    want = O.elementwise("relu", [O.elementwise("add", [O.gemm(A, Bm, C0, 0.5, 1.0), bias])])
    check(host(Cd), want, TOL_SUM, 0.5 * S + np.abs(C0) + np.abs(bias), "split-K epilogue")
    gi = lambda s, d: RNG.integers(-3, 4, size=s).astype(np.float32)
    A, Bm, Ad, Bd = operands(M, N, K, layout, dt, gi)
    assert np.array_equal(host(B.gemm(Ad, Bd, empty((M, N)), ws=w)), A.astype(np.float64) @ Bm.astype(np.float64))


@pytest.mark.parametrize("dt,cdt", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32")])
@pytest.mark.parametrize("layout", ["nt", "nn", "tn"])
def test_gemm_direct_copy_epilogues(dt, cdt, layout, direct_kernel):
    # every epilogue, beta and both C dtypes on the 256x256 direct-copy kernel: an interior of full tiles
    # (vector path), a ragged last tile in M (rows past the end) and in N (element-wise path)
    if dt == "f32" and layout == "tn":
        pytest.skip("fp32 with both operands stored along M/N takes the register-staged kernel")
    if dt == "f32" and direct_kernel == "eight waves":
        pytest.skip("fp32 products have the four-wave kernel only")
    M, N, K = 3720, 3592, 1000      # (long enough for the planner to take the 256x256 tile)
    A, Bm, Ad, Bd = operands(M, N, K, layout, dt)
    assert B.gemm_plan(Ad, Bd, empty((M, N), cdt))[:2] == (2, True)
    tol = TOL_BF16 if cdt == "bf16" else TOL_SUM
    rd = (lambda a: bf16r(a)) if cdt == "bf16" else (lambda a: a)
    bias = rnd((N,))
    aux = rd(rnd((M, N)))
    c0 = rd(rnd((M, N)))
    # the linear part in fp64 by a library product, tied to the oracle on sampled rows
    lin = A.astype(np.float64) @ Bm.astype(np.float64)
    S = np.abs(A).astype(np.float64) @ np.abs(Bm).astype(np.float64)
    rows = RNG.integers(0, M, 16)
    assert np.allclose(O.gemm(A[rows], Bm), lin[rows], rtol=1e-12, atol=1e-12)
    # alpha / beta
    out = B.gemm(Ad, Bd, dev(c0, cdt), alpha=0.5, beta=-1.25)
    check(host(out), 0.5 * lin - 1.25 * c0.astype(np.float64), tol, 0.5 * S + 1.25 * np.abs(c0), "alpha/beta")
    # bias, bias+relu, bias+gelu (+ pre-activation)
    z = lin + bias
    Sz = S + np.abs(bias)
    check(host(B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias", bias=dev(bias))), z, tol, Sz, "bias")
    check(host(B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias_relu", bias=dev(bias))), np.maximum(z, 0), tol, Sz, "bias_relu")
    pre = empty((M, N), cdt)
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias_gelu", bias=dev(bias), preact_out=pre)
    check(host(pre), z, tol, Sz, "preact")
    check(host(out), O.elementwise("gelu", [z]), tol, Sz, "bias_gelu")
    # activation gradients against the retained activation / pre-activation
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="relu_bwd", aux=dev(aux, cdt))
    check(host(out), np.where(aux > 0, lin, 0.0), tol, S, "relu_bwd")
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="gelu_bwd", aux=dev(aux, cdt))
    gp = O.elementwise("gelu_bwd", [np.ones_like(aux, dtype=np.float64), aux.astype(np.float64)])
    # (the epilogue's gelu' has an absolute error of up to 3e-7 -- a 1.5e-7 rational erf plus fp32
    # rounding -- which the product magnifies by |lin| <= S: 3e-7 S = tol * 3e-3 S at the fp32 bar)
    check(host(out), lin * gp, tol, S * np.abs(gp) + 3e-3 * S, "gelu_bwd")
    # gelu_bwd with beta: accumulate into old C
    out = B.gemm(Ad, Bd, dev(c0, cdt), beta=1.0, epilogue="gelu_bwd", aux=dev(aux, cdt))
    check(host(out), (lin + c0) * gp, tol, (S + np.abs(c0)) * (np.abs(gp) + 3e-3), "gelu_bwd beta")


@pytest.mark.parametrize("dt,cdt", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32")])
@pytest.mark.parametrize("layout,shape", [("nn", (512, 768, 200)), ("nt", (768, 256, 1000)), ("tn", (256, 512, 72))])
def test_gemm_activation_gradient_with_row_block_column_sums(dt, cdt, layout, shape, direct_kernel):
    """The activation-gradient epilogues can leave, beside C, the column sums of C over blocks of 128
    rows (the bias gradient of the layer below is their column sum).  C is checked against the oracle
    as without the sums; the sums against the stored C, to fp32 summation accuracy, which pins them to
    the values as stored (rounded to bf16 where C is bf16)."""
    if dt == "f32" and direct_kernel == "eight waves":
        pytest.skip("fp32 products have the four-wave kernel only")
    M, N, K = shape
    A, Bm, Ad, Bd = operands(M, N, K, layout, dt)
    tol = TOL_BF16 if cdt == "bf16" else TOL_SUM
    aux = rnd((M, N))
    aux = bf16r(aux) if cdt == "bf16" else aux
    lin = O.gemm(A, Bm)
    S = np.abs(A).astype(np.float64) @ np.abs(Bm).astype(np.float64)
    gp = O.elementwise("gelu_bwd", [np.ones_like(aux, dtype=np.float64), aux.astype(np.float64)])
    for epi, ref, scale in (("relu_bwd", np.where(aux > 0, lin, 0.0), S), ("gelu_bwd", lin * gp, S * np.abs(gp) + 3e-3 * S)):
        plain = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue=epi, aux=dev(aux, cdt))
        sums = empty((M // 128, N))
        sums.fill_(float("nan"))
        out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue=epi, aux=dev(aux, cdt), preact_out=sums)
        check(host(out), ref, tol, scale, epi)
        if B.gemm_plan(Ad, Bd, out)[0] == 2 and B.gemm_plan(Ad, Bd, out)[2] == 1:
            assert torch.equal(out, plain)                       # same kernel, same C
        c = host(out).reshape(M // 128, 128, N)
        got = host(sums)
        assert np.all(np.abs(got - c.sum(axis=1)) <= 1e-5 * np.abs(c).sum(axis=1) + 1e-30), epi
        # and so the bias gradient: one small reduction instead of a pass over C
        db = B.reduce_axis("sum", sums, 0, empty((N,)))
        check(host(db), ref.sum(axis=0), tol, scale.sum(axis=0), epi + " bias gradient")
    # what the call refuses (nothing is launched)
    with pytest.raises(B.ChnError):
        B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="gelu_bwd", aux=dev(aux, cdt), preact_out=empty((M // 128 + 1, N)))
    with pytest.raises(B.ChnError):
        B.gemm(Ad, Bd, dev(aux, cdt), beta=1.0, epilogue="gelu_bwd", aux=dev(aux, cdt), preact_out=empty((M // 128, N)))
    with pytest.raises(B.ChnError):
        B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias", bias=dev(rnd((N,))), preact_out=empty((M // 128, N)))


@pytest.mark.parametrize("layout", ["nt", "tn"])
def test_gemm_direct_copy_split_k(layout, direct_kernel):
    # few tiles and a long K: the direct-copy kernel writes fp32 slabs, the finishing kernel adds them
    M, N, K = 1000, 4096, 8192
    gen = lambda s, d: RNG.integers(-2, 3, size=s).astype(np.float32)
    A, Bm, Ad, Bd = operands(M, N, K, layout, "bf16", gen)
    out = empty((M, N))
    tile, dc, splits = B.gemm_plan(Ad, Bd, out, have_workspace=True)
    assert (tile, dc) == (2, True) and splits > 1
    need = B.gemm_workspace_bytes(Ad, Bd, out)
    assert need > 0
    B.gemm(Ad, Bd, out, ws=ws(need))
    assert np.array_equal(host(out), A.astype(np.float64) @ Bm.astype(np.float64))


@pytest.fixture
def narrow_tile():
    B.gemm_plan_override(tile=3)
    yield
    B.gemm_plan_override()


@pytest.mark.parametrize("cdt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(300, 200, 128), (513, 129, 200), (1030, 1000, 520), (256, 128, 64), (2, 3, 8)])
def test_gemm_256x128_tile(shape, cdt, narrow_tile):
    # the 256 x 128 tile of the eight-wave kernel (bf16, both operands unit-stride along K): full tiles, ragged last
    # tiles in M, N and K, every epilogue, cut along K or not; small integers must come out bit for bit
    M, N, K = shape
    gi = lambda s, d: RNG.integers(-3, 4, size=s).astype(np.float32)
    A, Bm, Ad, Bd = operands(M, N, K, "nt", "bf16", gi)
    assert B.gemm_plan(Ad, Bd, empty((M, N), cdt))[:2] == (3, True)
    w = ws(4 * M * ((N + 3) // 4 * 4) * 4 + 256)
    lin = O.gemm(A, Bm)
    for splits in (1, 2):
        B.gemm_plan_override(tile=3, splits=splits)
        assert np.array_equal(host(B.gemm(Ad, Bd, empty((M, N), cdt), ws=w)), O.round_bf16(lin) if cdt == "bf16" else lin), splits
    B.gemm_plan_override(tile=3)
    A, Bm, Ad, Bd = operands(M, N, K, "nt", "bf16")
    tol = TOL_BF16 if cdt == "bf16" else TOL_SUM
    rd = (lambda a: bf16r(a)) if cdt == "bf16" else (lambda a: a)
    bias, aux, c0 = rnd((N,)), rd(rnd((M, N))), rd(rnd((M, N)))
    lin, S = O.gemm(A, Bm), O.gemm(np.abs(A), np.abs(Bm))
    out = B.gemm(Ad, Bd, dev(c0, cdt), alpha=0.5, beta=-1.25)
    check(host(out), 0.5 * lin - 1.25 * c0.astype(np.float64), tol, 0.5 * S + 1.25 * np.abs(c0), "alpha/beta")
    z, Sz = lin + bias, S + np.abs(bias)
    check(host(B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias", bias=dev(bias))), z, tol, Sz, "bias")
    check(host(B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias_relu", bias=dev(bias))), np.maximum(z, 0), tol, Sz, "bias_relu")
    pre = empty((M, N), cdt)
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="bias_gelu", bias=dev(bias), preact_out=pre)
    check(host(pre), z, tol, Sz, "preact")
    check(host(out), O.elementwise("gelu", [z]), tol, Sz, "bias_gelu")
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="relu_bwd", aux=dev(aux, cdt))
    check(host(out), np.where(aux > 0, lin, 0.0), tol, S, "relu_bwd")
    out = B.gemm(Ad, Bd, empty((M, N), cdt), epilogue="gelu_bwd", aux=dev(aux, cdt))
    gp = O.elementwise("gelu_bwd", [np.ones_like(aux, dtype=np.float64), aux.astype(np.float64)])
    check(host(out), lin * gp, tol, S * np.abs(gp) + 3e-3 * S, "gelu_bwd")
    if cdt == "f32":
        W0, low = rnd((M, N)), empty((M, N), "bf16")
        Wd = dev(W0)
        B.gemm(Ad, Bd, Wd, alpha=-0.01, beta=1.0, epilogue="bf16_copy", preact_out=low)
        check(host(Wd), W0 - 0.01 * lin, TOL_SUM, np.abs(W0) + 0.01 * S, "update")
        assert np.array_equal(host(low), O.round_bf16(host(Wd)))


def test_gemm_256x128_tile_is_planned_for_a_classifier_layer_only():
    x, W3 = empty((8192, 4096), "bf16"), empty((1000, 4096), "bf16")
    assert B.gemm_plan(x, W3.t(), empty((8192, 1000)), True) == (3, True, 1)            # logits of the wide MLP
    assert B.gemm_plan(x, empty((4096, 4096), "bf16").t(), empty((8192, 4096), "bf16"), True)[0] == 2
    assert B.gemm_plan(x, empty((4096, 1000), "bf16"), empty((8192, 1000)), True)[0] != 3   # B unit-stride along N
    assert B.gemm_plan(empty((8192, 4096)), empty((1000, 4096)).t(), empty((8192, 1000)), True)[0] != 3   # fp32
    B.gemm_plan_override(direct_copy=2)                                                  # four-wave kernel forced
    try:
        assert B.gemm_plan(x, W3.t(), empty((8192, 1000)), True)[0] != 3
    finally:
        B.gemm_plan_override()


def test_gemm_degenerate_sizes():
    # K == 0: nothing to multiply, the epilogue still runs on beta * C;  M == 0 or N == 0: nothing to do
    c0 = rnd((70, 90))
    bias = rnd((90,))
    a = torch.empty((70, 0), device="cuda")
    b = torch.empty((0, 90), device="cuda")
    out = B.gemm(a, b, dev(c0), alpha=3.0, beta=2.0, epilogue="bias", bias=dev(bias))
    check(host(out), 2.0 * c0.astype(np.float64) + bias, 1e-6, np.abs(bias), "K = 0")
    out = B.gemm(a, b, dev(c0))                      # beta = 0: C must not be read (it may hold NaNs)
    assert np.all(host(out) == 0.0)
    nan = dev(np.full((70, 90), np.nan, np.float32))
    assert np.all(host(B.gemm(a, b, nan)) == 0.0)
    x = dev(rnd((0, 33)))
    B.gemm(x, dev(rnd((33, 20))), torch.empty((0, 20), device="cuda"))
    B.gemm(dev(rnd((20, 33))), torch.empty((33, 0), device="cuda"), torch.empty((20, 0), device="cuda"))
    # beta = 0 never reads C either when there is something to multiply
    A, Bm, Ad, Bd = operands(64, 48, 40, "nt", "f32")
    check(host(B.gemm(Ad, Bd, dev(np.full((64, 48), np.nan, np.float32)))), O.gemm(A, Bm), TOL_SUM, O.gemm(np.abs(A), np.abs(Bm)), "NaN in C, beta 0")


@pytest.mark.parametrize("shape,layout", [((150, 200, 90), "tn"), ((3720, 3592, 192), "tn"), ((1000, 4096, 8192), "tn"), ((257, 130, 100), "nt")])
def test_gemm_bf16_copy_epilogue_is_an_sgd_update(shape, layout, direct_kernel):
    # C (fp32 master weights) <- C - lr * A B, preact_out <- bf16(C): small tile, direct-copy kernel,
    # split-K finishing kernel, element-wise path (N not a multiple of 4)
    M, N, K = shape
    lr = 0.05
    A, Bm, Ad, Bd = operands(M, N, K, layout, "bf16")
    W0 = rnd((M, N))
    Wd = dev(W0)
    low = empty((M, N), "bf16")
    need = B.gemm_workspace_bytes(Ad, Bd, Wd)
    B.gemm(Ad, Bd, Wd, alpha=-lr, beta=1.0, epilogue="bf16_copy", preact_out=low, ws=ws(need) if need else None)
    g = A.astype(np.float64) @ Bm.astype(np.float64)
    S = np.abs(A).astype(np.float64) @ np.abs(Bm).astype(np.float64)
    check(host(Wd), W0 - lr * g, TOL_SUM, np.abs(W0) + lr * S, "update")
    assert np.array_equal(host(low), O.round_bf16(host(Wd)))
    with pytest.raises(B.ChnError):
        B.gemm(Ad, Bd, Wd, epilogue="bf16_copy")                                   # needs preact_out
    with pytest.raises(B.ChnError):
        B.gemm(Ad, Bd, empty((M, N), "bf16"), epilogue="bf16_copy", preact_out=low)  # C must be fp32


def test_gemm_random_shapes_exact_integers():
    # a seeded sweep over dtypes, layouts, ragged and aligned sizes, epilogues, beta and C dtypes with
    # small-integer operands: every sum is exact in fp32, so whatever kernel, tile and K split the
    # planner picks the result must equal the fp64 product bit for bit (after C's own rounding)
    rng = np.random.default_rng(1908_00213)
    for it in range(120):
        dt = rng.choice(["bf16", "f32"])
        lay = rng.choice(["nt", "nn", "tn", "tt"])
        m8 = 8 if dt == "bf16" else 4
        M, N, K = (int(rng.integers(1, 160)) * m8 for _ in range(3))
        if rng.random() < 0.3:
            K = int(rng.integers(1, 2000))
        if rng.random() < 0.2:
            M = int(rng.integers(1, 1200))
        if rng.random() < 0.2:
            N = int(rng.integers(1, 1200))
        cdt = "f32" if dt == "f32" else rng.choice(["bf16", "f32"])
        gen = lambda s: rng.integers(-3, 4, size=s).astype(np.float32)
        a = gen((M, K)) if lay[0] == "n" else gen((K, M))
        b = gen((K, N)) if lay[1] == "n" else gen((N, K))
        A, Bm = (a if lay[0] == "n" else a.T), (b if lay[1] == "n" else b.T)
        Ad = dev(a, dt) if lay[0] == "n" else dev(a, dt).t()
        Bd = dev(b, dt) if lay[1] == "n" else dev(b, dt).t()
        ref = A.astype(np.float64) @ Bm.astype(np.float64)
        c0 = gen((M, N))
        Cd = dev(c0, cdt)
        epi = rng.choice(["none", "bias", "bias_relu", "relu_bwd", "beta"])
        kw = {}
        if epi in ("bias", "bias_relu"):
            bias = gen((N,))
            kw = dict(epilogue=epi, bias=dev(bias))
            ref = ref + bias
            if epi == "bias_relu":
                ref = np.maximum(ref, 0)
        elif epi == "relu_bwd":
            aux = gen((M, N))
            kw = dict(epilogue=epi, aux=dev(aux, cdt))
            ref = np.where(aux > 0, ref, 0.0)
        elif epi == "beta":
            kw = dict(alpha=2.0, beta=-1.0)
            ref = 2.0 * ref - c0
        need = B.gemm_workspace_bytes(Ad, Bd, Cd)
        out = host(B.gemm(Ad, Bd, Cd, ws=ws(need) if need else None, **kw))
        want = bf16r(ref.astype(np.float32)).astype(np.float64) if cdt == "bf16" else ref
        assert np.array_equal(out, want), (it, dt, cdt, lay, (M, N, K), epi, B.gemm_plan(Ad, Bd, Cd, need > 0))
