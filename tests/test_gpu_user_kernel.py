"""GPU parity of user-defined kernels (snippets compiled at run time on the box, launched through
the C ABI) against the oracle's evaluation of the same snippets: element by element, integers bit
for bit, floating point within the element-wise / reduction tolerances of the fixed-function kernels."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from oracle import user_kernel as OU
from paper_1908_00213_amd import binding as B
from tests.util import TOL_BF16, TOL_EW, TOL_SUM, bf16r, check, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _cache(tmp_path_factory):
    B.user_kernel_config(str(tmp_path_factory.getbasetemp() / "chn_kernels"), None)


MAD = ("float32 x, float32 y, float32 z", "float32 w", "w = x * y + z", "my_mad")


@pytest.mark.parametrize("shape", [(1,), (3,), (4,), (1000,), (257, 129), (64, 1024), (5, 6, 7, 8), ()])
def test_my_mad_of_the_figure(shape):
    rng = np.random.default_rng(len(shape) * 1000 + int(np.prod(shape)))
    x, y, z = (rng.standard_normal(shape).astype(np.float32) for _ in range(3))
    w = B.ElementwiseKernel(*MAD)(*[dev(a.reshape(-1)).reshape(shape) for a in (x, y, z)])
    assert tuple(w.shape) == tuple(shape) and w.dtype == torch.float32
    check(host(w), OU.ElementwiseKernel(*MAD)(x, y, z), TOL_EW, np.abs(x * y) + np.abs(z), "my_mad %s" % (shape,))


def test_one_generic_kernel_serves_every_dtype():
    k = B.ElementwiseKernel("T x, T y, T z", "T w", "w = x * y + z", "mad_T")
    ko = OU.ElementwiseKernel("T x, T y, T z", "T w", "w = x * y + z", "mad_T")
    rng = np.random.default_rng(7)
    shape = (131, 77)
    f = [rng.standard_normal(shape).astype(np.float32) for _ in range(3)]
    check(host(k(*[dev(a) for a in f])), ko(*f), TOL_EW, np.abs(f[0] * f[1]) + np.abs(f[2]), "f32")
    h = [bf16r(a) for a in f]
    w = k(*[dev(a, "bf16") for a in h])
    assert w.dtype == torch.bfloat16
    check(host(w), ko(*h), TOL_BF16, np.abs(h[0] * h[1]) + np.abs(h[2]), "bf16")
    for dt, lim in ((np.int32, 30000), (np.int64, 2**31)):
        a = [rng.integers(-lim, lim, shape).astype(dt) for _ in range(3)]
        w = k(*[dev(v) for v in a])
        assert w.dtype == {np.int32: torch.int32, np.int64: torch.int64}[dt]
        assert np.array_equal(host(w), ko(*a)), dt           # integer arithmetic: bit for bit


def test_broadcasting_views_and_misaligned_pointers():
    k = B.ElementwiseKernel(*MAD)
    ko = OU.ElementwiseKernel(*MAD)
    rng = np.random.default_rng(8)
    r = lambda *s: rng.standard_normal(s).astype(np.float32)
    cases = [
        (r(64, 200), r(200), r(64, 1)),                       # row and column operands
        (r(64, 200), r(1, 1), r(64, 200)),                    # a single repeated element
        (r(3, 1, 50), r(1, 40, 1), r(50)),                    # every operand broadcast
    ]
    for x, y, z in cases:
        S = np.abs(x * y) + np.abs(z)
        check(host(k(dev(x), dev(y), dev(z))), ko(x, y, z), TOL_EW, S, "broadcast")
    x, y, z = r(96, 160), r(160, 96), r(96, 200)
    xd, yd, zd = dev(x), dev(y), dev(z)
    w = k(xd, yd.t(), zd[:, 3:163])                           # transposed view, pitched + misaligned view
    check(host(w), ko(x, y.T, z[:, 3:163]), TOL_EW, np.abs(x * y.T) + np.abs(z[:, 3:163]), "views")
    out = torch.zeros(96, 200, device="cuda")
    k(xd, yd.t(), zd[:, 3:163], out[:, 1:161])                # output is a misaligned, pitched view
    check(host(out[:, 1:161]), ko(x, y.T, z[:, 3:163]), TOL_EW, np.abs(x * y.T) + np.abs(z[:, 3:163]), "out view")
    assert float(out[:, 0].abs().sum()) == 0 and float(out[:, 161:].abs().sum()) == 0    # nothing written outside
    flat = r(1003)
    fd = dev(flat)
    w = k(fd[1:], fd[1:], fd[1:])                             # contiguous but 4-byte aligned only
    check(host(w), ko(flat[1:], flat[1:], flat[1:]), TOL_EW, flat[1:] ** 2 + np.abs(flat[1:]), "misaligned")
    e = torch.empty(0, 5, device="cuda")
    assert tuple(k(e, e, e).shape) == (0, 5)


def test_scalars_preamble_two_outputs_and_mixed_storage():
    rng = np.random.default_rng(9)
    x = bf16r(rng.standard_normal((70, 33)).astype(np.float32))
    decl = ("T x, float32 slope, float32 shift", "bfloat16 y, float32 g",
            "const float t = leaky(x, slope); y = t + shift; g = x > 0 ? 1.0f : slope", "leaky_relu",
            "__device__ __forceinline__ float leaky(float v, float s) { return v > 0 ? v : v * s; }")
    y, g = B.ElementwiseKernel(*decl)(dev(x, "bf16"), 0.125, 2.0)
    yo, go = OU.ElementwiseKernel(*decl)(x, 0.125, 2.0)
    assert y.dtype == torch.bfloat16 and g.dtype == torch.float32
    check(host(y), yo, TOL_BF16, np.abs(x) + 2.0, "y")
    assert np.array_equal(host(g), go)
    # the index of the element is visible to the snippet
    iota = B.ElementwiseKernel("T x", "int64 k", "k = i", "iota")(dev(x, "bf16"))
    assert np.array_equal(host(iota), np.arange(x.size).reshape(x.shape))
    yt = B.ElementwiseKernel("T x", "int64 k", "k = i", "iota")(dev(x, "bf16").t())
    assert np.array_equal(host(yt), np.arange(x.size).reshape(x.T.shape))


SUM = ("T x", "T y", "x", "a + b", "y = a", "0", "sum")
L2 = ("T x", "T y", "x * x", "a + b", "y = sqrt(a)", "0", "l2norm")
MAX = ("T x", "T y", "x", "max(a, b)", "y = a", "-3.0e38f", "amax")


@pytest.mark.parametrize("shape,axis", [((300, 513), 0), ((300, 513), 1), ((300, 513), None), ((7, 300, 65), 1),
                                        ((7, 300, 65), 0), ((7, 300, 65), -1), ((2049,), 0), ((1, 1), None),
                                        ((40, 70000), 0), ((70000, 40), 0), ((3, 200000), 1)])
def test_sum_l2norm_and_max_over_one_axis_or_all(shape, axis):
    rng = np.random.default_rng(sum(shape) * 10 + (7 if axis is None else axis + 1))
    x = rng.standard_normal(shape).astype(np.float32)
    xd = dev(x)
    ax = tuple(range(x.ndim)) if axis is None else axis
    for decl, S in ((SUM, np.abs(x).sum(axis=ax)), (L2, None), (MAX, None)):
        got = B.ReductionKernel(*decl)(xd, axis=axis)
        ref = OU.ReductionKernel(*decl)(x, axis=axis)
        assert tuple(got.shape) == ref.shape
        if decl is MAX:
            assert np.array_equal(host(got), ref)              # a selection: exact
        else:
            check(host(got), ref, TOL_SUM, S if S is not None else ref, decl[-1])
    kd = B.ReductionKernel(*SUM)(xd, axis=axis, keepdims=True)
    assert tuple(kd.shape) == OU.ReductionKernel(*SUM)(x, axis=axis, keepdims=True).shape


@pytest.mark.parametrize("axes", [(0, 2), (1, 3), (0, 1, 2), (1, 2), (0, 3), (2, 3), (0, 1, 2, 3)])
def test_reductions_over_several_axes(axes):
    rng = np.random.default_rng(sum(axes) + 40)
    x = rng.standard_normal((4, 50, 6, 72)).astype(np.float32)
    xd = dev(x)
    for decl in (SUM, L2, MAX):
        got = B.ReductionKernel(*decl)(xd, axis=axes)
        ref = OU.ReductionKernel(*decl)(x, axis=axes)
        assert tuple(got.shape) == ref.shape
        if decl is MAX:
            assert np.array_equal(host(got), ref)
        else:
            check(host(got), ref, TOL_SUM, np.abs(x).sum(axis=axes) if decl is SUM else ref, decl[-1])
    kd = B.ReductionKernel(*SUM)(xd, axis=axes, keepdims=True)
    assert tuple(kd.shape) == x.sum(axis=axes, keepdims=True).shape
    check(host(kd), x.astype(np.float64).sum(axis=axes, keepdims=True), TOL_SUM, np.abs(x).sum(axis=axes, keepdims=True), "keepdims")
    # a transposed view reduces to the same numbers
    xt = xd.permute(3, 1, 2, 0)
    at = tuple(sorted({0: 3, 1: 1, 2: 2, 3: 0}[a] for a in axes))
    check(host(B.ReductionKernel(*SUM)(xt, axis=at)), OU.ReductionKernel(*SUM)(x.transpose(3, 1, 2, 0), axis=at), TOL_SUM,
          np.abs(x.transpose(3, 1, 2, 0)).sum(axis=at), "permuted")


def test_reduction_types_views_two_inputs_and_reproducibility():
    rng = np.random.default_rng(10)
    xi = rng.integers(-1000, 1000, (513, 300)).astype(np.int64)
    for axis in (0, 1, None):
        assert np.array_equal(host(B.ReductionKernel(*SUM)(dev(xi), axis=axis)), OU.ReductionKernel(*SUM)(xi, axis=axis))
    xh = bf16r(rng.standard_normal((200, 300)).astype(np.float32))
    got = B.ReductionKernel(*SUM)(dev(xh, "bf16"), axis=0)
    assert got.dtype == torch.bfloat16
    check(host(got), OU.ReductionKernel(*SUM)(xh, axis=0), TOL_BF16, np.abs(xh).sum(axis=0), "bf16 sum")
    # bf16 in, fp32 out; transposed and sliced views; a second, broadcast input and a scalar
    dot = ("T x, T y, float32 c", "float32 z", "x * y", "a + b", "z = a * c", "0", "dot")
    u, v = bf16r(rng.standard_normal((300, 200)).astype(np.float32)), bf16r(rng.standard_normal((200,)).astype(np.float32))
    got = B.ReductionKernel(*dot)(dev(u, "bf16"), dev(v, "bf16"), 0.25, axis=1)
    check(host(got), OU.ReductionKernel(*dot)(u, v, 0.25, axis=1), TOL_SUM, 0.25 * (np.abs(u) @ np.abs(v)), "dot")
    x = rng.standard_normal((260, 300)).astype(np.float32)
    xd = dev(x)
    for view, ref in ((xd.t(), x.T), (xd[3:250, 5:290], x[3:250, 5:290])):
        for axis in (0, 1):
            check(host(B.ReductionKernel(*SUM)(view, axis=axis)), OU.ReductionKernel(*SUM)(ref, axis=axis), TOL_SUM,
                  np.abs(ref).sum(axis=axis), "view")
    # an empty reduced range gives the final expression of the identity
    assert np.array_equal(host(B.ReductionKernel(*L2)(torch.empty(5, 0, device="cuda"), axis=1)), np.zeros(5))
    # the order of the fold is fixed: the same call gives the same bits
    big = dev(rng.standard_normal((4096, 2048)).astype(np.float32))
    k = B.ReductionKernel(*SUM)
    for axis in (0, 1, None):
        a, b = k(big, axis=axis), k(big, axis=axis)
        assert torch.equal(a, b)


def test_agreement_with_the_fixed_function_kernels():
    # a user-written sum and the library's own reduce_axis answer the same question
    rng = np.random.default_rng(11)
    x = rng.standard_normal((1000, 777)).astype(np.float32)
    xd = dev(x)
    for axis in (0, 1):
        out = torch.empty(x.shape[1 - axis], device="cuda")
        ws = torch.empty(max(256, B.reduce_axis_workspace_bytes(xd, axis)), dtype=torch.uint8, device="cuda")
        B.reduce_axis("sum", xd, axis, out, ws=ws)
        check(host(B.ReductionKernel(*SUM)(xd, axis=axis)), host(out), 2 * TOL_SUM, np.abs(x).sum(axis=axis), "vs reduce_axis")
    ref = O.elementwise("mad", [x, x, x])
    check(host(B.ElementwiseKernel(*MAD)(xd, xd, xd)), ref, TOL_EW, x * x + np.abs(x), "vs oracle mad")


def test_cache_counters_and_errors_on_the_device():
    c0, d0, m0 = B.user_kernel_stats()
    x = torch.ones(100, device="cuda")
    decl = ("float32 x", "float32 w", "w = x * 3.0f + 0.5f", "affine_probe_for_the_cache_test")
    k = B.ElementwiseKernel(*decl)
    assert float(k(x)[7]) == 3.5
    c1, d1, m1 = B.user_kernel_stats()
    assert (c1 - c0) + (d1 - d0) == 1                         # compiled, or found on disk from an earlier run
    k(x)
    assert B.user_kernel_stats() == (c1, d1, m1 + 1)          # loaded specialisation: nothing else happens
    k2 = B.ElementwiseKernel(*decl)
    assert float(k2(x)[0]) == 3.5
    assert B.user_kernel_stats()[0] == c1 and B.user_kernel_stats()[1] == d1 + 1
    bad = B.ElementwiseKernel("float32 x", "float32 w", "w = no_such_function(x)", "broken")
    with pytest.raises(B.ChnError) as e:
        bad(x)
    assert e.value.status == -10
    with pytest.raises(B.ChnError) as e:
        B.ElementwiseKernel("T x, T y", "T w", "w = x + y", "add2")(x, x.to(torch.bfloat16))
    assert e.value.status == -3
    torch.cuda.synchronize()
