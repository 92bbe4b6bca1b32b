"""User-defined kernels without a GPU: the oracle's user-kernel evaluator pinned against NumPy's
closed forms, and the library's host side (declaration parsing, type-parameter binding, choice of
the generated form, run-time compilation for gfx950, the code-object cache, error reporting)."""
import os

import numpy as np
import pytest

from oracle import user_kernel as OU
from paper_1908_00213_amd import binding as B


# ---- the oracle against NumPy ---------------------------------------------------------------------------
def test_oracle_my_mad_is_x_times_y_plus_z():
    # figure "Example of a user-defined kernel"
    rng = np.random.default_rng(0)
    x, y, z = rng.standard_normal((3, 37, 5))
    k = OU.ElementwiseKernel("float32 x, float32 y, float32 z", "float32 w", "w = x * y + z", "my_mad")
    np.testing.assert_array_equal(k(x, y, z), x * y + z)


def test_oracle_type_parameter_broadcast_scalar_and_two_outputs():
    rng = np.random.default_rng(1)
    k = OU.ElementwiseKernel("T x, T y, float32 s", "T lo, T hi", "lo = min(x, y) * (T)s; hi = max(x, y)", "minmax")
    a, b = rng.integers(-50, 50, (4, 6)).astype(np.int32), rng.integers(-50, 50, (6,)).astype(np.int32)
    lo, hi = k(a, b, 3.0)
    assert lo.dtype == np.int32 and np.array_equal(lo, np.minimum(a, b) * 3) and np.array_equal(hi, np.maximum(a, b))
    x, y = rng.standard_normal((4, 1)), rng.standard_normal((1, 6))
    lo, hi = k(x, y, 0.5)
    np.testing.assert_array_equal(lo, np.minimum(x, y) * 0.5)
    np.testing.assert_array_equal(hi, np.maximum(x, y) * np.ones((4, 6)))
    big = np.array([2**40 + 1, -2**41], dtype=np.int64)
    assert np.array_equal(k(big, big[::-1].copy(), 1.0)[1], np.array([2**40 + 1, 2**40 + 1]))


def test_oracle_reductions_are_numpy_folds():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 7, 3))
    s = OU.ReductionKernel("T x", "T y", "x", "a + b", "y = a", "0", "sum")
    for axis in (0, 1, 2, -1, None):
        np.testing.assert_allclose(s(x, axis=axis), x.sum(axis=axis), rtol=1e-14, atol=1e-14)
    assert s(x, axis=1, keepdims=True).shape == (5, 1, 3)
    y = rng.standard_normal((4, 5, 6, 7))
    for axes in ((0, 2), (1, 3), (0, 1, 2), (1, 2), (3,)):
        np.testing.assert_allclose(s(y, axis=axes), y.sum(axis=axes), rtol=1e-13)
        assert s(y, axis=axes, keepdims=True).shape == y.sum(axis=axes, keepdims=True).shape
    l2 = OU.ReductionKernel("T x", "T y", "x * x", "a + b", "y = sqrt(a)", "0", "l2norm")
    np.testing.assert_allclose(l2(x, axis=None), np.linalg.norm(x.ravel()), rtol=1e-14)
    np.testing.assert_allclose(l2(x, axis=2), np.linalg.norm(x, axis=2), rtol=1e-14)
    mx = OU.ReductionKernel("T x", "T y", "x", "max(a, b)", "y = a", "-1e300", "max")
    np.testing.assert_array_equal(mx(x, axis=0), x.max(axis=0))
    xi = rng.integers(-1000, 1000, (9, 11)).astype(np.int64)
    assert np.array_equal(s(xi, axis=0), xi.sum(axis=0)) and s(xi, axis=0).dtype == np.int64
    # two inputs, a scalar in the final expression: scaled dot product of rows
    dot = OU.ReductionKernel("T x, T y, float32 c", "float32 z", "x * y", "a + b", "z = a * c", "0", "dot")
    u, v = rng.standard_normal((4, 8)), rng.standard_normal((8,))
    np.testing.assert_allclose(dot(u, v, 0.25, axis=1), 0.25 * (u @ v), rtol=1e-13)
    # an empty reduced range gives the final expression of the identity
    assert np.array_equal(l2(np.zeros((3, 0)), axis=1), np.zeros(3))


# ---- the library's host side ---------------------------------------------------------------------------------
@pytest.fixture
def cache(tmp_path):
    B.user_kernel_config(str(tmp_path), "gfx950")
    return tmp_path


def fake(shape, dtype=B.F32, strides=None, ptr=0x7f0000000000):
    isz = {B.F32: 4, B.BF16: 2, B.I32: 4, B.I64: 8}[dtype]
    if strides is None:
        strides, acc = [], isz
        for n in reversed(shape):
            strides.insert(0, acc)
            acc *= n
    return B.raw_desc(ptr, shape, strides, dtype)


def test_declarations_are_checked_at_creation():
    for bad in (dict(in_params="float32"), dict(in_params="float32 x y"), dict(in_params="float64 x"),
                dict(in_params="float32 x, float32 x"), dict(in_params="float32 i"), dict(out_params=""),
                dict(in_params="float32 chn_x"), dict(name="my mad")):
        kw = dict(in_params="float32 x", out_params="float32 w", operation="w = x", name="k")
        kw.update(bad)
        with pytest.raises(B.ChnError):
            B.ElementwiseKernel(**kw)
    with pytest.raises(B.ChnError):
        B.ReductionKernel("T a", "T y", "a", "a + b", "y = a", "0", "r")     # `a` names the fold operand


def test_generated_form_follows_layout_and_types(cache):
    k = B.ElementwiseKernel("T x, T y", "T w", "w = x + y", "add2")
    x = fake((64, 100))
    flat = k.source(x, x, x)
    assert "chn_pack<float, 4>" in flat and "typedef float T;" in flat and "chn_rem" not in flat
    h = fake((64, 100), B.BF16)
    assert "chn_pack<chn_bf16, 8>" in k.source(h, h, h)                       # 16 bytes per lane
    li = fake((64, 100), B.I64)
    assert "chn_pack<long long, 2>" in k.source(li, li, li) and "typedef long long T;" in k.source(li, li, li)
    # a repeated single element is read once
    one = fake((1, 1))
    assert "chn_io<float>::ld(chn_p1);" in k.source(x, one, x)
    # a row operand, a column operand, rows pitched by whole vectors: one vector of the row per thread
    for other in (fake((100,)), fake((64, 1)), fake((64, 100), strides=[512, 4])):
        src = k.source(x, other, x)
        assert "chn_row" in src and "chn_pack<float, 4>" in src and "chn_rem" not in src
    assert "chn_io<float>::ld(chn_p1 + chn_o1);" in k.source(x, fake((64, 1)), x)      # the column: once per thread
    # transposed view, rows pitched by an odd count, a row length that is no whole number of
    # vectors, a pointer that is not 16-byte aligned: one element per thread
    assert "chn_rem" in k.source(fake((64, 100), strides=[4, 256]), x, x)
    assert "chn_rem" in k.source(fake((64, 100), strides=[404, 4]), x, x)
    assert "chn_rem" in k.source(fake((64, 99)), fake((99,)), fake((64, 99)))
    assert "chn_rem" in k.source(fake((64, 100), ptr=0x7f0000000004), x, x)
    # more than 2^31 elements: 64-bit index arithmetic
    big = fake((1 << 16, 1 << 16), strides=[0, 0])
    bigo = fake((1 << 16, 1 << 16), strides=[8 << 16, 8])
    assert "long long chn_rem" in k.source(big, big, bigo)
    mixed = B.ElementwiseKernel("T x, float32 s", "bfloat16 y", "y = x * s", "scale_to_bf16")
    src = mixed.source(x, 2.0, h)
    assert "chn_scalar<float>" in src and "chn_pack<chn_bf16, 4>" in src and "chn_pack<float, 4>" in src


def test_type_binding_and_shape_errors(cache):
    k = B.ElementwiseKernel("T x, T y, float32 z", "T w", "w = x * y + z", "k")
    x, h = fake((8, 8)), fake((8, 8), B.BF16)
    for args, status in (((x, h, x, x), -3),          # T bound to two dtypes
                         ((x, x, h, x), -3),          # z is declared float32
                         ((x, x, x, h), -3),          # the output's T against the inputs'
                         ((x, x, fake((8, 7)), x), -4),
                         ((fake((2, 8, 8)), x, x, x), -4)):
        with pytest.raises(B.ChnError) as e:
            k.prepare(*args)
        assert e.value.status == status, args
    only_scalar = B.ElementwiseKernel("float32 x, T s", "float32 w", "w = x * s", "k2")
    with pytest.raises(B.ChnError) as e:
        only_scalar.prepare(x, 2.0, x)
    assert e.value.status == -3
    with pytest.raises(TypeError):
        k.prepare(x, x)


def test_compile_cache_memory_then_disk_then_compiler(cache):
    c0, d0, m0 = B.user_kernel_stats()
    x = fake((32, 32))
    k = B.ElementwiseKernel("float32 x, float32 y, float32 z", "float32 w", "w = x * y + z", "my_mad")
    k.prepare(x, x, x, x)
    assert B.user_kernel_stats() == (c0 + 1, d0, m0)
    files = os.listdir(cache)
    assert len(files) == 1 and files[0].endswith(".hsaco")
    with open(os.path.join(cache, files[0]), "rb") as f:
        assert f.read(4) == b"\x7fELF"
    k.prepare(x, x, x, x)                                    # same object: memory
    assert B.user_kernel_stats() == (c0 + 1, d0, m0 + 1)
    k2 = B.ElementwiseKernel("float32 x, float32 y, float32 z", "float32 w", "w = x * y + z", "my_mad")
    k2.prepare(x, x, x, x)                                   # a later object (or run): disk
    assert B.user_kernel_stats() == (c0 + 1, d0 + 1, m0 + 1)
    k2.prepare(fake((32, 32), strides=[4, 128]), x, x, x)    # another form of the same kernel: compiled
    assert B.user_kernel_stats()[0] == c0 + 2 and len(os.listdir(cache)) == 2
    k3 = B.ElementwiseKernel("float32 x, float32 y, float32 z", "float32 w", "w = x * y - z", "my_mad")
    k3.prepare(x, x, x, x)                                   # another snippet: compiled
    assert B.user_kernel_stats()[0] == c0 + 3
    # a damaged cache file is not trusted
    for f in os.listdir(cache):
        with open(os.path.join(cache, f), "wb") as fh:
            fh.write(b"garbage")
    k4 = B.ElementwiseKernel("float32 x, float32 y, float32 z", "float32 w", "w = x * y + z", "my_mad")
    k4.prepare(x, x, x, x)
    assert B.user_kernel_stats()[0] == c0 + 4
    # nor is a good file that somebody else could have written (group- or world-writable)
    assert all((os.stat(os.path.join(cache, f)).st_mode & 0o022) == 0 for f in os.listdir(cache))
    for f in os.listdir(cache):
        os.chmod(os.path.join(cache, f), 0o666)
    c1, d1, _ = B.user_kernel_stats()
    k5 = B.ElementwiseKernel("float32 x, float32 y, float32 z", "float32 w", "w = x * y + z", "my_mad")
    k5.prepare(x, x, x, x)
    assert B.user_kernel_stats()[:2] == (c1 + 1, d1)         # compiled again, not loaded


def test_a_snippet_that_does_not_compile_reports_the_compilers_error(cache):
    k = B.ElementwiseKernel("float32 x", "float32 w", "w = x +* undefined_name", "broken")
    with pytest.raises(B.ChnError) as e:
        k.prepare(fake((4,)), fake((4,)))
    assert e.value.status == -10 and "error" in str(e.value)
    assert os.listdir(cache) == []


def test_reduction_declaration_shapes_and_workspace(cache):
    s = B.ReductionKernel("T x", "T y", "x", "a + b", "y = a", "0", "sum")
    x = fake((8192, 4096))
    L = B.lib()
    ws = lambda out, axis, keep=0: L.chn_reduction_kernel_workspace_bytes(
        s._h, 1, B._ptrs([x]), 1, B._ptrs([out]), axis, keep)
    assert ws(fake((8192,)), 1) == 0                          # one block per row, rows enough to fill the chip
    assert ws(fake((4096,)), 0) > 0                           # column sums: the rows are cut into slices
    assert ws(fake(()), B.AXIS_ALL) > 0
    s.prepare(x, fake((8192,)), axis=1)
    s.prepare(x, fake((4096,)), axis=0)
    s.prepare(x, fake((8192, 1)), axis=-1, keepdims=True)
    for out, axis, status in ((fake((4096,)), 1, -4), (fake((8192,)), 2, -7), (fake((8192,), B.BF16), 1, -3)):
        with pytest.raises(B.ChnError) as e:
            s.prepare(x, out, axis=axis)
        assert e.value.status == status
    y4 = fake((4, 50, 6, 70))
    s.prepare(y4, fake((50, 70)), axis=(0, 2))
    s.prepare(y4, fake((4, 1, 1, 70)), axis=(1, 2), keepdims=True)
    with pytest.raises(B.ChnError) as e:
        s.prepare(y4, fake((50, 70)), axis=(0, 1))               # the output has the shape of another axis set
    assert e.value.status == -4
    L2 = B.lib()
    assert L2.chn_reduction_kernel_prepare(s._h, 1, B._ptrs([y4]), 1, B._ptrs([fake((50, 70))]), 0x40000000 + (1 << 5), 0) == -7
    src_row = s.source(x, fake((8192,)), axis=1)
    src_col = s.source(x, fake((4096,)), axis=0)
    assert "chn_sm[256]" in src_row.split("_finish")[0]                            # a block folds a row
    assert "chn_sm[16][16 * 4 + 1]" in src_col.split("_finish")[0]                 # 16 row lanes share 4 columns
    assert "chn_pack<float, 4>" in src_row and "chn_acc[4]" in src_col             # 16 bytes per lane in both
    assert "__shared__" not in s.source(fake((8192, 4095)), fake((4095,)), axis=0).split("_finish")[0]   # scalar form: a thread per column
    odd = fake((8192, 4095))
    assert "chn_pack<float" not in s.source(odd, fake((8192,)), axis=1)              # rows off the vector grid
    assert "chn_pack<float" not in s.source(odd, fake((4095,)), axis=0)
    assert "chn_sl += 256" in s.source(x, fake(()), axis=None).split("_finish")[1]   # one result: a block folds the slices


def test_new_entry_points_are_exported():
    L = B.lib()
    for name in B.EXPORTS:
        assert hasattr(L, name), name
