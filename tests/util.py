"""Helpers shared by the GPU parity tests: host<->device transfer that keeps bits, and the error bar.

Error bar (floating point): |gpu - oracle| <= tol * (|oracle| + S) per element, where S is the sum of
the absolute values of the terms the oracle added up for that element (|a*b| + |c| for x*y+z, sum |in|
for a reduction, sum |A||B| for a product; 0 for a single-term result).  Plain relative error is
unbounded where such sums cancel, which is why S appears.  tol: fp32 element-wise 1e-5, fp32
products/reductions 1e-4, bf16 inputs with fp32 accumulation 2e-2.
"""
import numpy as np
import torch

from paper_1908_00213_amd import workloads as W

TOL_EW = 1e-5
TOL_SUM = 1e-4
TOL_BF16 = 2e-2


def dev(a, dtype="f32"):
    """NumPy float32 array -> CUDA tensor of the given storage type holding the same values
    (bf16: the values must already be bf16-exact, see workloads.bf16_exact)."""
    a = np.asarray(a)
    if a.dtype.kind in "iu":
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return torch.from_numpy(a32).cuda()
    bits = W.bf16_bits(a32)
    assert np.array_equal(W.bf16_to_f32(bits), a32), "value not representable in bf16"
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def host(t):
    """CUDA tensor -> float64 NumPy array with the same values and shape (strides not kept)."""
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    if t.dtype == torch.float32:
        return t.cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


def empty(shape, dtype="f32"):
    return torch.empty(shape, dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")


def ws(nbytes):
    return torch.empty(max(256, int(nbytes)), dtype=torch.uint8, device="cuda")


def check(got, ref, tol, S=None, what=""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got) == np.isfinite(ref)), what + ": non-finite mismatch"
    fin = np.isfinite(ref)
    bound = tol * (np.abs(ref) + (0.0 if S is None else np.asarray(S, dtype=np.float64)))
    err = np.abs(got - ref)
    bad = fin & (err > bound)
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(fin, err - bound, -np.inf)), err.shape)
        raise AssertionError("%s: %d of %d outside tol %g; worst at %s: got %r ref %r bound %r" % (
            what, int(bad.sum()), err.size, tol, i, got[i], ref[i], bound[i] if np.ndim(bound) else bound))
    # infinities must agree in sign
    assert np.array_equal(got[~fin], ref[~fin]), what


def bf16r(a):
    """float32 array rounded so every value is bf16-exact (input quantisation)."""
    return W.bf16_exact(np.asarray(a, dtype=np.float32))
