"""Helpers for the GPU parity tests: move padded host buffers to the device, call the C ABI, compare."""
import numpy as np
import torch

import oracle
from paper_2003_00532_amd import binding, synth

TOL = 1e-13  # |C - C_ref| <= TOL * sum_k |a_ik b_kj|, the bar set for this path
# float32: both the sequential binary32 nest and the MFMA order are within gamma_K * S of the exact value;
# on zero-mean data each is off by about u = 2^-24 of S (random walk), the worst element over 10^8 by a
# few times that.  2^-19 = 32 u leaves a wide margin and is still 1/500 of the rigorous bound at K = 8192.
TOL32 = 2.0 ** -19


def tol_for(x):
    return TOL32 if x.dtype == np.float32 else TOL


def to_dev(buf, dev="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(buf)).to(dev)


def run_device(Abuf, Bbuf, Cbuf, M, N, K, variant=-1, stream=None):
    """Copy padded (rows, ld) host buffers to the GPU, run C += A B there, return (A, B, C) device buffers as NumPy."""
    lda, ldb, ldc = Abuf.shape[1], Bbuf.shape[1], Cbuf.shape[1]
    dA, dB, dC = to_dev(Abuf), to_dev(Bbuf), to_dev(Cbuf)
    fn = binding.gemm_f32_ex if Cbuf.dtype == np.float32 else binding.gemm_f64_ex
    fn(M, N, K, dA, lda, dB, ldb, dC, ldc, stream=stream, variant=variant)
    torch.cuda.synchronize()
    return dA.cpu().numpy(), dB.cpu().numpy(), dC.cpu().numpy()


def make_impl(variant=-1, force_ld=None):
    """Adapter with the `impl(A, B, C)` signature of tests/pins.py that runs on the GPU.

    Each operand is placed in a fresh sentinel-filled (rows, ld) device buffer whose ld is the
    view's row stride (so padded and odd leading dimensions reach the kernel); after the call the
    device-side padding of all three buffers must still hold the sentinel.
    """
    def ld_of(x):
        sz = x.dtype.itemsize
        if x.shape[0] > 1 and x.size > 0 and x.strides[0] % sz == 0 and x.strides[0] // sz >= x.shape[1]:
            return max(1, x.strides[0] // sz)
        return max(1, x.shape[1])

    def impl(A, B, C):
        M, K = A.shape
        N = B.shape[1]
        bufs = []
        for x in (A, B, C):
            ld = ld_of(x) if force_ld is None else max(1, x.shape[1]) + force_ld
            b = synth.padded(x.shape[0], x.shape[1], ld, dtype=x.dtype)
            b[:, :x.shape[1]] = x
            bufs.append(b)
        a2, b2, c2 = run_device(bufs[0], bufs[1], bufs[2], M, N, K, variant=variant)
        assert synth.padding_intact(a2, K) and synth.padding_intact(b2, N) and synth.padding_intact(c2, N), \
            "device padding was written"
        C[...] = c2[:, :N]
    return impl


def check_tolerance(got, want, S, what=""):
    """Elementwise |got - want| <= TOL * S; exact equality where S == 0.  Returns the worst ratio."""
    assert not np.isnan(got).any(), what + ": NaN in result"
    tol = tol_for(got)
    diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
    zero = S == 0
    if zero.any():
        assert np.all(diff[zero] == 0), what + ": mismatch where the scale is zero"
    ratio = np.max(diff[~zero] / S[~zero]) if (~zero).any() else 0.0
    assert ratio <= tol, "%s: max |diff|/S = %.3g exceeds %.3g" % (what, ratio, tol)
    return float(ratio)


def check_against_oracle(A, B, C0, got, integer, what=""):
    f32 = got.dtype == np.float32
    want = C0.copy()
    (oracle.gemm_f32_ref if f32 else oracle.gemm_f64_ref)(A, B, want)
    if integer:
        iv = np.uint32 if f32 else np.uint64
        bad = np.flatnonzero(np.ascontiguousarray(got).view(iv).ravel() != want.view(iv).ravel())
        assert bad.size == 0, "%s: %d elements differ bitwise (first flat index %d: got %r want %r)" % (
            what, bad.size, bad[0], got.ravel()[bad[0]], want.ravel()[bad[0]])
        return 0.0
    S = np.zeros(want.shape, dtype=np.float64)
    (oracle.gemm_f32_absref if f32 else oracle.gemm_f64_absref)(A, B, S)
    return check_tolerance(got, want, S, what)


def check_full_in_row_blocks(A, B, C0, got, integer, what="", block=2048):
    """Every element of `got` against the oracle, a block of complete rows at a time (row i of the result depends on
    row i of A and of C alone, so the blocks are independent calls of the same oracle routine; only one block of
    expected values and scales is alive at a time).  Returns the worst |diff| / S over all elements."""
    worst = 0.0
    for r0 in range(0, A.shape[0], block):
        r1 = min(A.shape[0], r0 + block)
        ratio = check_against_oracle(A[r0:r1], B, np.ascontiguousarray(C0[r0:r1]), got[r0:r1], integer,
                                     "%s rows %d..%d" % (what, r0, r1 - 1))
        worst = max(worst, ratio)
    return worst
