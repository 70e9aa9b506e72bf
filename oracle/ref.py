"""ctypes binding of the CPU oracle (oracle/gemm_ref.c).  Test infrastructure.

All functions take 2-D float64 NumPy arrays whose last axis is contiguous; the
leading dimension is taken from the row stride, so padded views (a[:, :K] of
a wider buffer) are passed without copying and their padding is never touched.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build()
        lib = ctypes.CDLL(path)
        i64, dp = ctypes.c_int64, ctypes.c_void_p
        for name in ("gemm_f64_ref", "gemm_f64_ref_ijk", "gemm_f64_absref"):
            fn = getattr(lib, name)
            fn.argtypes = [i64, i64, i64, dp, i64, dp, i64, dp, i64]
            fn.restype = ctypes.c_int
        for name in ("gemm_f32_ref", "gemm_f32_ref_ijk", "gemm_f32_absref"):
            fn = getattr(lib, name)
            fn.argtypes = [i64, i64, i64, dp, i64, dp, i64, dp, i64]
            fn.restype = ctypes.c_int
        lib.gemm_f64_general_ref.argtypes = [ctypes.c_int, ctypes.c_int, i64, i64, i64, ctypes.c_double, dp, i64,
                                             dp, i64, ctypes.c_double, dp, i64]
        lib.gemm_f64_general_ref.restype = ctypes.c_int
        lib.gemm_f32_general_ref.argtypes = [ctypes.c_int, ctypes.c_int, i64, i64, i64, ctypes.c_float, dp, i64,
                                             dp, i64, ctypes.c_float, dp, i64]
        lib.gemm_f32_general_ref.restype = ctypes.c_int
        lib.gemm_f64_strided_ref.argtypes = [i64, i64, i64, ctypes.c_double, dp, i64, i64, dp, i64, i64,
                                             ctypes.c_double, dp, i64, i64]
        lib.gemm_f64_strided_ref.restype = ctypes.c_int
        lib.gemm_f32_strided_ref.argtypes = [i64, i64, i64, ctypes.c_float, dp, i64, i64, dp, i64, i64,
                                             ctypes.c_float, dp, i64, i64]
        lib.gemm_f32_strided_ref.restype = ctypes.c_int
        lib.gemm_f64_ref_threads.restype = ctypes.c_int
        lib.gemm_f64_ref_set_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _ld(x: np.ndarray) -> int:
    assert x.dtype in (np.float64, np.float32) and x.ndim == 2
    sz = x.dtype.itemsize
    if x.size == 0:
        # no element is touched; any legal leading dimension will do
        return max(1, x.shape[1], x.strides[0] // sz if x.strides[0] % sz == 0 else 1)
    if x.shape[1] > 1:
        assert x.strides[1] == sz, "last axis must be contiguous"
    if x.shape[0] > 1:
        assert x.strides[0] % sz == 0 and x.strides[0] > 0
        return x.strides[0] // sz
    return max(1, x.shape[1])


def _call(name, A, B, C, lda=None, ldb=None, ldc=None):
    want = np.float32 if "f32" in name else np.float64
    assert A.dtype == want and B.dtype == want, "%s takes %s operands" % (name, np.dtype(want).name)
    assert C.dtype == (np.float64 if name.endswith("absref") else want)
    M, K = A.shape
    K2, N = B.shape
    assert K2 == K and C.shape == (M, N)
    assert C.flags.writeable
    fn = getattr(_load(), name)
    rc = fn(M, N, K, A.ctypes.data, lda or _ld(A), B.ctypes.data, ldb or _ld(B),
            C.ctypes.data, ldc or _ld(C))
    if rc != 0:
        raise ValueError("%s failed with code %d" % (name, rc))
    return C


def gemm_f64_ref(A, B, C):
    """C += A @ B, the definition (Section 2.1 loop nest), in place; returns C."""
    return _call("gemm_f64_ref", A, B, C)


def gemm_f64_ref_ijk(A, B, C):
    """Same result through the literal i-j-k nest (serial, slow)."""
    return _call("gemm_f64_ref_ijk", A, B, C)


def gemm_f64_absref(A, B, C):
    """C += |A| @ |B| by the same loop; with C = 0 gives the tolerance scale S."""
    return _call("gemm_f64_absref", A, B, C)


def gemm_f32_ref(A, B, C):
    """float32 C += A @ B, every product and sum rounded to binary32 (Section 2.13), in place."""
    return _call("gemm_f32_ref", A, B, C)


def gemm_f32_ref_ijk(A, B, C):
    return _call("gemm_f32_ref_ijk", A, B, C)


def gemm_f32_absref(A, B, S):
    """float64 S += |A| @ |B| for float32 operands: the tolerance scale."""
    return _call("gemm_f32_absref", A, B, S)


def gemm_general_ref(transa, transb, alpha, A, B, beta, C):
    """C <- alpha * op(A) @ op(B) + beta * C in place (oracle/gemm_general_ref.c); returns C.

    A and B are the arrays as stored: A is (K, M) when transa, B is (N, K) when transb.  The element
    type (float64 or float32) is taken from C; alpha and beta are converted to it.
    """
    f32 = C.dtype == np.float32
    want = np.float32 if f32 else np.float64
    assert A.dtype == want and B.dtype == want and C.dtype == want and C.flags.writeable
    M, N = C.shape
    K = A.shape[0] if transa else A.shape[1]
    assert A.shape == ((K, M) if transa else (M, K)), "A shape"
    assert B.shape == ((N, K) if transb else (K, N)), "B shape"
    fn = getattr(_load(), "gemm_f32_general_ref" if f32 else "gemm_f64_general_ref")
    rc = fn(int(bool(transa)), int(bool(transb)), M, N, K, float(want(alpha)), A.ctypes.data, _ld(A),
            B.ctypes.data, _ld(B), float(want(beta)), C.ctypes.data, _ld(C))
    if rc != 0:
        raise ValueError("gemm_general_ref failed with code %d" % rc)
    return C


def general_scale(transa, transb, alpha, A, B, beta, C0):
    """float64 S = |alpha| * |op(A)| @ |op(B)| + |beta * C0|: the scale of the elementwise tolerance of the
    general operation, obtained by running the binary64 oracle on absolute values (C0 is ignored when beta == 0).
    Pinned against exact rational arithmetic by tests/test_oracle_scale_pins.py."""
    S = np.abs(C0.astype(np.float64))
    if beta == 0:
        S = np.zeros(C0.shape, dtype=np.float64)  # C0 is not read then and may hold NaN
    return gemm_general_ref(transa, transb, abs(float(alpha)), np.abs(A.astype(np.float64)),
                            np.abs(B.astype(np.float64)), abs(float(beta)), np.ascontiguousarray(S))


def element_strides(x: np.ndarray):
    """(row stride, column stride) of a 2-D view in elements; an axis of extent 0 or 1 reports 1."""
    assert x.ndim == 2
    sz = x.dtype.itemsize
    out = []
    for axis in (0, 1):
        if x.shape[axis] > 1 and x.size:
            assert x.strides[axis] > 0 and x.strides[axis] % sz == 0, "strides must be positive element multiples"
            out.append(x.strides[axis] // sz)
        else:
            out.append(1)
    return tuple(out)


def gemm_strided_ref(alpha, A, B, beta, C):
    """C <- alpha * A @ B + beta * C in place for 2-D views with any positive strides (oracle/gemm_strided_ref.c):
    row-major, column-major (a transposed view), or regularly sampled sub-matrices of either.  Returns C."""
    f32 = C.dtype == np.float32
    want = np.float32 if f32 else np.float64
    assert A.dtype == want and B.dtype == want and C.dtype == want and C.flags.writeable
    M, N = C.shape
    K = A.shape[1]
    assert A.shape == (M, K) and B.shape == (K, N)
    (rsa, csa), (rsb, csb), (rsc, csc) = element_strides(A), element_strides(B), element_strides(C)
    fn = getattr(_load(), "gemm_f32_strided_ref" if f32 else "gemm_f64_strided_ref")
    rc = fn(M, N, K, float(want(alpha)), A.ctypes.data, rsa, csa, B.ctypes.data, rsb, csb, float(want(beta)),
            C.ctypes.data, rsc, csc)
    if rc != 0:
        raise ValueError("gemm_strided_ref failed with code %d" % rc)
    return C


def raw(name):
    """The raw C entry point (for argument-validation tests)."""
    return getattr(_load(), name)


def ref_threads() -> int:
    return int(_load().gemm_f64_ref_threads())


def set_ref_threads(n: int) -> None:
    _load().gemm_f64_ref_set_threads(int(n))


def _ref_fn(A):
    return gemm_f32_ref if A.dtype == np.float32 else gemm_f64_ref


def ref_rows(A, B, C0, rows):
    """Oracle result for selected rows only: out[r] = C0[rows[r]] + A[rows[r]] @ B.

    Row i of the result depends on row i of A and of C alone, so the selected
    rows are gathered into compact arrays and the same oracle routine is run on
    them; nothing else is computed.
    """
    rows = np.asarray(rows, dtype=np.int64)
    Ar = np.ascontiguousarray(A[rows, :])
    Cr = np.ascontiguousarray(C0[rows, :])
    return _ref_fn(A)(Ar, B, Cr)


def abs_rows(A, B, rows):
    """Tolerance scale S[r, j] = sum_k |A[rows[r], k] * B[k, j]| for selected rows."""
    rows = np.asarray(rows, dtype=np.int64)
    Ar = np.ascontiguousarray(A[rows, :])
    S = np.zeros((len(rows), B.shape[1]), dtype=np.float64)
    return (gemm_f32_absref if A.dtype == np.float32 else gemm_f64_absref)(Ar, B, S)
