"""Pins for `C <- alpha * A @ B + beta * C` on operands addressed through two strides each
(`X(r, c) = X[r * rs + c * cs]`): facts fixed by the mathematics and by the term-by-term definition,
none of which comes from running the implementation under test.

Every pin is a function `pin(impl)` with `impl(alpha, A, B, beta, C)`: A, B and C are 2-D NumPy views
with arbitrary positive strides into larger buffers filled with a NaN sentinel; C is updated in place.
The element type follows `pins.DT`.

The paper treats strides and transposes as layout maps on the operands (Section 2.9, whose example is a
126 x 100 float matrix with access strides 128 and 2 inside a larger buffer; Section 2.15 Q4); the
arithmetic pinned is that of the full signature (see pins_general).
"""
from fractions import Fraction

import numpy as np

import pins
import pins_general as pg
from pins import assert_bitwise

# name -> (row stride, column stride) as functions of the view's shape (rows, cols)
LAYOUTS = {
    "row": lambda r, c: (c + 2, 1),                # row-major with a padded leading dimension
    "col": lambda r, c: (1, r + 3),                # column-major (the transposed view of a row-major array)
    "row_step2": lambda r, c: (2 * c + 5, 2),      # every second element of the rows of a row-major array
    "col_step3": lambda r, c: (3, 3 * r + 1),      # every third element of the columns of a column-major array
}


def place(X, layout, offset=3):
    """A fresh sentinel-filled 1-D buffer and a view of it with the named layout that holds X."""
    rows, cols = X.shape
    rs, cs = LAYOUTS[layout](max(rows, 1), max(cols, 1)) if isinstance(layout, str) else layout
    span = (max(rows, 1) - 1) * rs + (max(cols, 1) - 1) * cs + 1
    buf = np.full(offset + span + 4, np.nan, dtype=pins.DT)
    sz = buf.dtype.itemsize
    view = np.lib.stride_tricks.as_strided(buf[offset:], shape=(rows, cols), strides=(rs * sz, cs * sz))
    view[...] = X
    return buf, view


def untouched(buf, view):
    """True when every element of buf outside the view still holds the sentinel."""
    mask = np.zeros(buf.shape, dtype=bool)
    sz = buf.dtype.itemsize
    start = (view.__array_interface__["data"][0] - buf.__array_interface__["data"][0]) // sz
    if view.size:
        r = np.arange(view.shape[0])[:, None] * (view.strides[0] // sz if view.shape[0] > 1 else 0)
        c = np.arange(view.shape[1])[None, :] * (view.strides[1] // sz if view.shape[1] > 1 else 0)
        mask[(start + r + c).ravel()] = True
    return bool(np.isnan(buf[~mask]).all())


def _check_exact(impl, M, N, K, la, lb, lc, alpha, beta, seed, denom):
    A, B, C0 = pg._logical(seed, M, N, K)
    for X in (A, B, C0):
        pg._dyadic(X, denom)
    Ab, Av = place(A, la)
    Bb, Bv = place(B, lb)
    Cb, Cv = place(C0, lc)
    impl(alpha, Av, Bv, beta, Cv)
    want = pg._exact_general(alpha, A, B, beta, C0)
    for i in range(M):
        for j in range(N):
            assert np.isfinite(Cv[i, j]) and Fraction(float(Cv[i, j])) == want[i][j], "strided exact %s layouts %s alpha %g beta %g at (%d,%d): got %r want %r" % (
                (M, N, K), (la, lb, lc), alpha, beta, i, j, Cv[i, j], float(want[i][j]))
    assert untouched(Ab, Av) and untouched(Bb, Bv) and untouched(Cb, Cv), "memory outside the views changed: %s %s" % ((M, N, K), (la, lb, lc))
    assert np.array_equal(Av, A) and np.array_equal(Bv, B), "A or B was written"


def pin_strided_tiny_exact(impl, limit=3):
    """Shapes in {0..limit}^3, every operand in each of four layouts (row-major, column-major, and sampled
    versions of both), dyadic data and scalars: the result equals exact rational arithmetic bit for bit, and
    nothing outside the views changes."""
    denom = 16.0 if pins.DT == np.float32 else 1024.0
    scalars = [(1.0, 1.0), (1.0, 0.0), (0.0, 1.0), (-1.0, 0.5), (2.0, -1.5), (0.25, 3.0), (-0.75, 0.0)]
    names = list(LAYOUTS)
    seed = 900
    for M in range(limit + 1):
        for N in range(limit + 1):
            for K in range(limit + 1):
                # every pair of layouts appears for every operand pair over the sweep; all 64 triples at the largest shape
                triples = [(names[(seed + t) % 4], names[(seed // 4 + 2 * t) % 4], names[(seed // 16 + t) % 4]) for t in range(2)]
                if (M, N, K) == (limit, limit, limit):
                    triples = [(a, b, c) for a in names for b in names for c in names]
                for (la, lb, lc) in triples:
                    alpha, beta = scalars[seed % len(scalars)]
                    _check_exact(impl, M, N, K, la, lb, lc, alpha, beta, seed, denom)
                    seed += 1


def pin_strided_paper_layout(impl):
    """The layout of the paper's example, a 126 x 100 matrix with access strides 128 and 2 in a larger buffer,
    as the A operand (and, transposed, as B): small integers, so the exact integer product is the answer.
    (With 100 columns two apart a row spans 199 elements, more than the row stride: rows share elements, which
    a read-only operand may; the matrix used is whatever the view reads back.)"""
    rng = np.random.default_rng(11)
    A = rng.integers(-4, 5, size=(126, 100)).astype(pins.DT)
    B = rng.integers(-4, 5, size=(100, 9)).astype(pins.DT)
    C0 = rng.integers(-4, 5, size=(126, 9)).astype(pins.DT)
    Ab, Av = place(A, (128, 2))
    A = Av.copy()
    Bb, Bv = place(B, "row")
    Cb, Cv = place(C0, "row")
    impl(1.0, Av, Bv, 1.0, Cv)
    want = (C0.astype(np.int64) + A.astype(np.int64) @ B.astype(np.int64)).astype(pins.DT)
    assert_bitwise(np.ascontiguousarray(Cv), want, "paper layout as A")
    assert untouched(Cb, Cv) and untouched(Ab, Av)
    # the same buffer read as the 100 x 126 B operand through swapped strides
    L = rng.integers(-4, 5, size=(7, 100)).astype(pins.DT)
    Bt = np.lib.stride_tricks.as_strided(Av, shape=(100, 126), strides=(Av.strides[1], Av.strides[0]))
    C1 = np.zeros((7, 126), dtype=pins.DT)
    _, C1v = place(C1, "col")
    impl(-2.0, place(L, "col")[1], Bt, 0.0, C1v)
    want = pins.DT.type(-2.0) * (L.astype(np.int64) @ A.T.astype(np.int64)).astype(pins.DT)   # a zero sum gives -0
    assert_bitwise(np.ascontiguousarray(C1v), want, "paper layout transposed as B")


def pin_strided_integer_exact(impl, shape=(37, 29, 45), seed=4):
    """Small-integer data in every combination of the four layouts: exact in any order of summation."""
    M, N, K = shape
    rng = np.random.default_rng(seed)
    A = rng.integers(-4, 5, size=(M, K)).astype(pins.DT)
    B = rng.integers(-4, 5, size=(K, N)).astype(pins.DT)
    C0 = rng.integers(-4, 5, size=(M, N)).astype(pins.DT)
    exact = A.astype(np.int64) @ B.astype(np.int64)
    t = 0
    for la in LAYOUTS:
        for lb in LAYOUTS:
            for lc in LAYOUTS:
                alpha, beta = [(1, 1), (-2, 3), (3, 0), (1, -1)][t % 4]
                t += 1
                Ab, Av = place(A, la)
                Bb, Bv = place(B, lb)
                Cb, Cv = place(C0, lc)
                impl(float(alpha), Av, Bv, float(beta), Cv)
                want = (alpha * exact + beta * C0.astype(np.int64)).astype(pins.DT)
                assert_bitwise(np.ascontiguousarray(Cv), want, "strided integers %s alpha %d beta %d" % ((la, lb, lc), alpha, beta))
                assert untouched(Cb, Cv), "memory outside C changed, layouts %s" % ((la, lb, lc),)


def pin_strided_overlapping_reads(impl):
    """A and B are only read, so their elements may share memory: A(i, k) = v[i + k] (strides 1 and 1, a Hankel
    matrix of a vector) and B(k, j) = w[2 k + j] (strides 2 and 1)."""
    M, N, K = 13, 11, 17
    rng = np.random.default_rng(5)
    v = rng.integers(-4, 5, size=M + K).astype(pins.DT)
    w = rng.integers(-4, 5, size=2 * K + N).astype(pins.DT)
    sz = v.dtype.itemsize
    Av = np.lib.stride_tricks.as_strided(v, shape=(M, K), strides=(sz, sz))
    Bv = np.lib.stride_tricks.as_strided(w, shape=(K, N), strides=(2 * sz, sz))
    for lc in LAYOUTS:
        Cb, Cv = place(np.zeros((M, N), dtype=pins.DT), lc)
        impl(1.0, Av, Bv, 0.0, Cv)
        want = np.array([[sum(int(v[i + k]) * int(w[2 * k + j]) for k in range(K)) for j in range(N)] for i in range(M)])
        assert_bitwise(np.ascontiguousarray(Cv), want.astype(pins.DT), "overlapping reads, C %s" % lc)


def pin_strided_rounded_sequence(impl):
    """Full-precision random data: the definition fixes every rounding, whatever the layouts."""
    cases = [((3, 4, 7), 0.7310585786300049, -1.3862943611198906, ("col", "row_step2", "col_step3")),
             ((2, 9, 33), -2.718281828459045, 0.0, ("row_step2", "col", "col")),
             ((5, 3, 64), 1.0, 1.0, ("col_step3", "col_step3", "row")),
             ((4, 4, 5), 1.0, -0.3333333333333333, ("row", "col", "row_step2"))]
    for t, ((M, N, K), alpha, beta, (la, lb, lc)) in enumerate(cases):
        A, B, C0 = pg._logical(720 + t, M, N, K)
        want = pg.general_rounded_sequence(alpha, A, B, beta, C0)
        _, Av = place(A, la)
        _, Bv = place(B, lb)
        _, Cv = place(C0, lc)
        impl(alpha, Av, Bv, beta, Cv)
        assert_bitwise(np.ascontiguousarray(Cv), want, "strided rounded sequence %s %s" % ((M, N, K), (la, lb, lc)))


def pin_strided_unread_operands(impl):
    """beta == 0: C may hold NaN and is not read.  alpha == 0 or K == 0: A and B may hold NaN and are not read."""
    M, N, K = 6, 5, 7
    A, B, C0 = pg._logical(31, M, N, K, "int")
    nanA, nanB = np.full_like(A, np.nan), np.full_like(B, np.nan)
    for lc in LAYOUTS:
        _, Cv = place(np.full((M, N), np.nan, dtype=pins.DT), lc)
        impl(2.0, place(A, "col")[1], place(B, "row_step2")[1], 0.0, Cv)
        want = (2 * (A.astype(np.int64) @ B.astype(np.int64))).astype(pins.DT)
        assert_bitwise(np.ascontiguousarray(Cv), want, "beta == 0 must not read C (%s)" % lc)
        _, Cv = place(C0, lc)
        impl(0.0, place(nanA, "col")[1], place(nanB, "col")[1], -3.0, Cv)
        assert_bitwise(np.ascontiguousarray(Cv), pins.DT.type(-3.0) * C0, "alpha == 0 must not read A, B (%s)" % lc)
        _, Cv = place(np.full((M, N), np.nan, dtype=pins.DT), lc)
        impl(0.0, place(nanA, "row")[1], place(nanB, "row")[1], 0.0, Cv)
        assert_bitwise(np.ascontiguousarray(Cv), np.zeros((M, N), dtype=pins.DT), "alpha == beta == 0 gives +0 (%s)" % lc)
    _, Cv = place(C0, "col_step3")
    impl(1.0, place(np.zeros((M, 0), dtype=pins.DT), "row")[1], place(np.zeros((0, N), dtype=pins.DT), "row")[1], 0.5, Cv)
    assert_bitwise(np.ascontiguousarray(Cv), (C0.astype(np.float64) * 0.5).astype(pins.DT), "K == 0 scales C by beta")


ALL_PINS = [pin_strided_tiny_exact, pin_strided_paper_layout, pin_strided_integer_exact, pin_strided_overlapping_reads,
            pin_strided_rounded_sequence, pin_strided_unread_operands]


def as_general_impl(strided_impl, c_layout):
    """Adapter: run a pin of the transposed signature (pins_general) through a strided implementation.  The stored
    operands become transposed views; C is used in place (row-major) or through a column-major copy."""
    def impl(ta, tb, alpha, A, B, beta, C):
        Av = A.T if ta else A
        Bv = B.T if tb else B
        if c_layout == "row":
            strided_impl(alpha, Av, Bv, beta, C)
        else:
            _, Cv = place(C, c_layout)
            strided_impl(alpha, Av, Bv, beta, Cv)
            C[...] = Cv
    return impl
