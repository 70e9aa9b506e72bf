"""Pins for an fp64 `C += A @ B` implementation: facts fixed by the paper or by
mathematics, none of which comes from running the implementation under test.

Every pin is a function `pin(impl)` where `impl(A, B, C)` updates the 2-D
float64 view C in place (views may be padded: row stride > width).  A pin
raises AssertionError when the fact does not hold.  They are applied to the
CPU oracle (which they are meant to pin), to deliberately wrong variants (to
show that a plausible mistake is caught) and, through a device adapter, the
order-independent ones are reused on the HIP path.
"""
import contextlib
import os
from fractions import Fraction

import numpy as np

from paper_2003_00532_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

# The element type the pins are stated for.  float64 is the path's own precision; the float32 variant
# (the paper's Section 2.13 substitution) re-uses every pin with u = 2^-24 via `with precision(np.float32)`.
DT = np.dtype(np.float64)


@contextlib.contextmanager
def precision(dtype):
    global DT
    old, DT = DT, np.dtype(dtype)
    try:
        yield
    finally:
        DT = old


def mant_bits():
    return 24 if DT == np.float32 else 53


def bits(x):
    x = np.ascontiguousarray(x)
    return x.view(np.uint32 if x.dtype == np.float32 else np.uint64)


def rn(x: Fraction) -> float:
    """Round an exact rational to the nearest DT value, ties to even (normal range only)."""
    if x == 0:
        return 0.0
    p = mant_bits()
    sign = -1 if x < 0 else 1
    x = abs(x)
    e = x.numerator.bit_length() - x.denominator.bit_length()
    if Fraction(2) ** e > x:
        e -= 1
    assert Fraction(2) ** e <= x < Fraction(2) ** (e + 1)
    scaled = x / Fraction(2) ** (e - p + 1)          # in [2^(p-1), 2^p)
    q, r = divmod(scaled.numerator, scaled.denominator)
    twice = 2 * r
    if twice > scaled.denominator or (twice == scaled.denominator and (q & 1)):
        q += 1
    return float(sign * Fraction(q) * Fraction(2) ** (e - p + 1))


def ones(shape, value=1.0):
    return np.full(shape, value, dtype=DT)


def zeros(shape):
    return np.zeros(shape, dtype=DT)


def eye(n):
    return np.eye(n, dtype=DT)


def assert_bitwise(got, want, what=""):
    got = np.ascontiguousarray(got)
    want = np.ascontiguousarray(want)
    assert got.shape == want.shape, what
    bad = np.flatnonzero(bits(got).ravel() != bits(want).ravel())
    if bad.size:
        k = bad[0]
        raise AssertionError("%s: %d of %d elements differ bitwise; first at flat %d: got %r want %r"
                             % (what, bad.size, got.size, k, got.ravel()[k], want.ravel()[k]))


def _mat(seed, tag, rows, cols, ld=None, kind="int"):
    return synth.matrix(seed, tag, rows, cols, ld, kind, DT)


def _abs_product(A, B):
    return np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64))


# ---------------------------------------------------------------- closed forms

def pin_paper_all_ones(impl, shapes=None):
    """Section 2.1 driver input: all-ones operands give c_in + K everywhere."""
    rows = []
    with open(os.path.join(GOLDEN, "paper_all_ones.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                M, N, K, cin, want = line.split()
                rows.append((int(M), int(N), int(K), float(cin), float(want)))
    for M, N, K, cin, want in rows:
        if shapes is not None and (M, N, K) not in shapes:
            continue
        A = ones((M, K)); B = ones((K, N)); C = ones((M, N), cin)
        impl(A, B, C)
        assert_bitwise(C, ones((M, N), want), "all-ones %dx%dx%d" % (M, N, K))


def pin_all_ones_small(impl):
    for (M, N, K) in [(1, 1, 1), (3, 5, 7), (17, 33, 65), (64, 48, 200)]:
        A = ones((M, K)); B = ones((K, N)); C = ones((M, N))
        impl(A, B, C)
        assert_bitwise(C, ones((M, N), 1.0 + K), "ones %s" % ((M, N, K),))


def pin_identity(impl):
    """A = I gives RN(C + B) (one non-zero product per element, the rest add 0); B = I gives RN(C + A)."""
    n = 37
    _, X = _mat(5, synth.TAG_B, n, 29, kind="uniform")
    _, C0 = _mat(5, synth.TAG_C, n, 29, kind="uniform")
    C = C0.copy()
    impl(eye(n), X, C)
    assert_bitwise(C, C0 + X, "A = I")
    _, Y = _mat(6, synth.TAG_A, 23, n, kind="uniform")
    _, D0 = _mat(6, synth.TAG_C, 23, n, kind="uniform")
    D = D0.copy()
    impl(Y, eye(n), D)
    assert_bitwise(D, D0 + Y, "B = I")


def pin_column_sums(impl):
    """A = ones: every row of the update is the vector of column sums of B (integers, exact)."""
    M, N, K = 9, 41, 53
    _, B = _mat(7, synth.TAG_B, K, N)
    _, C0 = _mat(7, synth.TAG_C, M, N)
    C = C0.copy()
    impl(ones((M, K)), B, C)
    want = C0 + B.astype(np.int64).sum(axis=0)[None, :].astype(DT)
    assert_bitwise(C, want, "column sums")
    # and B = ones: row sums of A
    _, A = _mat(8, synth.TAG_A, M, K)
    C = C0.copy()
    impl(A, ones((K, N)), C)
    want = C0 + A.astype(np.int64).sum(axis=1)[:, None].astype(DT)
    assert_bitwise(C, want, "row sums")


def pin_rank_one(impl):
    """K = 1: the update is the outer product, a single exactly-representable product per element."""
    M, N = 19, 23
    _, a = _mat(9, synth.TAG_A, M, 1)
    _, b = _mat(9, synth.TAG_B, 1, N)
    _, C0 = _mat(9, synth.TAG_C, M, N)
    C = C0.copy()
    impl(a, b, C)
    assert_bitwise(C, C0 + np.outer(a[:, 0], b[0, :]), "rank one")


def pin_one_hot_index(impl):
    """A has a single 1 at (i0, k0): the update copies row k0 of B into row i0 of C, nothing else.
    Catches transposed operands and swapped indices even on non-square shapes."""
    M, N, K = 6, 11, 8
    _, B = _mat(10, synth.TAG_B, K, N)
    for (i0, k0) in [(0, 0), (5, 7), (2, 6), (4, 1)]:
        A = zeros((M, K)); A[i0, k0] = 1.0
        C = zeros((M, N))
        impl(A, B, C)
        want = zeros((M, N)); want[i0, :] = B[k0, :]
        assert_bitwise(C, want, "one-hot A at %s" % ((i0, k0),))
    _, A = _mat(10, synth.TAG_A, M, K)
    for (k0, j0) in [(0, 0), (7, 10), (3, 9)]:
        Bh = zeros((K, N)); Bh[k0, j0] = 1.0
        C = zeros((M, N))
        impl(A, Bh, C)
        want = zeros((M, N)); want[:, j0] = A[:, k0]
        assert_bitwise(C, want, "one-hot B at %s" % ((k0, j0),))


# ------------------------------------------------- exact rational brute force

def _exact(A, B, C0):
    M, K = A.shape
    N = B.shape[1]
    out = [[Fraction(float(C0[i, j])) for j in range(N)] for i in range(M)]
    for i in range(M):
        for k in range(K):
            a = Fraction(float(A[i, k]))
            for j in range(N):
                out[i][j] += a * Fraction(float(B[k, j]))
    return out


def pin_tiny_exact(impl, limit=5):
    """All shapes in {0..limit}^3 with padded leading dimensions, on small integers and on dyadic
    rationals (multiples of 2^-10 in [-1, 1]): every partial sum is exactly representable, so the
    result must equal exact rational arithmetic bit for bit."""
    seed = 11
    for M in range(limit + 1):
        for N in range(limit + 1):
            for K in range(limit + 1):
                for kind in ("int", "dyadic"):
                    k = "int" if kind == "int" else "uniform"
                    Ab, A = synth.matrix(seed, synth.TAG_A, M, K, K + 2, k, DT)
                    Bb, B = synth.matrix(seed, synth.TAG_B, K, N, N + 3, k, DT)
                    Cb, C = synth.matrix(seed, synth.TAG_C, M, N, N + 1, k, DT)
                    if kind == "dyadic":
                        for X in (A, B, C):
                            X[...] = (np.round(X.astype(np.float64) * 1024.0) / 1024.0).astype(DT)
                    C0 = C.copy()
                    impl(A, B, C)
                    want = _exact(A, B, C0)
                    for i in range(M):
                        for j in range(N):
                            w = want[i][j]
                            assert Fraction(float(C[i, j])) == w, \
                                "tiny exact %s %s at (%d,%d): got %r want %r" % ((M, N, K), kind, i, j, C[i, j], float(w))
                    assert synth.padding_intact(Ab, K) and synth.padding_intact(Bb, N) and synth.padding_intact(Cb, N), \
                        "padding touched at %s" % ((M, N, K),)
                    seed += 1


def rounded_sequence(A, B, C0):
    """Step-by-step emulation with exact rationals and correctly rounded conversions:
    p = RN(a*b), c = RN(c + p), k ascending, starting from c_in (Section 2.1 loop body)."""
    M, K = A.shape
    N = B.shape[1]
    out = np.empty((M, N), dtype=DT)
    for i in range(M):
        for j in range(N):
            c = float(C0[i, j])
            for k in range(K):
                p = rn(Fraction(float(A[i, k])) * Fraction(float(B[k, j])))
                c = rn(Fraction(c) + Fraction(p))
            out[i, j] = c
    return out


def pin_rounded_sequence(impl):
    """Full-precision random doubles: the definition fixes every rounding, so the result is bitwise
    the emulated sequence.  rn() rounds an exact rational to the nearest value, ties to even."""
    for t, (M, N, K) in enumerate([(3, 4, 7), (2, 9, 33), (5, 3, 64)]):
        _, A = synth.matrix(100 + t, synth.TAG_A, M, K, K + 1, "uniform", DT)
        _, B = synth.matrix(100 + t, synth.TAG_B, K, N, N + 2, "uniform", DT)
        _, C = synth.matrix(100 + t, synth.TAG_C, M, N, N + 5, "uniform", DT)
        want = rounded_sequence(A, B, C.copy())
        impl(A, B, C)
        assert_bitwise(C, want, "rounded sequence %s" % ((M, N, K),))


def pin_rounding_cases(impl):
    """Hand-derived binary64 cases: unfused product, ascending k, start from c_in, ties to even."""
    fixture = "rounding_cases_f32.txt" if DT == np.float32 else "rounding_cases.txt"
    with open(os.path.join(GOLDEN, fixture)) as f:
        for line in f:
            if not line.strip() or line.startswith("#"):
                continue
            name, cin, a, b, want = [s.strip() for s in line.split("|")]
            a = [float.fromhex(x) for x in a.split()]
            b = [float.fromhex(x) for x in b.split()]
            K = len(a)
            assert len(b) == K
            # embed the case at position (1, 2) of a 3x4 problem; other entries are zero
            A = zeros((3, K)); B = zeros((K, 4)); C = zeros((3, 4))
            A[1, :] = a; B[:, 2] = b; C[1, 2] = float.fromhex(cin)
            impl(A, B, C)
            w = zeros((3, 4)); w[1, 2] = float.fromhex(want)
            assert_bitwise(C, w, "rounding case " + name)


# ------------------------------------------------------------ integer exactness

def pin_integer_exact(impl, shape=(256, 256, 256), lds=None, seed=0):
    """Entries in {-4..4}: |sum| <= 16 K + 4, far below 2^53 (and below 2^24 for K < 2^20), so every
    partial sum is an exact integer in any order; the result must equal int64 arithmetic bit for bit."""
    M, N, K = shape
    lda, ldb, ldc = lds or (K, N, N)
    Ab, A = synth.matrix(seed, synth.TAG_A, M, K, lda, "int", DT)
    Bb, B = synth.matrix(seed, synth.TAG_B, K, N, ldb, "int", DT)
    Cb, C = synth.matrix(seed, synth.TAG_C, M, N, ldc, "int", DT)
    want = (C.astype(np.int64) + A.astype(np.int64) @ B.astype(np.int64)).astype(DT)
    impl(A, B, C)
    assert_bitwise(C, want, "integer exact %s" % (shape,))
    assert synth.padding_intact(Ab, K) and synth.padding_intact(Bb, N) and synth.padding_intact(Cb, N)


# ------------------------------------------------------------------ error bound

def pin_error_bound(impl, shape=(256, 256, 256), samples=300, seed=0):
    """Uniform[-1,1) inputs: against the exactly rounded value, the recursive-summation bound
    |c_hat - c| <= gamma_{K+1} (|c_in| + S_ij), gamma_n = n u / (1 - n u), u = 2^-53 (2^-24 in float32), must hold."""
    M, N, K = shape
    _, A = synth.matrix(seed, synth.TAG_A, M, K, None, "uniform", DT)
    _, B = synth.matrix(seed, synth.TAG_B, K, N, None, "uniform", DT)
    _, C = synth.matrix(seed, synth.TAG_C, M, N, None, "uniform", DT)
    C0 = C.copy()
    impl(A, B, C)
    u = Fraction(1, 2 ** mant_bits())
    gamma = (K + 1) * u / (1 - (K + 1) * u)
    rng = np.random.default_rng(seed + 1)
    pts = {(0, 0), (M - 1, N - 1), (0, N - 1), (M - 1, 0)}
    while len(pts) < samples:
        pts.add((int(rng.integers(M)), int(rng.integers(N))))
    worst = Fraction(0)
    for (i, j) in sorted(pts):
        exact = Fraction(float(C0[i, j]))
        S = abs(exact)
        for k in range(K):
            t = Fraction(float(A[i, k])) * Fraction(float(B[k, j]))
            exact += t
            S += abs(t)
        err = abs(Fraction(float(C[i, j])) - exact)
        assert err <= gamma * S, "error bound broken at (%d,%d): err %g bound %g" % (i, j, float(err), float(gamma * S))
        worst = max(worst, err / S)
    return float(worst)


# -------------------------------------------------------------------- invariants

def pin_block_split_invariance(impl, bitwise_k=True):
    """Row and column blocks are independent (bitwise).  Splitting K into two consecutive calls
    continues the same ascending sequence, so it is bitwise too for an implementation that follows
    the definition's order (bitwise_k=False relaxes that to the tolerance for other orders)."""
    M, N, K = 21, 34, 77
    _, A = synth.matrix(21, synth.TAG_A, M, K, K + 3, "uniform", DT)
    _, B = synth.matrix(21, synth.TAG_B, K, N, N + 6, "uniform", DT)
    _, C0 = synth.matrix(21, synth.TAG_C, M, N, N + 2, "uniform", DT)
    whole = C0.copy(); impl(A, B, whole)
    parts = C0.copy()
    for (r0, r1) in [(0, 8), (8, 21)]:
        for (c0, c1) in [(0, 13), (13, 34)]:
            impl(A[r0:r1, :], B[:, c0:c1], parts[r0:r1, c0:c1])
    assert_bitwise(parts, whole, "row/column block split")
    ks = C0.copy()
    impl(A[:, :30], B[:30, :], ks)
    impl(A[:, 30:], B[30:, :], ks)
    if bitwise_k:
        assert_bitwise(ks, whole, "k split")
    else:
        S = _abs_product(A, B)
        tol = 2.0 ** -19 if DT == np.float32 else 1e-13
        assert np.all(np.abs(ks.astype(np.float64) - whole) <= tol * S)


def pin_ld_independence(impl):
    """The result does not depend on the leading dimensions; padding is neither read (the NaN
    sentinel would leak) nor written."""
    M, N, K = 13, 27, 31
    _, A = synth.matrix(31, synth.TAG_A, M, K, None, "uniform", DT)
    _, B = synth.matrix(31, synth.TAG_B, K, N, None, "uniform", DT)
    _, C0 = synth.matrix(31, synth.TAG_C, M, N, None, "uniform", DT)
    dense = C0.copy(); impl(A, B, dense)
    Ab, Ap = synth.matrix(31, synth.TAG_A, M, K, K + 9, "uniform", DT)
    Bb, Bp = synth.matrix(31, synth.TAG_B, K, N, N + 4, "uniform", DT)
    Cb, Cp = synth.matrix(31, synth.TAG_C, M, N, N + 7, "uniform", DT)
    impl(Ap, Bp, Cp)
    assert not np.isnan(Cp).any(), "NaN padding leaked into C"
    assert_bitwise(Cp, dense, "ld independence")
    assert synth.padding_intact(Ab, K) and synth.padding_intact(Bb, N) and synth.padding_intact(Cb, N)


def pin_degenerate(impl):
    """M*N = 0 is a no-op; K = 0 leaves C unchanged."""
    _, C0 = synth.matrix(41, synth.TAG_C, 4, 6, 8, "uniform", DT)
    C = C0.copy()
    impl(zeros((4, 0)), zeros((0, 6)), C)
    assert_bitwise(C, C0, "K = 0")
    impl(zeros((0, 5)), zeros((5, 6)), zeros((0, 6)))
    impl(zeros((4, 5)), zeros((5, 0)), zeros((4, 0)))


ORDER_DEPENDENT = [pin_rounded_sequence, pin_rounding_cases]

ALL_PINS = [pin_all_ones_small, pin_identity, pin_column_sums, pin_rank_one, pin_one_hot_index,
            pin_tiny_exact, pin_rounded_sequence, pin_rounding_cases, pin_integer_exact,
            pin_error_bound, pin_block_split_invariance, pin_ld_independence, pin_degenerate]
