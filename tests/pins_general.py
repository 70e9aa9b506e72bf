"""Pins for `C <- alpha * op(A) @ op(B) + beta * C` (row-major, op = identity or transpose): facts
fixed by the mathematics and by the term-by-term definition, none of which comes from running the
implementation under test.

Every pin is a function `pin(impl)` with `impl(transa, transb, alpha, A, B, beta, C)` updating the 2-D
view C in place; A and B are given AS STORED (A is K x M when transa, B is N x K when transb) and may be
padded views.  The element type follows `pins.DT` (float64, or float32 under `pins.precision`).

The definition pinned here (the paper only names the operation, Section 2.15 Q4, and says that the
cases alpha, beta in {0, 1} fold away; Section 2.2 makes a transpose a layout map on the operand):
    s = 0; k ascending: s = RN(s + RN(opA(i,k) * opB(k,j)));  t = RN(alpha * s);
    c = t if beta == 0 (C unread) else RN(t + RN(beta * c_in));  alpha == 0 or K == 0: c = beta * c_in,
    A and B unread.
"""
import os
from fractions import Fraction

import numpy as np

from paper_2003_00532_amd import synth

import pins
from pins import assert_bitwise, rn

COMBOS = [(0, 0), (0, 1), (1, 0), (1, 1)]


def stored(X, trans, pad=0):
    """The array as stored for logical operand X: X itself or its transpose, in a fresh sentinel-padded buffer."""
    L = X.T if trans else X
    buf = synth.padded(L.shape[0], L.shape[1], max(1, L.shape[1] + pad), dtype=pins.DT)
    buf[:, :L.shape[1]] = L
    return buf, buf[:, :L.shape[1]]


def _logical(seed, M, N, K, kind="uniform"):
    _, A = synth.matrix(seed, synth.TAG_A, M, K, None, kind, pins.DT)
    _, B = synth.matrix(seed, synth.TAG_B, K, N, None, kind, pins.DT)
    _, C = synth.matrix(seed, synth.TAG_C, M, N, None, kind, pins.DT)
    return A, B, C


def _dyadic(X, denom):
    X[...] = (np.round(X.astype(np.float64) * denom) / denom).astype(pins.DT)


def _exact_general(alpha, A, B, beta, C0):
    """Exact rational alpha * A B + beta * C0 on logical operands (beta == 0: C0 ignored)."""
    M, K = A.shape
    N = B.shape[1]
    al, be = Fraction(float(alpha)), Fraction(float(beta))
    out = [[Fraction(0)] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            s = Fraction(0)
            for k in range(K):
                s += Fraction(float(A[i, k])) * Fraction(float(B[k, j]))
            out[i][j] = al * s + (be * Fraction(float(C0[i, j])) if be != 0 else 0)
    return out


def pin_general_tiny_exact(impl, limit=3):
    """All shapes in {0..limit}^3, the four transpose combinations, dyadic alpha and beta (0, 1 and others),
    padded leading dimensions, data on a dyadic grid coarse enough that every intermediate value is
    exactly representable: the result must equal exact rational arithmetic bit for bit."""
    denom = 16.0 if pins.DT == np.float32 else 1024.0
    scalars = [(1.0, 1.0), (1.0, 0.0), (0.0, 1.0), (0.0, 0.0), (-1.0, 0.5), (2.0, -1.5), (0.25, 3.0), (-0.75, 0.0)]
    seed = 500
    for M in range(limit + 1):
        for N in range(limit + 1):
            for K in range(limit + 1):
                for (ta, tb) in COMBOS:
                    alpha, beta = scalars[seed % len(scalars)]
                    A, B, C0 = _logical(seed, M, N, K)
                    for X in (A, B, C0):
                        _dyadic(X, denom)
                    Ab, As = stored(A, ta, pad=2)
                    Bb, Bs = stored(B, tb, pad=3)
                    Cb, C = stored(C0, 0, pad=1)
                    impl(ta, tb, alpha, As, Bs, beta, C)
                    want = _exact_general(alpha, A, B, beta, C0)
                    for i in range(M):
                        for j in range(N):
                            assert Fraction(float(C[i, j])) == want[i][j], \
                                "tiny exact %s trans %s alpha %g beta %g at (%d,%d): got %r want %r" % (
                                    (M, N, K), (ta, tb), alpha, beta, i, j, C[i, j], float(want[i][j]))
                    assert synth.padding_intact(Ab, As.shape[1]) and synth.padding_intact(Bb, Bs.shape[1]) \
                        and synth.padding_intact(Cb, N), "padding touched at %s" % ((M, N, K),)
                    seed += 1


def general_rounded_sequence(alpha, A, B, beta, C0):
    """The definition step by step on logical operands, every operation an exact rational rounded once."""
    M, K = A.shape
    N = B.shape[1]
    out = np.empty((M, N), dtype=pins.DT)
    alpha, beta = float(pins.DT.type(alpha)), float(pins.DT.type(beta))
    for i in range(M):
        for j in range(N):
            if alpha == 0 or K == 0:
                out[i, j] = rn(Fraction(beta) * Fraction(float(C0[i, j]))) if beta != 0 else 0.0
                continue
            s = 0.0
            for k in range(K):
                p = rn(Fraction(float(A[i, k])) * Fraction(float(B[k, j])))
                s = rn(Fraction(s) + Fraction(p))
            t = rn(Fraction(alpha) * Fraction(s))
            if beta == 0:
                out[i, j] = t
            else:
                u = rn(Fraction(beta) * Fraction(float(C0[i, j])))
                out[i, j] = rn(Fraction(t) + Fraction(u))
    return out


def pin_general_rounded_sequence(impl):
    """Full-precision random data and scalars: the definition fixes every rounding, so the result is bitwise
    the emulated sequence, for every transpose combination."""
    cases = [((3, 4, 7), 0.7310585786300049, -1.3862943611198906), ((2, 9, 33), -2.718281828459045, 0.0),
             ((5, 3, 64), 1.0, 1.0), ((4, 4, 5), 1.0, -0.3333333333333333), ((3, 2, 9), 0.0, 1.7320508075688772)]
    for t, ((M, N, K), alpha, beta) in enumerate(cases):
        A, B, C0 = _logical(700 + t, M, N, K)
        want = general_rounded_sequence(alpha, A, B, beta, C0)
        for (ta, tb) in COMBOS:
            _, As = stored(A, ta, pad=1)
            _, Bs = stored(B, tb, pad=2)
            _, C = stored(C0, 0, pad=5)
            impl(ta, tb, alpha, As, Bs, beta, C)
            assert_bitwise(C, want, "general rounded sequence %s trans %s" % ((M, N, K), (ta, tb)))


def pin_general_rounding_cases(impl):
    """Hand-derived cases whose result depends on where alpha and beta are applied and on what is fused."""
    fixture = "rounding_cases_general_f32.txt" if pins.DT == np.float32 else "rounding_cases_general.txt"
    with open(os.path.join(pins.GOLDEN, fixture)) as f:
        for line in f:
            if not line.strip() or line.startswith("#"):
                continue
            name, alpha, beta, cin, a, b, want = [s.strip() for s in line.split("|")]
            a = [float.fromhex(x) for x in a.split()]
            b = [float.fromhex(x) for x in b.split()]
            K = len(a)
            assert len(b) == K
            for (ta, tb) in COMBOS:
                # the case sits at (1, 2) of a 3 x 4 problem; every other entry is zero
                A = pins.zeros((3, K)); B = pins.zeros((K, 4)); C = pins.zeros((3, 4))
                A[1, :] = a; B[:, 2] = b; C[1, 2] = float.fromhex(cin)
                _, As = stored(A, ta)
                _, Bs = stored(B, tb)
                impl(ta, tb, float.fromhex(alpha), As, Bs, float.fromhex(beta), C)
                w = pins.zeros((3, 4)); w[1, 2] = float.fromhex(want)
                assert_bitwise(C, w, "general rounding case %s trans %s" % (name, (ta, tb)))


def pin_general_all_ones(impl):
    """All-ones operands: every element is alpha * K + beta (dyadic scalars, exact in any order)."""
    for (M, N, K, alpha, beta) in [(3, 5, 7, 2.0, 0.5), (17, 9, 33, -0.25, 4.0), (8, 8, 100, 1.0, 0.0), (6, 4, 12, 0.0, -2.0)]:
        for (ta, tb) in COMBOS:
            A = pins.ones((K, M) if ta else (M, K)); B = pins.ones((N, K) if tb else (K, N)); C = pins.ones((M, N))
            impl(ta, tb, alpha, A, B, beta, C)
            assert_bitwise(C, pins.ones((M, N), alpha * K + beta), "general all ones %s" % ((M, N, K, alpha, beta),))


def pin_general_one_hot(impl):
    """Non-square one-hot operands under every transpose combination: a single 1 at logical (i0, k0) of op(A)
    copies alpha * row k0 of op(B) into row i0 of C.  Catches a transpose applied to the wrong operand, a
    leading dimension read as if the operand were not transposed, and swapped indices."""
    M, N, K = 6, 11, 8
    _, B = synth.matrix(10, synth.TAG_B, K, N, None, "int", pins.DT)
    _, A = synth.matrix(10, synth.TAG_A, M, K, None, "int", pins.DT)
    for (ta, tb) in COMBOS:
        for (i0, k0) in [(0, 0), (5, 7), (2, 6), (4, 1)]:
            Ah = pins.zeros((M, K)); Ah[i0, k0] = 1.0
            _, As = stored(Ah, ta, pad=3)
            _, Bs = stored(B, tb, pad=1)
            C = pins.zeros((M, N))
            impl(ta, tb, -2.0, As, Bs, 0.0, C)
            want = pins.zeros((M, N)); want[i0, :] = B[k0, :]
            want = pins.DT.type(-2.0) * want     # one rounding-free product per element; zeros become -0
            assert_bitwise(C, want, "one-hot op(A) at %s trans %s" % ((i0, k0), (ta, tb)))
        for (k0, j0) in [(0, 0), (7, 10), (3, 9)]:
            Bh = pins.zeros((K, N)); Bh[k0, j0] = 1.0
            _, As = stored(A, ta, pad=2)
            _, Bs = stored(Bh, tb, pad=5)
            C = pins.ones((M, N))
            impl(ta, tb, 1.0, As, Bs, 3.0, C)
            want = pins.ones((M, N), 3.0); want[:, j0] += A[:, k0]
            assert_bitwise(C, want, "one-hot op(B) at %s trans %s" % ((k0, j0), (ta, tb)))


def pin_general_unread_operands(impl):
    """beta == 0: C may hold NaN and must not be read.  alpha == 0: A and B may hold NaN and must not be
    read; C becomes beta * C (one rounding), or +0 everywhere when beta is zero too.  K == 0 likewise."""
    M, N, K = 7, 10, 13
    A, B, C0 = _logical(800, M, N, K, kind="int")
    iA, iB = A.astype(np.int64), B.astype(np.int64)
    nan = float("nan")
    for (ta, tb) in COMBOS:
        _, As = stored(A, ta, pad=1)
        _, Bs = stored(B, tb, pad=1)
        C = pins.ones((M, N), nan)
        impl(ta, tb, 3.0, As, Bs, 0.0, C)
        assert_bitwise(C, (3 * (iA @ iB)).astype(pins.DT), "beta = 0 with NaN in C, trans %s" % ((ta, tb),))
        _, Cu = synth.matrix(801, synth.TAG_C, M, N, None, "uniform", pins.DT)
        C = Cu.copy()
        impl(ta, tb, 0.0, As * nan, Bs * nan, 0.7, C)
        assert_bitwise(C, (pins.DT.type(0.7) * Cu).astype(pins.DT), "alpha = 0 with NaN in A and B")
        C = pins.ones((M, N), nan)
        impl(ta, tb, 0.0, As * nan, Bs * nan, 0.0, C)
        assert_bitwise(C, pins.zeros((M, N)), "alpha = beta = 0")
        C = Cu.copy()
        impl(ta, tb, 5.0, pins.zeros((0, M) if ta else (M, 0)), pins.zeros((N, 0) if tb else (0, N)), -1.5, C)
        assert_bitwise(C, (pins.DT.type(-1.5) * Cu).astype(pins.DT), "K = 0 scales C by beta")


def pin_general_integer_exact(impl, shape=(96, 80, 112), seed=0):
    """Small-integer data and integer scalars: every intermediate value is an exact integer in any order."""
    M, N, K = shape
    A, B, C0 = _logical(seed, M, N, K, kind="int")
    for n, (ta, tb) in enumerate(COMBOS):
        alpha, beta = [(1.0, 1.0), (-3.0, 2.0), (2.0, 0.0), (1.0, -1.0)][n]
        Ab, As = stored(A, ta, pad=4)
        Bb, Bs = stored(B, tb, pad=6)
        Cb, C = stored(C0, 0, pad=2)
        impl(ta, tb, alpha, As, Bs, beta, C)
        want = (int(alpha) * (A.astype(np.int64) @ B.astype(np.int64)) + int(beta) * C0.astype(np.int64)).astype(pins.DT)
        assert_bitwise(C, want, "general integer exact %s trans %s" % (shape, (ta, tb)))
        assert synth.padding_intact(Ab, As.shape[1]) and synth.padding_intact(Bb, Bs.shape[1]) and synth.padding_intact(Cb, N)


def pin_general_error_bound(impl, shape=(64, 48, 256), samples=80, seed=3):
    """Against the exact value: |c_hat - c| <= gamma_{K+3} * (|alpha| S + |beta c_in|), S = sum |a b|
    (K-1 additions and K products, then two products and one addition; gamma_n = n u / (1 - n u))."""
    M, N, K = shape
    alpha, beta = -1.75, 0.6180339887498949
    A, B, C0 = _logical(seed, M, N, K)
    _, As = stored(A, 1, pad=3)
    _, Bs = stored(B, 1, pad=1)
    C = C0.copy()
    impl(1, 1, alpha, As, Bs, beta, C)
    al, be = Fraction(float(pins.DT.type(alpha))), Fraction(float(pins.DT.type(beta)))
    u = Fraction(1, 2 ** pins.mant_bits())
    gamma = (K + 3) * u / (1 - (K + 3) * u)
    rng = np.random.default_rng(seed)
    pts = {(0, 0), (M - 1, N - 1), (0, N - 1), (M - 1, 0)}
    while len(pts) < samples:
        pts.add((int(rng.integers(M)), int(rng.integers(N))))
    for (i, j) in sorted(pts):
        s = Fraction(0); S = Fraction(0)
        for k in range(K):
            t = Fraction(float(A[i, k])) * Fraction(float(B[k, j]))
            s += t; S += abs(t)
        exact = al * s + be * Fraction(float(C0[i, j]))
        scale = abs(al) * S + abs(be * Fraction(float(C0[i, j])))
        err = abs(Fraction(float(C[i, j])) - exact)
        assert err <= gamma * scale, "general error bound broken at (%d,%d)" % (i, j)


ORDER_DEPENDENT = [pin_general_rounded_sequence, pin_general_rounding_cases]

ALL_PINS = [pin_general_tiny_exact, pin_general_rounded_sequence, pin_general_rounding_cases, pin_general_all_ones,
            pin_general_one_hot, pin_general_unread_operands, pin_general_integer_exact, pin_general_error_bound]
