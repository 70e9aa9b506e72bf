"""Pins of `oracle.general_scale`, the scale S of the elementwise tolerance of the general, split-K and strided
parity tests: S = |alpha| * sum_k |opA(i,k) * opB(k,j)| + |beta * c_in|, with c_in ignored when beta == 0
(Section 2.15 Q4 names the operation C = alpha*A*B + beta*C; the tolerance is that of the plain operation with
each term replaced by its magnitude).  Checked against exact rational arithmetic written out here, on data for
which every intermediate value is representable, and against planted mistakes (no GPU)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

COMBOS = [(0, 0), (0, 1), (1, 0), (1, 1)]
SCALARS = [(1.0, 1.0), (1.0, 0.0), (0.0, 1.0), (0.0, 0.0), (-1.0, 0.5), (2.0, -1.5), (0.25, 3.0), (-0.75, 0.0),
           (-3.0, -0.125)]


def _dyadic(rng, shape, dtype):
    # multiples of 1/16 in [-2, 2]: products are multiples of 1/256, every sum here is exact in either precision
    return (rng.integers(-32, 33, size=shape) / 16.0).astype(dtype)


def _exact_scale(ta, tb, alpha, As, Bs, beta, C0):
    """|alpha| * sum_k |opA opB| + |beta| * |c_in| in rational arithmetic; As, Bs as stored."""
    M, N = C0.shape
    K = As.shape[0] if ta else As.shape[1]
    out = np.empty((M, N), dtype=object)
    for i in range(M):
        for j in range(N):
            s = Fraction(0)
            for k in range(K):
                a = As[k, i] if ta else As[i, k]
                b = Bs[j, k] if tb else Bs[k, j]
                s += abs(Fraction(float(a)) * Fraction(float(b)))
            s *= abs(Fraction(float(alpha)))
            if beta != 0:
                s += abs(Fraction(float(beta)) * Fraction(float(C0[i, j])))
            out[i, j] = s
    return out


def pin_scale(scale):
    rng = np.random.default_rng(11)
    n = 0
    for dtype in (np.float64, np.float32):
        for M in range(0, 4):
            for N in range(0, 4):
                for K in range(0, 5):
                    for (ta, tb) in COMBOS:
                        alpha, beta = SCALARS[n % len(SCALARS)]
                        n += 1
                        A = _dyadic(rng, (K, M) if ta else (M, K), dtype)
                        B = _dyadic(rng, (N, K) if tb else (K, N), dtype)
                        C0 = _dyadic(rng, (M, N), dtype)
                        want = _exact_scale(ta, tb, alpha, A, B, beta, C0)
                        if beta == 0:
                            C0 = np.full((M, N), np.nan, dtype=dtype)   # not read: must not poison the scale
                        S = scale(ta, tb, alpha, A, B, beta, C0)
                        assert S.dtype == np.float64 and S.shape == (M, N)
                        assert np.all(np.isfinite(S)), "an operand that must not be read reached the scale"
                        for i in range(M):
                            for j in range(N):
                                assert Fraction(float(S[i, j])) == want[i, j], (dtype.__name__, M, N, K, ta, tb, alpha, beta, i, j)


def test_general_scale_is_the_exact_magnitude_sum():
    pin_scale(oracle.general_scale)


def test_general_scale_never_negative_and_bounds_the_result():
    # |alpha op(A) op(B) + beta C0| <= S element by element, with equality when no term cancels
    rng = np.random.default_rng(5)
    A, B, C0 = _dyadic(rng, (7, 9), np.float64), _dyadic(rng, (9, 5), np.float64), _dyadic(rng, (7, 5), np.float64)
    for alpha, beta in SCALARS:
        S = oracle.general_scale(0, 0, alpha, A, B, beta, C0)
        want = C0.copy()
        oracle.gemm_general_ref(0, 0, alpha, A, B, beta, want)
        assert np.all(S >= 0) and np.all(np.abs(want) <= S)
        Spos = oracle.general_scale(0, 0, abs(alpha), np.abs(A), np.abs(B), abs(beta), np.abs(C0))
        pos = np.abs(C0)
        oracle.gemm_general_ref(0, 0, abs(alpha), np.abs(A), np.abs(B), abs(beta), pos)
        assert np.array_equal(Spos, pos)


def _mutants():
    def drop_alpha(ta, tb, alpha, A, B, beta, C0):
        return oracle.general_scale(ta, tb, 1.0, A, B, beta, C0)

    def signed_alpha(ta, tb, alpha, A, B, beta, C0):
        S = np.zeros(C0.shape) if beta == 0 else np.abs(C0.astype(np.float64))
        return oracle.gemm_general_ref(ta, tb, float(alpha), np.abs(A.astype(np.float64)), np.abs(B.astype(np.float64)),
                                       abs(float(beta)), np.ascontiguousarray(S))

    def c_read_when_beta_zero(ta, tb, alpha, A, B, beta, C0):
        S = np.abs(C0.astype(np.float64))
        return oracle.gemm_general_ref(ta, tb, abs(float(alpha)), np.abs(A.astype(np.float64)), np.abs(B.astype(np.float64)),
                                       1.0 if beta == 0 else abs(float(beta)), np.ascontiguousarray(S))

    def drop_c_term(ta, tb, alpha, A, B, beta, C0):
        return oracle.general_scale(ta, tb, alpha, A, B, 0.0, C0)

    def beta_not_applied(ta, tb, alpha, A, B, beta, C0):
        return oracle.general_scale(ta, tb, alpha, A, B, 1.0 if beta != 0 else 0.0, C0)

    def magnitudes_forgotten(ta, tb, alpha, A, B, beta, C0):
        S = np.zeros(C0.shape) if beta == 0 else C0.astype(np.float64)
        return oracle.gemm_general_ref(ta, tb, abs(float(alpha)), A.astype(np.float64), B.astype(np.float64), abs(float(beta)),
                                       np.ascontiguousarray(S))

    def transposes_swapped(ta, tb, alpha, A, B, beta, C0):
        if ta == tb:
            return oracle.general_scale(ta, tb, alpha, A, B, beta, C0)
        K = A.shape[0] if ta else A.shape[1]
        if A.shape != ((K, C0.shape[0]) if tb else (C0.shape[0], K)) or B.shape != ((C0.shape[1], K) if ta else (K, C0.shape[1])):
            raise AssertionError("shapes do not fit the swapped flags")
        return oracle.general_scale(tb, ta, alpha, A, B, beta, C0)

    return [drop_alpha, signed_alpha, c_read_when_beta_zero, drop_c_term, beta_not_applied, magnitudes_forgotten,
            transposes_swapped]


@pytest.mark.parametrize("mutant", _mutants(), ids=lambda m: m.__name__)
def test_planted_mistakes_in_the_scale_are_caught(mutant):
    with pytest.raises(AssertionError):
        pin_scale(mutant)
