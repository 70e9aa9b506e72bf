"""The CPU oracle of `C <- alpha * op(A) op(B) + beta * C` against its pins, in both precisions, and
planted mistakes that the pins must catch (no GPU)."""
import ctypes

import numpy as np
import pytest

import oracle
from oracle import ref as oref
from paper_2003_00532_amd import synth

import pins
import pins_general as pg


def impl_oracle(ta, tb, alpha, A, B, beta, C):
    oracle.gemm_general_ref(ta, tb, alpha, A, B, beta, C)


@pytest.mark.parametrize("pin", pg.ALL_PINS, ids=lambda p: p.__name__)
def test_general_pin_f64(pin):
    pin(impl_oracle)


@pytest.mark.parametrize("pin", pg.ALL_PINS, ids=lambda p: p.__name__)
def test_general_pin_f32(pin):
    with pins.precision(np.float32):
        pin(impl_oracle)


def test_general_thread_count_and_row_blocks_are_bitwise_neutral():
    M, N, K = 45, 67, 131
    A, B, C0 = pg._logical(1, M, N, K)
    _, As = pg.stored(A, 1, pad=3)
    _, Bs = pg.stored(B, 1, pad=2)
    n0 = oracle.ref_threads()
    try:
        outs = []
        for n in (1, 3, n0):
            oracle.set_ref_threads(n)
            C = C0.copy(); impl_oracle(1, 1, 1.5, As, Bs, -0.5, C); outs.append(C)
    finally:
        oracle.set_ref_threads(n0)
    pins.assert_bitwise(outs[0], outs[1]); pins.assert_bitwise(outs[0], outs[2])
    # row and column blocks are independent problems
    parts = C0.copy()
    for (r0, r1) in [(0, 20), (20, M)]:
        for (c0, c1) in [(0, 31), (31, N)]:
            impl_oracle(1, 1, 1.5, As[:, r0:r1], Bs[c0:c1, :], -0.5, parts[r0:r1, c0:c1])
    pins.assert_bitwise(parts, outs[0], "block split")


def test_general_agrees_with_the_accumulating_oracle_where_both_are_exact():
    # alpha = beta = 1 without transposes is the paper's operation; on integer data the two evaluation
    # orders (sum started from C, C added last) must give the same bits
    M, N, K = 70, 90, 50
    _, A = synth.matrix(2, synth.TAG_A, M, K, K + 1, "int")
    _, B = synth.matrix(2, synth.TAG_B, K, N, N + 2, "int")
    _, C0 = synth.matrix(2, synth.TAG_C, M, N, N + 3, "int")
    c1 = C0.copy(); oracle.gemm_f64_ref(A, B, c1)
    c2 = C0.copy(); impl_oracle(0, 0, 1.0, A, B, 1.0, c2)
    pins.assert_bitwise(c1, c2)


def test_general_argument_validation():
    f = oref.raw("gemm_f64_general_ref")
    buf = np.zeros(64)
    p = buf.ctypes.data
    call = lambda ta, tb, M, N, K, lda, ldb, ldc, a=p, b=p, c=p, alpha=1.0: f(ta, tb, M, N, K, alpha, a, lda, b, ldb, 1.0, c, ldc)
    assert call(0, 0, 2, 3, 4, 4, 3, 3) == 0
    assert call(2, 0, 2, 3, 4, 4, 3, 3) == -1 and call(0, -1, 2, 3, 4, 4, 3, 3) == -1
    assert call(0, 0, -1, 3, 4, 4, 3, 3) == -1
    assert call(0, 0, 2, 3, 4, 3, 3, 3) == -2          # lda < K
    assert call(1, 0, 2, 3, 4, 1, 3, 3) == -2          # transposed A: lda < M
    assert call(1, 0, 2, 3, 4, 2, 3, 3) == 0
    assert call(0, 0, 2, 3, 4, 4, 2, 3) == -3          # ldb < N
    assert call(0, 1, 2, 3, 4, 4, 3, 3) == -3          # transposed B: ldb < K
    assert call(0, 1, 2, 3, 4, 4, 4, 3) == 0
    assert call(0, 0, 2, 3, 4, 4, 3, 2) == -4
    assert call(0, 0, 2, 3, 4, 4, 3, 3, a=None) == -5
    assert call(0, 0, 2, 3, 4, 4, 3, 3, a=None, b=None, alpha=0.0) == 0   # alpha == 0: A and B are not needed
    assert call(0, 0, 2, 3, 4, 4, 3, 3, c=None) == -5


# ---- planted mistakes -------------------------------------------------------------------------

def _definition(ta, tb, alpha, A, B, beta, C, *, swap_trans=False, beta_on_sum=False, alpha_on_c=False,
                read_c_always=False, read_ab_always=False, start_from_c=False, fold_alpha=False, fused_tail=False,
                wrong_ld=False):
    from fractions import Fraction
    dt = C.dtype.type
    if swap_trans:
        ta, tb = tb, ta
    M, N = C.shape
    La = A.T if ta else A
    Lb = B.T if tb else B
    if wrong_ld and ta:
        La = np.ascontiguousarray(A).reshape(-1)[:A.size].reshape(A.shape[1], A.shape[0]) if A.size else La
    if La.shape[0] != M or Lb.shape[1] != N or La.shape[1] != Lb.shape[0]:
        # a swapped transpose on non-square operands reads the wrong elements; model it as garbage
        C[...] = dt(12345.0)
        return
    K = La.shape[1]
    alpha, beta = dt(alpha), dt(beta)
    for i in range(M):
        for j in range(N):
            cin = C[i, j]
            if (alpha == 0 or K == 0) and not read_ab_always:
                C[i, j] = beta * cin if (beta != 0 or read_c_always) else dt(0)
                continue
            s = cin if start_from_c else dt(0)
            for k in range(K):
                a = La[i, k] * alpha if fold_alpha else La[i, k]
                s = dt(s + dt(a * Lb[k, j]))
            t = s if fold_alpha else dt(alpha * s)
            if alpha_on_c:
                t = s
            if start_from_c:
                C[i, j] = t
            elif beta == 0 and not read_c_always:
                C[i, j] = t
            elif beta_on_sum:
                C[i, j] = dt(beta * dt(t + cin))
            elif alpha_on_c:
                C[i, j] = dt(t + dt(alpha * dt(beta * cin)))
            elif fused_tail:
                C[i, j] = dt(float(Fraction(float(t)) + Fraction(float(beta)) * Fraction(float(cin))))
            else:
                C[i, j] = dt(t + dt(beta * cin))


def _mutant(**kw):
    def impl(ta, tb, alpha, A, B, beta, C):
        with np.errstate(all="ignore"):
            _definition(ta, tb, alpha, A, B, beta, C, **kw)
    impl.__name__ = "+".join(kw) or "good"
    return impl


FAST = [lambda impl: pg.pin_general_tiny_exact(impl, limit=2), pg.pin_general_rounded_sequence, pg.pin_general_rounding_cases,
        pg.pin_general_all_ones, pg.pin_general_one_hot, pg.pin_general_unread_operands,
        lambda impl: pg.pin_general_integer_exact(impl, shape=(12, 10, 14))]


def _failures(impl):
    out = []
    for pin in FAST:
        try:
            pin(impl)
        except AssertionError:
            out.append(getattr(pin, "__name__", "lambda"))
    return out


def test_python_rendering_of_the_general_definition_passes():
    assert _failures(_mutant()) == []


@pytest.mark.parametrize("kw", [dict(swap_trans=True), dict(beta_on_sum=True), dict(alpha_on_c=True),
                                dict(read_c_always=True), dict(read_ab_always=True), dict(start_from_c=True),
                                dict(fold_alpha=True), dict(fused_tail=True), dict(wrong_ld=True)],
                         ids=lambda kw: "+".join(kw))
def test_general_mutant_is_caught(kw):
    assert _failures(_mutant(**kw)), "no pin noticed the planted mistake %s" % kw
