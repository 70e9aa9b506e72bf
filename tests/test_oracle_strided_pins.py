"""The CPU oracle of the strided operation against its pins, in both precisions, and planted mistakes
that the pins must catch (no GPU)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import ref as oref

import pins
import pins_general as pg
import pins_strided as ps


def impl_oracle(alpha, A, B, beta, C):
    oracle.gemm_strided_ref(alpha, A, B, beta, C)


@pytest.mark.parametrize("pin", ps.ALL_PINS, ids=lambda p: p.__name__)
def test_strided_pin_f64(pin):
    pin(impl_oracle)


@pytest.mark.parametrize("pin", ps.ALL_PINS, ids=lambda p: p.__name__)
def test_strided_pin_f32(pin):
    with pins.precision(np.float32):
        pin(impl_oracle)


@pytest.mark.parametrize("c_layout", ["row", "col", "col_step3"])
@pytest.mark.parametrize("pin", pg.ALL_PINS, ids=lambda p: p.__name__)
def test_pins_of_the_transposed_signature_through_strides(pin, c_layout):
    pin(ps.as_general_impl(impl_oracle, c_layout))


def test_pins_of_the_transposed_signature_through_strides_f32():
    with pins.precision(np.float32):
        for pin in pg.ALL_PINS:
            pin(ps.as_general_impl(impl_oracle, "col"))


def test_strided_agrees_bitwise_with_the_transposed_oracle_where_both_apply():
    # secondary: two separately written loops, the same definition
    M, N, K = 23, 31, 40
    A, B, C0 = pg._logical(5, M, N, K)
    for (ta, tb) in pg.COMBOS:
        _, As = pg.stored(A, ta, pad=2)
        _, Bs = pg.stored(B, tb, pad=1)
        c1 = C0.copy(); oracle.gemm_general_ref(ta, tb, 1.25, As, Bs, -0.5, c1)
        c2 = C0.copy(); impl_oracle(1.25, As.T if ta else As, Bs.T if tb else Bs, -0.5, c2)
        pins.assert_bitwise(c1, c2, "trans %s" % ((ta, tb),))
        # column-major C is the transposed problem C^T = B^T A^T: the same sums term by term
        _, c3 = ps.place(C0, "col")
        impl_oracle(1.25, As.T if ta else As, Bs.T if tb else Bs, -0.5, c3)
        pins.assert_bitwise(np.ascontiguousarray(c3), c1, "column-major C, trans %s" % ((ta, tb),))


def test_strided_thread_count_is_bitwise_neutral():
    M, N, K = 45, 37, 90
    A, B, C0 = pg._logical(8, M, N, K)
    n0 = oracle.ref_threads()
    outs = []
    try:
        for n in (1, 3, n0):
            oracle.set_ref_threads(n)
            _, Cv = ps.place(C0, "col_step3")
            impl_oracle(1.5, ps.place(A, "col")[1], ps.place(B, "row_step2")[1], -0.5, Cv)
            outs.append(np.ascontiguousarray(Cv))
    finally:
        oracle.set_ref_threads(n0)
    pins.assert_bitwise(outs[0], outs[1]); pins.assert_bitwise(outs[0], outs[2])


def test_strided_argument_validation():
    f = oref.raw("gemm_f64_strided_ref")
    buf = np.zeros(256)
    p = buf.ctypes.data

    def call(M, N, K, sa=(4, 1), sb=(3, 1), sc=(3, 1), a=p, b=p, c=p, alpha=1.0):
        return f(M, N, K, alpha, a, sa[0], sa[1], b, sb[0], sb[1], 1.0, c, sc[0], sc[1])

    assert call(2, 3, 4) == 0
    assert call(-1, 3, 4) == -1 and call(2, -3, 4) == -1 and call(2, 3, -4) == -1
    assert call(2, 3, 4, sa=(0, 1)) == -2 and call(2, 3, 4, sa=(4, 0)) == -2 and call(2, 3, 4, sa=(-4, 1)) == -2
    assert call(2, 3, 4, sb=(0, 1)) == -3 and call(2, 3, 4, sb=(3, -1)) == -3
    assert call(2, 3, 4, sc=(0, 1)) == -4
    assert call(2, 3, 4, sa=(1, 1)) == 0                       # overlapping reads of A are allowed
    assert call(2, 3, 4, sc=(2, 1)) == -4                      # rows of C overlap: 2 < 1 * (3 - 1) + 1
    assert call(2, 3, 4, sc=(3, 1)) == 0
    assert call(2, 3, 4, sc=(1, 1)) == -4 and call(2, 3, 4, sc=(1, 2)) == 0    # column-major needs csc >= M
    assert call(2, 3, 4, sc=(4, 2)) == -4 and call(2, 3, 4, sc=(5, 2)) == 0    # sampled rows: 5 >= 2 * 2 + 1
    assert call(1, 3, 4, sc=(1, 1)) == 0 and call(2, 1, 4, sc=(1, 1)) == 0     # a single row or column
    assert call(2, 3, 4, a=None) == -5 and call(2, 3, 4, c=None) == -5
    assert call(2, 3, 4, a=None, b=None, alpha=0.0) == 0
    assert call(0, 3, 4, c=None) == 0


# ---- planted mistakes -------------------------------------------------------------------------

def _definition(alpha, A, B, beta, C, *, swap_a=False, swap_b=False, swap_c=False, unit_cs_a=False, unit_cs_c=False,
                c_rs_for_both=False, beta_on_sum=False, read_c_always=False, start_from_c=False):
    """The definition on raw buffers and element strides, with optional planted mistakes in the addressing or the tail."""
    dt = C.dtype.type
    sz = C.dtype.itemsize
    M, N = C.shape
    K = A.shape[1]

    def flat(X):
        # the whole underlying allocation as a 1-D array, the view's first element's index in it, its strides
        base = X.base if X.base is not None else X
        while base.base is not None:
            base = base.base
        base = base.reshape(-1)
        off = (X.__array_interface__["data"][0] - base.__array_interface__["data"][0]) // sz
        return base, off, oracle.element_strides(X)

    a, a0, (rsa, csa) = flat(A)
    b, b0, (rsb, csb) = flat(B)
    c, c0, (rsc, csc) = flat(C)
    if swap_a: rsa, csa = csa, rsa
    if swap_b: rsb, csb = csb, rsb
    if swap_c: rsc, csc = csc, rsc
    if unit_cs_a: csa = 1
    if unit_cs_c: csc = 1
    if c_rs_for_both: csc = rsc
    alpha, beta = dt(alpha), dt(beta)

    def at(buf, idx):
        return buf[idx] if 0 <= idx < buf.size else dt(777.0)   # a wild address: model it as garbage

    for i in range(M):
        for j in range(N):
            ci = c0 + i * rsc + j * csc
            if not (0 <= ci < c.size):
                continue
            cin = c[ci]
            if alpha == 0 or K == 0:
                c[ci] = beta * cin if (beta != 0 or read_c_always) else dt(0)
                continue
            s = cin if start_from_c else dt(0)
            for k in range(K):
                s = dt(s + dt(at(a, a0 + i * rsa + k * csa) * at(b, b0 + k * rsb + j * csb)))
            t = dt(alpha * s)
            if start_from_c:
                c[ci] = t
            elif beta == 0 and not read_c_always:
                c[ci] = t
            elif beta_on_sum:
                c[ci] = dt(beta * dt(t + cin))
            else:
                c[ci] = dt(t + dt(beta * cin))


def _mutant(**kw):
    def impl(alpha, A, B, beta, C):
        with np.errstate(all="ignore"):
            _definition(alpha, A, B, beta, C, **kw)
    impl.__name__ = "+".join(kw) or "good"
    return impl


FAST = [lambda impl: ps.pin_strided_tiny_exact(impl, limit=2), ps.pin_strided_rounded_sequence, ps.pin_strided_unread_operands,
        lambda impl: ps.pin_strided_integer_exact(impl, shape=(7, 6, 9)), ps.pin_strided_overlapping_reads]


def _failures(impl):
    out = []
    for pin in FAST:
        try:
            pin(impl)
        except AssertionError:
            out.append(getattr(pin, "__name__", "lambda"))
    return out


def test_python_rendering_of_the_strided_definition_passes():
    assert _failures(_mutant()) == []


@pytest.mark.parametrize("kw", [dict(swap_a=True), dict(swap_b=True), dict(swap_c=True), dict(unit_cs_a=True),
                                dict(unit_cs_c=True), dict(c_rs_for_both=True), dict(beta_on_sum=True),
                                dict(read_c_always=True), dict(start_from_c=True)],
                         ids=lambda kw: "+".join(kw))
def test_strided_mutant_is_caught(kw):
    assert _failures(_mutant(**kw)), "no pin noticed the planted mistake %s" % kw
