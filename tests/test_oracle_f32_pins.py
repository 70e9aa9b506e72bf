"""The float32 CPU oracle (the paper's Section 2.13 substitution f64 -> f32) against what the paper and the
mathematics fix, with u = 2^-24; and planted mistakes that the pins must catch (no GPU)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2003_00532_amd import synth

import pins

F32 = np.float32


def impl_oracle(A, B, C):
    oracle.gemm_f32_ref(A, B, C)


def impl_oracle_ijk(A, B, C):
    oracle.gemm_f32_ref_ijk(A, B, C)


@pytest.fixture(autouse=True)
def _single_precision():
    with pins.precision(F32):
        yield


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda p: p.__name__)
def test_pin_ikj(pin):
    pin(impl_oracle)


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda p: p.__name__)
def test_pin_paper_loop_order(pin):
    if pin is pins.pin_tiny_exact:
        pin(impl_oracle_ijk, limit=3)
    elif pin is pins.pin_integer_exact:
        pin(impl_oracle_ijk, shape=(96, 80, 112))
    elif pin is pins.pin_error_bound:
        pin(impl_oracle_ijk, shape=(64, 64, 256), samples=60)
    else:
        pin(impl_oracle_ijk)


def test_rn_helper_agrees_with_numpy_rounding():
    # the rational-to-binary32 rounding used by the emulation, against numpy's own double -> float32
    # conversion on values where no double rounding can occur (exact doubles)
    rng = np.random.default_rng(0)
    for x in rng.standard_normal(2000) * 10.0 ** rng.integers(-6, 6, 2000):
        assert pins.rn(Fraction(float(x))) == float(F32(x))
    with pins.precision(np.float64):
        assert pins.rn(Fraction(1, 3)) == 1.0 / 3.0 and pins.rn(Fraction(2 ** 53 + 1)) == float(2 ** 53)


def test_paper_driver_all_ones_full_size():
    pins.pin_paper_all_ones(impl_oracle, shapes={(2088, 2048, 2048)})


def test_interchange_and_threads_are_bitwise_neutral():
    _, A = synth.matrix(1, synth.TAG_A, 45, 131, 140, "uniform", F32)
    _, B = synth.matrix(1, synth.TAG_B, 131, 67, 70, "uniform", F32)
    _, C0 = synth.matrix(1, synth.TAG_C, 45, 67, 67, "uniform", F32)
    c1 = C0.copy(); oracle.gemm_f32_ref(A, B, c1)
    c2 = C0.copy(); oracle.gemm_f32_ref_ijk(A, B, c2)
    pins.assert_bitwise(c1, c2, "ikj vs ijk")
    n0 = oracle.ref_threads()
    try:
        oracle.set_ref_threads(1)
        c3 = C0.copy(); oracle.gemm_f32_ref(A, B, c3)
    finally:
        oracle.set_ref_threads(n0)
    pins.assert_bitwise(c1, c3, "thread count")


def test_absref_scale_is_exact_to_double_precision():
    _, A = synth.matrix(3, synth.TAG_A, 4, 9, 11, "uniform", F32)
    _, B = synth.matrix(3, synth.TAG_B, 9, 5, 6, "uniform", F32)
    S = np.zeros((4, 5)); oracle.gemm_f32_absref(A, B, S)
    for i in range(4):
        for j in range(5):
            exact = sum(abs(Fraction(float(A[i, k])) * Fraction(float(B[k, j]))) for k in range(9))
            assert abs(Fraction(float(S[i, j])) - exact) <= exact * Fraction(20, 2 ** 53)


def test_rows_helpers_dispatch_on_dtype():
    _, A = synth.matrix(5, synth.TAG_A, 40, 33, None, "uniform", F32)
    _, B = synth.matrix(5, synth.TAG_B, 33, 21, None, "uniform", F32)
    _, C0 = synth.matrix(5, synth.TAG_C, 40, 21, None, "uniform", F32)
    full = C0.copy(); oracle.gemm_f32_ref(A, B, full)
    rows = [0, 7, 8, 39]
    got = oracle.ref_rows(A, B, C0, rows)
    assert got.dtype == F32
    pins.assert_bitwise(got, full[rows])
    S = np.zeros((40, 21)); oracle.gemm_f32_absref(A, B, S)
    pins.assert_bitwise(oracle.abs_rows(A, B, rows), S[rows])


# ---- planted mistakes, in binary32 ------------------------------------------------------------

def _loops(A, B, C, body=None, korder=None, start=None, finish=None):
    M, K = A.shape
    N = B.shape[1]
    for i in range(M):
        for j in range(N):
            c0 = F32(C[i, j])
            c = c0 if start is None else start(c0)
            for k in (range(K) if korder is None else korder(K)):
                a, b = F32(A[i, k]), F32(B[k, j])
                c = F32(c + F32(a * b)) if body is None else body(c, a, b)
            C[i, j] = c if finish is None else finish(c, c0)


def good(A, B, C):
    _loops(A, B, C)


def fused(A, B, C):
    _loops(A, B, C, body=lambda c, a, b: F32(pins.rn(Fraction(float(c)) + Fraction(float(a)) * Fraction(float(b)))))


def double_accumulator(A, B, C):
    M, K = A.shape
    for i in range(M):
        for j in range(B.shape[1]):
            acc = float(C[i, j])
            for k in range(K):
                acc += float(A[i, k]) * float(B[k, j])
            C[i, j] = F32(acc)


def descending(A, B, C):
    _loops(A, B, C, korder=lambda K: range(K - 1, -1, -1))


def add_c_last(A, B, C):
    _loops(A, B, C, start=lambda c: F32(0), finish=lambda acc, c0: F32(c0 + acc))


def drop_last_term(A, B, C):
    _loops(A, B, C, korder=lambda K: range(max(K - 1, 0)))


def half_precision_product(A, B, C):
    _loops(A, B, C, body=lambda c, a, b: F32(c + F32(np.float16(a) * np.float16(b))))


FAST_PINS = [pins.pin_all_ones_small, pins.pin_identity, pins.pin_column_sums, pins.pin_rank_one,
             pins.pin_one_hot_index, pins.pin_rounded_sequence, pins.pin_rounding_cases,
             pins.pin_block_split_invariance, pins.pin_ld_independence, pins.pin_degenerate,
             lambda impl: pins.pin_tiny_exact(impl, limit=3)]


def failures(impl):
    out = []
    for pin in FAST_PINS:
        try:
            pin(impl)
        except AssertionError:
            out.append(getattr(pin, "__name__", "lambda"))
    return out


def test_binary32_rendering_of_the_definition_passes():
    assert failures(good) == []


@pytest.mark.parametrize("mutant", [fused, double_accumulator, descending, add_c_last, drop_last_term,
                                    half_precision_product], ids=lambda m: m.__name__)
def test_mutant_is_caught(mutant):
    assert failures(mutant), "no pin noticed the planted mistake %s" % mutant.__name__
