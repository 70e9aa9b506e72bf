"""The CPU oracle against what the paper and the mathematics fix (no GPU)."""
import ctypes

import numpy as np
import pytest

import oracle
from oracle import ref as oref
from paper_2003_00532_amd import synth

import pins


def impl_oracle(A, B, C):
    oracle.gemm_f64_ref(A, B, C)


def impl_oracle_ijk(A, B, C):
    oracle.gemm_f64_ref_ijk(A, B, C)


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


def test_paper_driver_all_ones_full_size():
    # the paper's own workload, 2088 x 2048 x 2048 filled with 1.0 (Sections 1.3, 2.1)
    pins.pin_paper_all_ones(impl_oracle, shapes={(2088, 2048, 2048)})


def test_integer_exact_edge_shape_rows():
    # the ragged benchmark shape with its padded leading dimensions, against int64 arithmetic on a band of rows
    M, N, K = 64, 2049, 2047
    pins.pin_integer_exact(impl_oracle, shape=(M, N, K), lds=(2056, 2064, 2064), seed=3)


def test_interchange_is_bitwise_neutral():
    # i-k-j (threaded) and the literal i-j-k nest see the same ascending k sequence per element
    _, A = synth.matrix(1, synth.TAG_A, 45, 131, 140, "uniform")
    _, B = synth.matrix(1, synth.TAG_B, 131, 67, 70, "uniform")
    _, C0 = synth.matrix(1, synth.TAG_C, 45, 67, 67, "uniform")
    c1 = C0.copy(); oracle.gemm_f64_ref(A, B, c1)
    c2 = C0.copy(); oracle.gemm_f64_ref_ijk(A, B, c2)
    pins.assert_bitwise(c1, c2, "ikj vs ijk")


def test_thread_count_is_bitwise_neutral():
    _, A = synth.matrix(2, synth.TAG_A, 97, 64, None, "uniform")
    _, B = synth.matrix(2, synth.TAG_B, 64, 55, None, "uniform")
    _, C0 = synth.matrix(2, synth.TAG_C, 97, 55, None, "uniform")
    n0 = oracle.ref_threads()
    outs = []
    try:
        for n in (1, 3, max(2, n0)):
            oracle.set_ref_threads(n)
            c = C0.copy(); oracle.gemm_f64_ref(A, B, c); outs.append(c)
    finally:
        oracle.set_ref_threads(n0)
    pins.assert_bitwise(outs[0], outs[1]); pins.assert_bitwise(outs[0], outs[2])


def test_absref_is_the_tolerance_scale():
    from fractions import Fraction
    _, A = synth.matrix(3, synth.TAG_A, 4, 9, 11, "uniform")
    _, B = synth.matrix(3, synth.TAG_B, 9, 5, 6, "uniform")
    S = np.zeros((4, 5)); oracle.gemm_f64_absref(A, B, S)
    for i in range(4):
        for j in range(5):
            exact = sum(abs(Fraction(float(A[i, k])) * Fraction(float(B[k, j]))) for k in range(9))
            assert abs(Fraction(float(S[i, j])) - exact) <= exact * Fraction(10, 2 ** 53) * 2
    # dominance: |A B| <= |A| |B| elementwise, exactly, on integers
    _, Ai = synth.matrix(4, synth.TAG_A, 30, 40, None, "int")
    _, Bi = synth.matrix(4, synth.TAG_B, 40, 20, None, "int")
    S = np.zeros((30, 20)); oracle.gemm_f64_absref(Ai, Bi, S)
    pins.assert_bitwise(S, (np.abs(Ai).astype(np.int64) @ np.abs(Bi).astype(np.int64)).astype(np.float64))


def test_rows_helpers_match_full_result():
    _, A = synth.matrix(5, synth.TAG_A, 40, 33, None, "uniform")
    _, B = synth.matrix(5, synth.TAG_B, 33, 21, None, "uniform")
    _, C0 = synth.matrix(5, synth.TAG_C, 40, 21, None, "uniform")
    full = C0.copy(); oracle.gemm_f64_ref(A, B, full)
    rows = [0, 7, 8, 39]
    pins.assert_bitwise(oracle.ref_rows(A, B, C0, rows), full[rows])
    S = np.zeros((40, 21)); oracle.gemm_f64_absref(A, B, S)
    pins.assert_bitwise(oracle.abs_rows(A, B, rows), S[rows])


def test_argument_validation():
    fn = oref.raw("gemm_f64_ref")
    a = np.zeros((4, 4)); p = a.ctypes.data
    assert fn(-1, 1, 1, p, 1, p, 1, p, 1) == -1
    assert fn(2, 2, 3, p, 2, p, 2, p, 2) == -2
    assert fn(2, 3, 2, p, 2, p, 2, p, 3) == -3
    assert fn(2, 3, 2, p, 2, p, 3, p, 2) == -4
    assert fn(2, 2, 2, None, 2, p, 2, p, 2) == -5
    assert fn(2, 2, 2, p, 2, p, 2, None, 2) == -5
    assert fn(0, 2, 2, None, 2, None, 2, None, 2) == 0
    assert fn(2, 2, 0, None, 1, None, 2, p, 2) == 0
