"""Plausible mistakes, planted in CPU re-implementations, must each fail a pin.

This shows the pin suite has teeth: a dropped term, a wrong sign or index, a
transposed operand, a fused product, a different summation order or a C that
is ignored or added last would not go unnoticed in the oracle.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import pins


def _loops(A, B, C, body=None, korder=None, start=None, finish=None):
    M, K = A.shape
    N = B.shape[1]
    for i in range(M):
        for j in range(N):
            c = float(C[i, j]) if start is None else start(float(C[i, j]))
            ks = range(K) if korder is None else korder(K)
            for k in ks:
                a, b = float(A[i, k]), float(B[k, j])
                c = (c + a * b) if body is None else body(c, a, b)
            C[i, j] = c if finish is None else finish(c, float(C[i, j]))


def good(A, B, C):
    _loops(A, B, C)


def fused(A, B, C):
    _loops(A, B, C, body=lambda c, a, b: float(Fraction(c) + Fraction(a) * Fraction(b)))


def descending(A, B, C):
    _loops(A, B, C, korder=lambda K: range(K - 1, -1, -1))


def add_c_last(A, B, C):
    _loops(A, B, C, start=lambda c: 0.0, finish=lambda acc, c0: c0 + acc)


def ignore_c(A, B, C):
    _loops(A, B, C, start=lambda c: 0.0)


def drop_last_term(A, B, C):
    _loops(A, B, C, korder=lambda K: range(max(K - 1, 0)))


def minus(A, B, C):
    _loops(A, B, C, body=lambda c, a, b: c - a * b)


def transposed_a(A, B, C):
    M, K = A.shape
    At = np.zeros((M, K))
    m = min(M, K)
    At[:m, :m] = A[:m, :m].T
    _loops(At, B, C)


def transposed_b(A, B, C):
    K, N = B.shape
    Bt = np.zeros((K, N))
    m = min(K, N)
    Bt[:m, :m] = B[:m, :m].T
    _loops(Bt if False else A, Bt, C)


def float32_product(A, B, C):
    _loops(A, B, C, body=lambda c, a, b: c + float(np.float32(a) * np.float32(b)))


def off_by_one_row(A, B, C):
    tmp = C.copy()
    _loops(A, B, tmp)
    C[...] = np.roll(tmp, 1, axis=0) if C.shape[0] > 1 else tmp


def writes_padding(A, B, C):
    _loops(A, B, C)
    base = C.base if C.base is not None else None
    if base is not None and base.ndim == 2 and base.shape[1] > C.shape[1]:
        base[:, C.shape[1]] = 0.0


FAST_PINS = [pins.pin_all_ones_small, pins.pin_identity, pins.pin_column_sums, pins.pin_rank_one,
             pins.pin_one_hot_index, pins.pin_rounded_sequence, pins.pin_rounding_cases,
             pins.pin_block_split_invariance, pins.pin_ld_independence, pins.pin_degenerate,
             lambda impl: pins.pin_tiny_exact(impl, limit=3),
             lambda impl: pins.pin_integer_exact(impl, shape=(12, 10, 14), lds=(15, 11, 13))]


def failures(impl):
    out = []
    for pin in FAST_PINS:
        try:
            pin(impl)
        except AssertionError:
            out.append(getattr(pin, "__name__", "lambda"))
    return out


def test_python_rendering_of_the_definition_passes():
    assert failures(good) == []


@pytest.mark.parametrize("mutant", [fused, descending, add_c_last, ignore_c, drop_last_term, minus,
                                    transposed_a, transposed_b, float32_product, off_by_one_row,
                                    writes_padding], ids=lambda m: m.__name__)
def test_mutant_is_caught(mutant):
    assert failures(mutant), "no pin noticed the planted mistake %s" % mutant.__name__
