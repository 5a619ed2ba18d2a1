"""Property tests of the CPU oracle on inputs drawn by hypothesis (CPU only): arbitrary finite binary64
values including subnormals, extreme exponents and ties.  Expected values come from exact rational
arithmetic (tests/exactref.py), never from the oracle or the HIP path."""
from fractions import Fraction

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import oracle
from tests import exactref as ex

finite = st.floats(allow_nan=False, allow_infinity=False, width=64)
# few significant bits at arbitrary positions: rounding ties and long carries
sparse = st.builds(lambda m, e, sgn: sgn * float(m) * 2.0 ** e, st.integers(0, 255), st.integers(-1060, 960),
                   st.sampled_from([-1.0, 1.0]))
entry = st.one_of(finite, sparse, st.just(0.0))
rows = st.lists(entry, min_size=1, max_size=6)


@settings(max_examples=150, deadline=None)
@given(rows, st.integers(1, 12), st.sampled_from([7, 5, 3]))
def test_truncated_slices_of_any_row(row, s, t):
    X = np.array([row])
    planes, e = oracle.split("A", X, s, t)
    ee = int(e[0])
    assert ee == ex.scale_exponent(max(abs(Fraction(v)) for v in row))
    for j, v in enumerate(row):
        x = Fraction(v)
        assert planes[:, 0, j].tolist() == ex.slices_by_recursion(x, ee, s, t)
        rec = sum(Fraction(int(planes[l, 0, j])) * Fraction(2) ** (ee - (l + 1) * t) for l in range(s))
        assert abs(x - rec) < Fraction(2) ** (ee - s * t) or x == rec


@settings(max_examples=150, deadline=None)
@given(rows, st.integers(1, 12), st.sampled_from([7, 5, 3]))
def test_nearest_slices_of_any_row(row, s, t):
    X = np.array([row])
    planes, e = oracle.split_nearest("A", X, s, t)
    ee = int(e[0])
    for j, v in enumerate(row):
        x = Fraction(v)
        assert planes[:, 0, j].tolist() == ex.slices_nearest(x, ee, s, t)
        assert max(abs(int(p)) for p in planes[:, 0, j]) <= 2 ** (t - 1)
        rec = sum(Fraction(int(planes[l, 0, j])) * Fraction(2) ** (ee + 1 - (l + 1) * t) for l in range(s))
        assert 2 * abs(x - rec) <= Fraction(2) ** (ee + 1 - s * t)


small = st.floats(min_value=-1e6, max_value=1e6, allow_nan=False, width=64)


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 4), st.integers(1, 4), st.integers(1, 5), st.integers(1, 9), st.integers(1, 9), st.booleans(),
       st.booleans(), st.integers(1, 3), st.data())
def test_product_against_exact_diagonals(m, n, k, sA, sB, full, nearest, Q, data):
    # every diagonal exact in rationals, one binary64 rounding per level of Q diagonals
    A = np.array(data.draw(st.lists(st.lists(small, min_size=k, max_size=k), min_size=m, max_size=m)))
    B = np.array(data.draw(st.lists(st.lists(small, min_size=n, max_size=n), min_size=k, max_size=k)))
    terms, eA, eB = ex.diagonal_terms(ex.frac_matrix(A), ex.frac_matrix(B), sA, 7, full=full, sB=sB, rounding=nearest)
    C = oracle.dgemm3(A, B, sA, sB, 7, full=full, nearest=nearest, Q=Q)
    for i in range(m):
        for j in range(n):
            assert C[i, j] == ex.accumulate_levels(terms, eA, eB, Q, i, j)
    # transposed problem: transposed result, bit for bit
    Ct = oracle.dgemm3(B.T.copy(), A.T.copy(), sB, sA, 7, full=full, nearest=nearest, Q=Q)
    assert np.array_equal(C, Ct.T)
