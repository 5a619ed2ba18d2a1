"""Pins for the CPU oracle: values the paper prints, exact rational arithmetic, closed forms,
invariants.  None of these tests uses a GPU, and none takes an expected value from the oracle
itself or from the HIP path."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle
from tests import exactref as ex
from paper_2506_11277_amd import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
U = 2.0 ** -53


def bits_to_int(sbits):
    neg = sbits.startswith("-")
    v = int(sbits.lstrip("-"), 2)
    return -v if neg else v


def small_cases():
    """A zoo of small inputs: well scaled, wide dynamic range, powers of two, zeros, subnormals."""
    rng = np.random.default_rng(7)
    cases = []
    cases.append(("uniform", rng.random((5, 6)) * 2 - 1, rng.random((6, 4)) * 2 - 1))
    cases.append(("lognormal2", (rng.random((4, 7)) - .5) * np.exp(2 * rng.standard_normal((4, 7))),
                  (rng.random((7, 5)) - .5) * np.exp(2 * rng.standard_normal((7, 5)))))
    cases.append(("lognormal8", (rng.random((3, 5)) - .5) * np.exp(8 * rng.standard_normal((3, 5))),
                  (rng.random((5, 3)) - .5) * np.exp(8 * rng.standard_normal((5, 3)))))
    A = np.array([[1.0, 0.5, -0.25, 0.0], [4.0, -4.0, 3.999999999999999, 2.0 ** -30], [0.0, 0.0, 0.0, 0.0]])
    B = np.array([[2.0 ** 10, 0.0, -1.0], [-(2.0 ** 10), 0.0, 1.0 - 2.0 ** -53], [3.0, 0.0, 2.0 ** -40],
                  [1e-3, 0.0, -0.0]])
    cases.append(("pow2_zero", A, B))
    tiny = 5e-324
    A = np.array([[tiny, 3 * tiny, -1000 * tiny], [2.0 ** -1022, 2.0 ** -1030, -tiny]])
    B = np.array([[1.0, 2.0 ** -1060], [-3.0, 7 * tiny], [0.125, 2.0 ** -1040]])
    cases.append(("subnormal", A, B))
    cases.append(("huge", np.array([[1.7e308, -3e307, 1.0]]), np.array([[2.0 ** -1000], [2.0 ** -990], [2.0 ** -980]])))
    return cases


# --------------------------------------------------------------------------- worked example

def test_worked_example_of_section_3():
    g = json.load(open(os.path.join(HERE, "golden", "worked_example.json")))
    t, s = g["t"], g["s"]
    A = np.array([g["A"]])                 # 1 x 3
    B = np.array(g["B"]).reshape(3, 1)     # 3 x 1
    eA = oracle.exponents("A", A)
    eB = oracle.exponents("B", B)
    assert eA.tolist() == [g["alpha_log2"]] and eB.tolist() == [g["beta_log2"]]
    pa, _ = oracle.split("A", A, s, t)
    pb, _ = oracle.split("B", B, s, t)
    for l in range(s):
        assert pa[l, 0, :].tolist() == [bits_to_int(b) for b in g["A_slices_bits"][l]]
        assert pb[l, :, 0].tolist() == [bits_to_int(b) for b in g["B_slices_bits"][l]]
    total = Fraction(0)
    for key, sbits in g["products_bits"].items():
        l, h = (int(v) for v in key.split(","))
        P = oracle.slice_product(pa[l - 1], pb[h - 1])
        assert P.shape == (1, 1) and int(P[0, 0]) == bits_to_int(sbits), key
        total += Fraction(bits_to_int(sbits)) * Fraction(2) ** g["diagonal_scale_log2"][str(l + h)]
    printed = Fraction(bits_to_int(g["result_bits"])) * Fraction(2) ** g["result_scale_log2"]
    exact = sum(Fraction(a) * Fraction(b) for a, b in zip(g["A"], g["B"]))
    assert total == printed == exact
    for order in (0, 1):
        C = oracle.dgemm(A, B, s, t, order=order, full=True)
        assert Fraction(float(C[0, 0])) == printed
    # with the reduced product set (l + h <= s + 1) the products (2,4) and (3,4) are dropped
    C = oracle.dgemm(A, B, s, t, order=0, full=False)
    dropped = Fraction(24) * Fraction(2) ** -11 + Fraction(8) * Fraction(2) ** -14
    assert Fraction(float(C[0, 0])) == printed - dropped


# --------------------------------------------------------------------------- scales

@pytest.mark.parametrize("name,A,B", small_cases())
def test_exponents_are_smallest_power_of_two_above_max(name, A, B):
    for side, X in (("A", A), ("B", B)):
        e = oracle.exponents(side, X)
        want = ex.block_exponents(side, ex.frac_matrix(X))
        assert e.tolist() == want
    # direct statement of eq. (alpha-def): 2^(e-1) <= M < 2^e
    e = oracle.exponents("A", A)
    for i in range(A.shape[0]):
        M = max(abs(Fraction(float(v))) for v in A[i])
        if M:
            assert Fraction(2) ** (int(e[i]) - 1) <= M < Fraction(2) ** int(e[i])


def test_exponent_of_exact_power_of_two_is_bumped():
    # M a power of two: alpha = 2 M (strictly larger)
    for p in (-1074, -1022, -3, 0, 1, 52, 1023):
        X = np.array([[math.ldexp(1.0, p), 0.0]])
        assert oracle.exponents("A", X).tolist() == [p + 1]
        Y = np.array([[math.ldexp(1.0, p)], [-math.ldexp(1.0, p)]])
        assert oracle.exponents("B", Y).tolist() == [p + 1]


def test_nonfinite_inputs_are_rejected():
    for bad in (np.nan, np.inf, -np.inf):
        A = np.ones((2, 2))
        A[1, 0] = bad
        with pytest.raises(oracle.OracleError) as ei:
            oracle.dgemm(A, np.ones((2, 2)), 3)
        assert ei.value.code == oracle.NONFINITE
        with pytest.raises(oracle.OracleError):
            oracle.dgemm(np.ones((2, 2)), A, 3)


# --------------------------------------------------------------------------- slices

@pytest.mark.parametrize("name,A,B", small_cases())
@pytest.mark.parametrize("t,s", [(7, 1), (7, 4), (7, 9), (7, 12), (3, 5), (5, 20), (1, 9)])
def test_slices_match_recursive_definition(name, A, B, t, s):
    for side, X in (("A", A), ("B", B)):
        planes, e = oracle.split(side, X, s, t)
        Xf = ex.frac_matrix(X)
        for i in range(X.shape[0]):
            for j in range(X.shape[1]):
                want = ex.slices_by_recursion(Xf[i][j], int(e[i] if side == "A" else e[j]), s, t)
                assert planes[:, i, j].tolist() == want, (side, i, j)


@pytest.mark.parametrize("name,A,B", small_cases())
def test_slice_range_and_sign(name, A, B):
    for side, X in (("A", A), ("B", B)):
        planes, e = oracle.split(side, X, 10, 7)
        assert planes.min() >= -127 and planes.max() <= 127
        sgn = np.sign(X)
        assert np.all((planes == 0) | (np.sign(planes) == sgn[None]))
        first = np.abs(planes[0])
        blockmax = first.max(axis=1 if side == "A" else 0)
        nonzero = (np.abs(X).max(axis=1 if side == "A" else 0) > 0)
        assert np.all(blockmax[nonzero] >= 64)      # 0.5 <= M / alpha < 1


@pytest.mark.parametrize("name,A,B", small_cases())
@pytest.mark.parametrize("t", [7, 4])
def test_reconstruction_and_truncation_bound(name, A, B, t):
    for side, X in (("A", A), ("B", B)):
        s_star = ex.min_exact_slices(side, X.tolist(), t)
        assert s_star <= max(1, ex.bit_spread_slices(side, X.tolist(), t))
        for s in sorted({1, 2, max(1, s_star - 1), s_star, min(s_star + 1, oracle.MAX_SLICES)}):
            if s > oracle.MAX_SLICES:
                continue
            planes, e = oracle.split(side, X, s, t)
            exact_everywhere = True
            for i in range(X.shape[0]):
                for j in range(X.shape[1]):
                    ee = int(e[i] if side == "A" else e[j])
                    x = Fraction(float(X[i, j]))
                    rec = sum(Fraction(int(planes[l, i, j])) * Fraction(2) ** (ee - (l + 1) * t) for l in range(s))
                    delta = x - rec
                    # eq. (a-split): |delta| < alpha 2^{-st}; truncation => delta has the sign of x
                    assert abs(delta) < Fraction(2) ** (ee - s * t)
                    assert delta == 0 or (delta > 0) == (x > 0)
                    exact_everywhere &= delta == 0
            assert exact_everywhere == (s >= s_star), (side, s, s_star)


def test_bit_spread_recipe_is_tight_when_smallest_entry_is_widest():
    t = 7
    row = [1.0, (1.0 + 2.0 ** -52) * 2.0 ** -20]         # spread 53 on the smallest entry
    assert ex.bit_spread_slices("A", [row], t) == -(-(20 + 53) // t)
    assert ex.min_exact_slices("A", [row], t) == -(-(1 + 20 + 52) // t)


# --------------------------------------------------------------------------- integer products

def test_slice_product_equals_library_integer_matmul():
    rng = np.random.default_rng(3)
    for (m, n, k) in [(1, 1, 1), (3, 5, 7), (17, 9, 300), (2, 2, 5000)]:
        Al = rng.integers(-127, 128, size=(m, k)).astype(np.int8)
        Bh = rng.integers(-127, 128, size=(k, n)).astype(np.int8)
        assert np.array_equal(oracle.slice_product(Al, Bh), Al.astype(np.int64) @ Bh.astype(np.int64))
    # extreme values: k * 127^2 exceeds 2^31, int64 must hold it
    k = 140000
    Al = np.full((1, k), 127, dtype=np.int8)
    Bh = np.full((k, 1), -127, dtype=np.int8)
    assert int(oracle.slice_product(Al, Bh)[0, 0]) == -127 * 127 * k


def test_single_slice_on_small_integers_is_the_integer_product():
    # entries that are integers of magnitude <= 127 (times a power of two per row of A /
    # column of B) live entirely in the first slice, so s = 1 must return A B exactly
    rng = np.random.default_rng(11)
    Ai = rng.integers(-127, 128, size=(9, 40))
    Bi = rng.integers(-127, 128, size=(40, 6))
    ra = rng.integers(-40, 40, size=9)
    cb = rng.integers(-40, 40, size=6)
    A = Ai * np.ldexp(1.0, ra)[:, None]
    B = Bi * np.ldexp(1.0, cb)[None, :]
    want = (Ai @ Bi).astype(np.float64) * np.ldexp(1.0, ra)[:, None] * np.ldexp(1.0, cb)[None, :]
    for order in (0, 1):
        assert np.array_equal(oracle.dgemm(A, B, 1, order=order), want)
        assert np.array_equal(oracle.dgemm(A, B, 3, order=order), want)


# --------------------------------------------------------------------------- whole path, exact

def to_float_matrix(F):
    out = np.empty((len(F), len(F[0])))
    for i, row in enumerate(F):
        for j, v in enumerate(row):
            f = float(v)
            assert Fraction(f) == v, "value is not a binary64 number"
            out[i, j] = f
    return out


@pytest.mark.parametrize("name,A,B", small_cases()[:4])
@pytest.mark.parametrize("t,s", [(7, 1), (7, 2), (7, 3), (7, 5), (3, 6), (4, 8)])
def test_reduced_product_set_in_the_exact_regime(name, A, B, t, s):
    # with ceil(log2 k) + (s+1) t + 1 <= 53 no addition of the accumulation can round, so C must be
    # C' of eq. (c-prime) exactly, whatever the order
    k = A.shape[1]
    assert math.ceil(math.log2(k)) + (s + 1) * t + 1 <= 53
    want = ex.reduced_product_exact(ex.frac_matrix(A), ex.frac_matrix(B), s, t)
    for order in (0, 1):
        C = oracle.dgemm(A, B, s, t, order=order)
        assert np.array_equal(C, to_float_matrix(want)), order
    want_full = ex.reduced_product_exact(ex.frac_matrix(A), ex.frac_matrix(B), s, t, full=True)
    if math.ceil(math.log2(k)) + 2 * s * t + 1 <= 53:
        assert np.array_equal(oracle.dgemm(A, B, s, t, full=True), to_float_matrix(want_full))


@pytest.mark.parametrize("name,A,B", small_cases()[:4])
@pytest.mark.parametrize("s", [7, 8, 10, 13])
def test_diagonal_order_rounds_once_per_diagonal_ascending(name, A, B, s):
    # outside the exact regime: exact diagonal values (rational), then one correctly rounded
    # binary64 addition per diagonal, d = 2, 3, ...  (Python float addition is IEEE binary64)
    t = 7
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    terms, eA, eB = ex.diagonal_terms(Af, Bf, s, t)
    C = oracle.dgemm(A, B, s, t, order=0)
    for i in range(A.shape[0]):
        for j in range(B.shape[1]):
            S = 0.0
            for d in sorted(terms):
                # the unscaled diagonal term is an integer times 2^{-dt}: exactly representable
                term = terms[d][i][j] / Fraction(2) ** (eA[i] + eB[j])
                f = float(term)
                assert Fraction(f) == term
                S = S + f
            assert C[i, j] == math.ldexp(S, eA[i] + eB[j]), (i, j)


@pytest.mark.parametrize("name,A,B", small_cases()[:4])
@pytest.mark.parametrize("s", [7, 8, 9, 10])
def test_algorithm_1_order_rounds_once_per_product_l_outer_h_inner(name, A, B, s):
    # the literal loop nest of Algorithm 1 outside the exact regime: exact value of every single product
    # (rational), one correctly rounded binary64 addition per product, l = 1, 2, ... outside, h = 1, 2, ... inside.
    # The other nesting (h outside) and the diagonal order are different sequences of roundings: the test also
    # checks that at least one of its cases tells them apart.
    t = 7
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    terms, eA, eB = ex.pair_terms(Af, Bf, s, t)
    C = oracle.dgemm(A, B, s, t, order=1)
    swapped_differs = False
    for i in range(A.shape[0]):
        for j in range(B.shape[1]):
            scale = Fraction(2) ** (eA[i] + eB[j])
            S = 0.0
            for l in range(1, s + 1):
                for h in range(1, s + 2 - l):
                    term = terms[(l, h)][i][j] / scale
                    f = float(term)
                    assert Fraction(f) == term          # an integer times 2^{-(l+h)t}: a binary64 number
                    S = S + f
            assert C[i, j] == math.ldexp(S, eA[i] + eB[j]), (i, j)
            S2 = 0.0
            for h in range(1, s + 1):
                for l in range(1, s + 2 - h):
                    S2 = S2 + float(terms[(l, h)][i][j] / scale)
            swapped_differs = swapped_differs or S2 != S
    _ORDER1_DISCRIMINATES[(name, s)] = swapped_differs


_ORDER1_DISCRIMINATES = {}


def test_algorithm_1_order_pin_tells_the_two_loop_nests_apart():
    # runs after the parametrised cases above (same module, definition order)
    assert _ORDER1_DISCRIMINATES and any(_ORDER1_DISCRIMINATES.values())


@pytest.mark.parametrize("phi,s", [(0.5, 3), (0.5, 6), (0.5, 8), (2.0, 4), (2.0, 9), (4.0, 7), (4.0, 12)])
def test_error_bound_of_reduced_product_variant(phi, s):
    # |C - C_hat'| <= (zeta + 2^{-st} s kA kB + gamma_psi (1 + zeta + 2^{-st} s kA kB)) |A||B|,
    # the bound at the end of the subsection "Reduction in number of products"
    t = 7
    A, B = workloads.lognormal(6, 5, 24, phi, seed=100 + s)
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    exact = ex.matmul(Af, Bf)
    absprod = ex.matmul(ex.absmat(Af), ex.absmat(Bf))
    kA, kB = ex.kappa("A", Af), ex.kappa("B", Bf)
    w = Fraction(2) ** (-s * t)
    zeta = w * kA + w * kB + w * w * kA * kB
    extra = w * s * kA * kB
    for order, psi in ((0, s), (1, s * (s + 1) // 2)):
        gamma = Fraction(psi) * Fraction(U) / (1 - Fraction(psi) * Fraction(U))
        bound = zeta + extra + gamma * (1 + zeta + extra)
        C = oracle.dgemm(A, B, s, t, order=order)
        for i in range(6):
            for j in range(5):
                assert abs(Fraction(float(C[i, j])) - exact[i][j]) <= bound * absprod[i][j]


def test_orders_agree_bitwise_in_exact_regime_at_config_size():
    A, B = workloads.uniform(128, 128, 128, 1000)
    assert np.array_equal(oracle.dgemm(A, B, 3, order=0), oracle.dgemm(A, B, 3, order=1))
    assert np.array_equal(oracle.dgemm(A, B, 5, order=0), oracle.dgemm(A, B, 5, order=1))


# --------------------------------------------------------------------------- symmetries

def test_power_of_two_scaling_invariance():
    A0, B0 = workloads.uniform(12, 9, 33, 5)
    rng = np.random.default_rng(5)
    a = rng.integers(-30, 31, size=12)
    b = rng.integers(-30, 31, size=9)
    A = A0 * np.ldexp(1.0, a)[:, None]
    B = B0 * np.ldexp(1.0, b)[None, :]
    s = 8
    p0, e0 = oracle.split("A", A0, s)
    p1, e1 = oracle.split("A", A, s)
    assert np.array_equal(p0, p1) and np.array_equal(e1, e0 + a)
    q0, f0 = oracle.split("B", B0, s)
    q1, f1 = oracle.split("B", B, s)
    assert np.array_equal(q0, q1) and np.array_equal(f1, f0 + b)
    C0 = oracle.dgemm(A0, B0, s)
    C = oracle.dgemm(A, B, s)
    assert np.array_equal(C, C0 * np.ldexp(1.0, a)[:, None] * np.ldexp(1.0, b)[None, :])


def test_negation_and_permutations():
    A, B = workloads.lognormal(10, 11, 50, 1.0, 9)
    s = 8
    C = oracle.dgemm(A, B, s)
    assert np.array_equal(oracle.dgemm(-A, B, s), -C)
    assert np.array_equal(oracle.dgemm(A, -B, s), -C)
    rng = np.random.default_rng(1)
    pk = rng.permutation(50)
    assert np.array_equal(oracle.dgemm(A[:, pk], B[pk, :], s), C)
    pm = rng.permutation(10)
    pn = rng.permutation(11)
    assert np.array_equal(oracle.dgemm(A[pm, :], B[:, pn], s), C[np.ix_(pm, pn)])
    # transposition duality: (A B)^T = B^T A^T with the roles of rows and columns swapped
    assert np.array_equal(oracle.dgemm(B.T.copy(), A.T.copy(), s), C.T)


def test_product_count():
    # number of computed products is s (s + 1) / 2.  Construction where every slice of the (0,0)
    # entries equals 1 (k = 2, second entry only pins the scale at 2^0): each computed pair (l,h)
    # contributes exactly 2^{-(l+h)t}, so the value of C identifies the set of pairs.
    for t, s in ((3, 1), (3, 2), (3, 5), (3, 9), (7, 3), (5, 5)):
        x = float(sum(Fraction(2) ** (-l * t) for l in range(1, s + 1)))
        assert Fraction(x) == sum(Fraction(2) ** (-l * t) for l in range(1, s + 1))
        A = np.array([[x, 0.75]])
        B = np.array([[x, 0.75], [0.0, 0.0]])
        C = oracle.dgemm(A, B, s, t)
        pairs = [(l, h) for l in range(1, s + 1) for h in range(1, s + 2 - l)]
        assert len(pairs) == s * (s + 1) // 2
        assert Fraction(float(C[0, 0])) == sum(Fraction(2) ** (-(l + h) * t) for l, h in pairs)
        Cfull = oracle.dgemm(A, B, s, t, full=True)
        assert Fraction(float(Cfull[0, 0])) == Fraction(x) ** 2


# --------------------------------------------------------------------------- estimator

def test_kappa_matches_definition():
    for name, A, B in small_cases():
        kA = ex.kappa("A", ex.frac_matrix(A))
        kB = ex.kappa("B", ex.frac_matrix(B))
        for got, want in ((oracle.kappa("A", A), kA), (oracle.kappa("B", B), kB)):
            if want > Fraction(1.7e308):
                assert got == math.inf
            else:
                # one division and one doubling: correctly rounded quotient
                assert got == float(want), name


def test_estimator_closed_form_on_two_vector_example():
    # a = [2^-phi x, 1], b = [2^phi y, 1]^T with x, y powers of two: kappa_A = 2^{phi+1} / |x|,
    # kappa_B = 2^{phi+1} |y| when 2^phi |y| >= 1 (max / min of the two entries)
    t = 7
    for phi in (0, 3, 20, 100):
        for xp, yp in ((0, 0), (-2, 1), (-1, 3)):
            x, y = 2.0 ** xp, 2.0 ** yp
            a = np.array([[2.0 ** -phi * x, 1.0]])
            b = np.array([[2.0 ** phi * y], [1.0]])
            kA = 2.0 ** (phi + 1 - xp)
            kB = 2.0 ** (phi + 1 + yp)
            for tol in (1e-3, 2.0 ** -30, 2.0 ** -53):
                s, rc, gA, gB = oracle.estimate_slices(a, b, tol, t, s_max=64)
                assert (gA, gB) == (kA, kB)
                want = next(ss for ss in range(1, 200) if Fraction(kA + kB) * Fraction(2) ** (-ss * t) <= Fraction(tol))
                assert rc == oracle.OK and s == want


def test_estimator_properties():
    A, B = workloads.lognormal(40, 30, 64, 0.5, 77)
    prev = None
    for tol in (1e-2, 1e-4, 1e-8, 1e-12, 1e-15):
        s, rc, kA, kB = oracle.estimate_slices(A, B, tol)
        assert rc == oracle.OK
        # definition, evaluated exactly
        lhs = lambda ss: (Fraction(kA) + Fraction(kB)) * Fraction(2) ** (-7 * ss)
        assert lhs(s) <= Fraction(tol) * (1 + Fraction(2) ** -50)
        assert s == 1 or lhs(s - 1) > Fraction(tol) * (1 - Fraction(2) ** -50)
        assert prev is None or s >= prev
        prev = s
    # one more slice per factor 2^7 in the tolerance
    s1 = oracle.estimate_slices(A, B, 1e-6)[0]
    s2 = oracle.estimate_slices(A, B, 1e-6 / 128)[0]
    assert s2 == s1 + 1
    # invariant under power-of-two row / column scaling
    rng = np.random.default_rng(0)
    A2 = A * np.ldexp(1.0, rng.integers(-30, 31, size=40))[:, None]
    B2 = B * np.ldexp(1.0, rng.integers(-30, 31, size=30))[None, :]
    assert oracle.estimate_slices(A2, B2, 1e-9) == oracle.estimate_slices(A, B, 1e-9)
    # zero entries and zero rows do not enter kappa
    A3 = A.copy()
    A3[3, :] = 0.0
    A3[5, 7] = 0.0
    assert oracle.kappa("A", A3) == float(ex.kappa("A", ex.frac_matrix(A3)))
    # unreachable tolerance
    s, rc, _, _ = oracle.estimate_slices(A, B, 1e-300, s_max=32)
    assert rc == oracle.UNREACHABLE and s == 32


def test_estimated_slices_deliver_the_tolerance_up_to_the_second_order_term():
    # with the estimator's s the first-order truncation terms are below tol; the measured error
    # relative to |A||B| must then be below tol + s kA kB 2^{-st} + rounding (full bound)
    t = 7
    A, B = workloads.lognormal(8, 8, 32, 0.5, 3)
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    exact = ex.matmul(Af, Bf)
    absprod = ex.matmul(ex.absmat(Af), ex.absmat(Bf))
    for tol in (1e-4, 1e-9, 1e-14):
        s, rc, kA, kB = oracle.estimate_slices(A, B, tol)
        C = oracle.dgemm(A, B, s)
        w = Fraction(2) ** (-s * t)
        full = Fraction(tol) + w * w * Fraction(kA) * Fraction(kB) + w * s * Fraction(kA) * Fraction(kB) + Fraction(2 * s) * Fraction(U)
        worst = max(abs(Fraction(float(C[i, j])) - exact[i][j]) / absprod[i][j] for i in range(8) for j in range(8))
        assert worst <= full


# --------------------------------------------------------------------------- qualitative outcomes

def test_two_vector_example_needs_more_slices_when_badly_scaled():
    # phi = 0: about 7 slices give binary64 accuracy; phi = 100: over 20 slices are needed
    rng = np.random.default_rng(2024)
    for _ in range(5):
        x, y = rng.standard_normal(2)
        if abs(x * y + 1) < 0.1:
            continue

        def err(phi, s):
            a = np.array([[math.ldexp(x, -phi), 1.0]])
            b = np.array([[math.ldexp(y, phi)], [1.0]])
            c = Fraction(math.ldexp(x, -phi)) * Fraction(math.ldexp(y, phi)) + 1
            got = Fraction(float(oracle.dgemm(a, b, s)[0, 0]))
            return float(abs(got - c) / abs(c))

        assert err(0, 3) > 1e-9
        assert err(0, 8) < 8 * U
        assert err(100, 8) > 1e-3
        assert err(100, 20) > 1e-14
        assert err(100, 24) < 8 * U


# --------------------------------------------------------------------------- different slice counts

def test_equal_slice_counts_reduce_to_algorithm_1():
    A, B = workloads.lognormal(9, 8, 40, 2.0, 12)
    for s in (1, 3, 8, 11):
        for order in (0, 1):
            for full in (False, True):
                assert np.array_equal(oracle.dgemm2(A, B, s, s, order=order, full=full),
                                      oracle.dgemm(A, B, s, order=order, full=full))


@pytest.mark.parametrize("name,A,B", small_cases()[:4])
@pytest.mark.parametrize("t,sA,sB", [(7, 1, 4), (7, 4, 1), (7, 2, 5), (7, 5, 3), (3, 2, 9), (4, 7, 3), (3, 6, 6)])
def test_different_slice_counts_in_the_exact_regime(name, A, B, t, sA, sB):
    # product set l <= sA, h <= sB, l + h <= max(sA, sB) + 1, written with truncation operators
    k = A.shape[1]
    assert math.ceil(math.log2(k)) + (max(sA, sB) + 1) * t + 1 <= 53
    want = ex.reduced_product_exact(ex.frac_matrix(A), ex.frac_matrix(B), sA, t, sB=sB)
    for order in (0, 1):
        assert np.array_equal(oracle.dgemm2(A, B, sA, sB, t, order=order), to_float_matrix(want)), order
    if math.ceil(math.log2(k)) + (sA + sB) * t + 1 <= 53:
        want_full = ex.reduced_product_exact(ex.frac_matrix(A), ex.frac_matrix(B), sA, t, full=True, sB=sB)
        assert np.array_equal(oracle.dgemm2(A, B, sA, sB, t, full=True), to_float_matrix(want_full))


@pytest.mark.parametrize("sA,sB", [(3, 9), (9, 3), (8, 12), (13, 7), (1, 10)])
def test_different_slice_counts_round_once_per_diagonal(sA, sB):
    t = 7
    A, B = workloads.lognormal(4, 5, 12, 2.0, 40 + sA)
    terms, eA, eB = ex.diagonal_terms(ex.frac_matrix(A), ex.frac_matrix(B), sA, t, sB=sB)
    assert sorted(terms) == list(range(2, max(sA, sB) + 2))
    C = oracle.dgemm2(A, B, sA, sB, t)
    for i in range(4):
        for j in range(5):
            S = 0.0
            for d in sorted(terms):
                term = terms[d][i][j] / Fraction(2) ** (eA[i] + eB[j])
                f = float(term)
                assert Fraction(f) == term
                S = S + f
            assert C[i, j] == math.ldexp(S, eA[i] + eB[j])


@pytest.mark.parametrize("phi,sA,sB", [(0.5, 3, 6), (0.5, 6, 3), (2.0, 5, 9), (2.0, 9, 4), (4.0, 8, 12), (1.0, 1, 8)])
def test_error_bounds_for_different_slice_counts(phi, sA, sB):
    # sA <= sB: extra term 2^{-sB t} sA kA kB;  sA > sB: 2^{-sA t} sB kA kB
    # (the two bounds at the end of the subsection "Reduction in number of products")
    t = 7
    A, B = workloads.lognormal(5, 6, 20, phi, seed=300 + sA * 17 + sB)
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    exact = ex.matmul(Af, Bf)
    absprod = ex.matmul(ex.absmat(Af), ex.absmat(Bf))
    kA, kB = ex.kappa("A", Af), ex.kappa("B", Bf)
    wA, wB = Fraction(2) ** (-sA * t), Fraction(2) ** (-sB * t)
    zeta = wA * kA + wB * kB + wA * wB * kA * kB
    extra = (wB * sA if sA <= sB else wA * sB) * kA * kB
    psi = max(sA, sB)
    gamma = Fraction(psi) * Fraction(U) / (1 - Fraction(psi) * Fraction(U))
    bound = zeta + extra + gamma * (1 + zeta + extra)
    C = oracle.dgemm2(A, B, sA, sB, t)
    for i in range(5):
        for j in range(6):
            assert abs(Fraction(float(C[i, j])) - exact[i][j]) <= bound * absprod[i][j]


def test_well_scaled_operand_needs_a_single_slice():
    # rows of A hold integers of magnitude <= 127 (times a power of two): A lives in its first slice,
    # so one slice of A gives bit for bit what s slices give -- the flexibility the analysis points out
    rng = np.random.default_rng(8)
    A = rng.integers(-127, 128, size=(7, 30)) * np.ldexp(1.0, rng.integers(-20, 20, size=7))[:, None]
    _, B = workloads.lognormal(7, 6, 30, 2.0, 9)
    for s in (3, 8, 12):
        ref = oracle.dgemm(A, B, s)
        assert np.array_equal(oracle.dgemm2(A, B, 1, s), ref)
        assert np.array_equal(oracle.dgemm2(A, B, 2, s), ref)
        # and symmetrically for B
        assert np.array_equal(oracle.dgemm2(B.T.copy(), A.T.copy(), s, 1), ref.T)


def test_chi_counts_the_computed_products():
    for sA in range(1, 10):
        for sB in range(1, 10):
            pairs = [(l, h) for l in range(1, sA + 1) for h in range(1, sB + 1) if l + h <= max(sA, sB) + 1]
            assert oracle.chi(sA, sB) == len(pairs)
    # the value of C identifies the set of products (every slice of the (0,0) entries equals 1)
    t = 3
    for sA, sB in ((2, 5), (5, 2), (4, 4), (1, 6)):
        xa = float(sum(Fraction(2) ** (-l * t) for l in range(1, sA + 1)))
        xb = float(sum(Fraction(2) ** (-l * t) for l in range(1, sB + 1)))
        A = np.array([[xa, 0.75]])
        B = np.array([[xb, 0.75], [0.0, 0.0]])
        C = oracle.dgemm2(A, B, sA, sB, t)
        want = sum(Fraction(2) ** (-(l + h) * t) for l in range(1, sA + 1) for h in range(1, sB + 1)
                   if l + h <= max(sA, sB) + 1)
        assert Fraction(float(C[0, 0])) == want


def test_two_dimensional_estimator_against_brute_force():
    t = 7
    rng = np.random.default_rng(5)
    for case in range(6):
        A, B = workloads.lognormal(12, 10, 16, [0.2, 1.0, 3.0][case % 3], 60 + case)
        if case >= 3:       # A well scaled (kappa_A = 2: equal magnitudes per row), B badly scaled
            A = np.sign(A) * np.ldexp(1.0, rng.integers(-5, 6, size=A.shape[0]))[:, None]
            _, B = workloads.lognormal(12, 10, 16, 3.0, 90 + case)
        kA = Fraction(oracle.kappa("A", A))
        kB = Fraction(oracle.kappa("B", B))
        for tol in (1e-3, 1e-9, 1e-15):
            sA, sB, rc, gA, gB = oracle.estimate_slices2(A, B, tol, t, s_max=32)
            feas = [(a, b) for a in range(1, 33) for b in range(1, 33)
                    if kA * Fraction(2) ** (-a * t) + kB * Fraction(2) ** (-b * t) <= Fraction(tol) * (1 - Fraction(2) ** -40)]
            chi = lambda a, b: min(a, b) * (2 * max(a, b) - min(a, b) + 1) // 2
            assert rc == oracle.OK and feas
            best = min(chi(a, b) for a, b in feas)
            assert chi(sA, sB) <= best                       # optimal cost (boundary cases aside)
            assert kA * Fraction(2) ** (-sA * t) + kB * Fraction(2) ** (-sB * t) <= Fraction(tol) * (1 + Fraction(2) ** -40)
            s1 = oracle.estimate_slices(A, B, tol, t)[0]
            assert chi(sA, sB) <= chi(s1, s1)                # never more products than equal counts
            if case >= 3 and tol < 1e-8:
                assert sA < sB                               # the well scaled operand gets fewer slices
    # swapping the roles of A and B swaps the answer
    A, B = workloads.lognormal(6, 6, 10, 2.0, 5)
    A = np.abs(A) + 1.0
    r = oracle.estimate_slices2(A, B, 1e-12)
    rT = oracle.estimate_slices2(B.T.copy(), A.T.copy(), 1e-12)
    assert oracle.chi(r[0], r[1]) == oracle.chi(rT[0], rT[1])
    assert oracle.estimate_slices2(A, B, 1e-300)[:3] == (32, 32, oracle.UNREACHABLE)


def test_badly_scaled_product_outcomes_of_the_gpu_benchmark_section():
    # A = Abar D, B = D^-1 Bbar, Abar, Bbar ~ U(1,2), geometric D with condition kappa_D, rows of A and
    # columns of B rotated.  Stated outcomes: 8 slices are not enough already at kappa_D = 1e10; more
    # slices recover binary64 accuracy for the lower kappa_D; 18 slices fail at 1e30 and 1e40.
    # (Reference in 80-bit arithmetic: all terms are positive, so it is accurate to ~1e-19.)
    n = 64

    def err(kd, s):
        A, B = workloads.diag_scaled(n, kd, 7)
        ref = A.astype(np.longdouble) @ B.astype(np.longdouble)
        C = oracle.dgemm(A, B, s).astype(np.longdouble)
        return float(np.max(np.abs((C - ref) / ref)))

    assert err(1e10, 8) > 1e-9
    assert err(1e10, 16) < 4 * U * 8
    assert err(1e20, 12) > 1e-9 and err(1e20, 18) < 4 * U * 8
    assert err(1e30, 18) > 1e-10
    assert err(1e40, 18) > 1e-3
    # the slice estimate asks for enough slices in every case
    for kd in (1e10, 1e20, 1e30):
        A, B = workloads.diag_scaled(n, kd, 7)
        s = oracle.estimate_slices(A, B, 2.0 ** -53)[0]
        assert err(kd, s) < 4 * U * 8


# --------------------------------------------------------------------------- round-to-nearest slices

@pytest.mark.parametrize("name,A,B", small_cases())
@pytest.mark.parametrize("t,s", [(7, 1), (7, 4), (7, 9), (7, 12), (3, 5), (5, 20), (2, 9)])
def test_nearest_slices_are_differences_of_nearest_integers(name, A, B, t, s):
    # the first l slices together are the integer nearest to 2^{lt} x / 2^{e+1} (ties to even), for every l
    for side, X in (("A", A), ("B", B)):
        planes, e = oracle.split_nearest(side, X, s, t)
        assert np.array_equal(e, oracle.exponents(side, X))
        Xf = ex.frac_matrix(X)
        for i in range(X.shape[0]):
            for j in range(X.shape[1]):
                want = ex.slices_nearest(Xf[i][j], int(e[i] if side == "A" else e[j]), s, t)
                assert planes[:, i, j].tolist() == want, (side, i, j)


def test_nearest_slices_on_ties_and_carries():
    # scale exponent e = 1 (max = 1.0), so x' = x / 4 and slice values are round(x' 2^{7l}) - 128 round(x' 2^{7(l-1)})
    t = 7
    X = np.array([[1.0, 4 * 0.5 / 128, 4 * 1.5 / 128, 4 * 2.5 / 128, 4 * (63.5 / 128), 4 * (1 / 128 + 64 / 128 ** 2),
                   4 * (1 / 128 + 64.5 / 128 ** 2), -4 * (2 / 128 + 127.75 / 128 ** 2), 1.0 - 2.0 ** -53]])
    planes, e = oracle.split_nearest("A", X, 3, t)
    assert e.tolist() == [1]
    got = planes[:, 0, :].T.tolist()
    assert got[0] == [32, 0, 0]                 # 1/4 = 32/128
    assert got[1] == [0, 64, 0]                 # 0.5 -> tie to the even integer 0, remainder +64
    assert got[2] == [2, -64, 0]                # 1.5 -> 2, remainder -64
    assert got[3] == [2, 64, 0]                 # 2.5 -> 2
    assert got[4] == [64, -64, 0]               # 63.5 -> 64: the first slice reaches 2^{t-1}
    assert got[5] == [2, -64, 0]                # 1.5 again, reached as 1 + 64/128: up to the even integer 2
    assert got[6] == [2, -64, 64]               # 1 + 64.5/128 -> 2; second: 192.5 -> 192 (even) - 256; third +64
    assert got[7] == [-3, 0, 32]                # -(2 + 127.75/128) -> -3; -(383.75) -> -384 - (-384) = 0; +0.25*128
    assert got[8] == [32, 0, 0]                 # 1 - 2^-53 rounds up to 1 at every cut


@pytest.mark.parametrize("name,A,B", small_cases())
@pytest.mark.parametrize("t", [7, 4])
def test_nearest_reconstruction_error_is_half_a_unit(name, A, B, t):
    for side, X in (("A", A), ("B", B)):
        for s in (1, 2, 5, 9):
            planes, e = oracle.split_nearest(side, X, s, t)
            assert planes.min() >= -(2 ** (t - 1)) and planes.max() <= 2 ** (t - 1)
            for i in range(X.shape[0]):
                for j in range(X.shape[1]):
                    ee = int(e[i] if side == "A" else e[j]) + 1
                    x = Fraction(float(X[i, j]))
                    rec = sum(Fraction(int(planes[l, i, j])) * Fraction(2) ** (ee - (l + 1) * t) for l in range(s))
                    # nearest multiple of 2^{e+1-st}: at most half of it away, i.e. alpha 2^{-st}, the
                    # truncation bound of eq. (a-split) with <= in place of <
                    assert abs(x - rec) * 2 <= Fraction(2) ** (ee - s * t)
        planes, _ = oracle.split_nearest(side, -X, 6, t)
        planes2, _ = oracle.split_nearest(side, X, 6, t)
        assert np.array_equal(planes, -planes2)


def test_nearest_slices_are_exact_with_enough_slices_and_beat_truncation_on_average():
    rng = np.random.default_rng(31)
    X = rng.standard_normal((6, 40)) * np.exp(rng.standard_normal((6, 40)))
    s_star = ex.min_exact_slices("A", X.tolist(), 7)
    planes, e = oracle.split_nearest("A", X, s_star + 1, 7)
    rec = sum(planes[l].astype(np.float64) * np.ldexp(1.0, (e[:, None] + 1) - 7 * (l + 1)) for l in range(s_star + 1))
    # (each partial sum of this float reconstruction is exact: all terms are multiples of the last unit below 2^53 units)
    assert np.array_equal(rec, X)
    for s in (2, 4):
        pt, e = oracle.split("A", X, s, 7)
        pn, _ = oracle.split_nearest("A", X, s, 7)
        rt = sum(pt[l].astype(np.float64) * np.ldexp(1.0, e[:, None] - 7 * (l + 1)) for l in range(s))
        rn = sum(pn[l].astype(np.float64) * np.ldexp(1.0, (e[:, None] + 1) - 7 * (l + 1)) for l in range(s))
        # same worst case and same mean magnitude (the unit is twice as large, the error at most half of it),
        # but truncation always errs towards zero while the rounding error has no preferred sign
        bias_t = (np.sign(X) * (X - rt) / np.ldexp(1.0, e[:, None] - 7 * s)).mean()
        bias_n = (np.sign(X) * (X - rn) / np.ldexp(1.0, e[:, None] - 7 * s)).mean()
        assert 0.4 < bias_t < 0.6 and abs(bias_n) < 0.15


@pytest.mark.parametrize("name,A,B", small_cases()[:4])
@pytest.mark.parametrize("t,sA,sB", [(7, 1, 1), (7, 3, 3), (7, 2, 5), (3, 6, 6), (4, 7, 3)])
def test_nearest_variant_in_the_exact_regime(name, A, B, t, sA, sB):
    k = A.shape[1]
    assert math.ceil(math.log2(k)) + (max(sA, sB) + 1) * t + 1 <= 53
    want = ex.reduced_product_exact(ex.frac_matrix(A), ex.frac_matrix(B), sA, t, sB=sB, rounding=True)
    for order in (0, 1):
        C, eA, eB = oracle.dgemm3(A, B, sA, sB, t, order=order, nearest=True, return_exponents=True)
        assert np.array_equal(C, to_float_matrix(want)), order
        assert np.array_equal(eA, oracle.exponents("A", A) + 1) and np.array_equal(eB, oracle.exponents("B", B) + 1)


@pytest.mark.parametrize("name,A,B", small_cases()[:4])
@pytest.mark.parametrize("s", [7, 9, 13])
def test_nearest_variant_rounds_once_per_diagonal(name, A, B, s):
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    terms, eA, eB = ex.diagonal_terms(Af, Bf, s, 7, rounding=True)
    C = oracle.dgemm3(A, B, s, s, 7, nearest=True)
    for i in range(A.shape[0]):
        for j in range(B.shape[1]):
            assert C[i, j] == ex.accumulate_levels(terms, eA, eB, 1, i, j), (i, j)


def test_nearest_variant_error_bound_and_average_gain():
    # |C - AB| <= (zeta + s kA kB 2^{-st} + gamma (1 + ...)) |A||B| holds with the truncation constants,
    # since |delta a| <= alpha 2^{-st} still.  On positive matrices (the U(0, 1) inputs of the GPU
    # benchmark section) truncation errors all have one sign and add up along k; rounding errors cancel
    rng = np.random.default_rng(77)
    A, B = rng.random((12, 48)), rng.random((48, 10))
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    exact = ex.matmul(Af, Bf)
    bound_base = ex.matmul(ex.absmat(Af), ex.absmat(Bf))
    kA, kB = ex.kappa("A", Af), ex.kappa("B", Bf)
    for s in (3, 5):
        Cn = oracle.dgemm3(A, B, s, s, 7, nearest=True)
        Ct = oracle.dgemm3(A, B, s, s, 7, nearest=False)
        u_s = Fraction(2) ** (-7 * s)
        zeta = kA * u_s + kB * u_s + kA * kB * u_s * u_s
        coeff = zeta + u_s * s * kA * kB
        gamma = Fraction(s + 1) * Fraction(U) / (1 - Fraction(s + 1) * Fraction(U))
        errn = errt = Fraction(0)
        for i in range(12):
            for j in range(10):
                en = abs(Fraction(float(Cn[i, j])) - exact[i][j])
                assert en <= (coeff + gamma * (1 + coeff)) * bound_base[i][j]
                errn += en
                errt += abs(Fraction(float(Ct[i, j])) - exact[i][j])
        assert errn < errt


# --------------------------------------------------------------------------- levels of diagonals

@pytest.mark.parametrize("name,A,B", small_cases()[:4])
@pytest.mark.parametrize("sA,sB,full,nearest", [(8, 8, False, False), (13, 13, False, False), (5, 11, False, False),
                                                 (6, 4, True, False), (9, 9, False, True)])
def test_levels_of_diagonals_round_once_per_level(name, A, B, sA, sB, full, nearest):
    # k <= 7: a level of up to 4 diagonals is an integer below 2^53 units (3 + 14 + 21 bits and carries)
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    terms, eA, eB = ex.diagonal_terms(Af, Bf, sA, 7, full=full, sB=sB, rounding=nearest)
    for Q in (1, 2, 3, 4):
        C = oracle.dgemm3(A, B, sA, sB, 7, full=full, nearest=nearest, Q=Q)
        for i in range(A.shape[0]):
            for j in range(B.shape[1]):
                assert C[i, j] == ex.accumulate_levels(terms, eA, eB, Q, i, j), (Q, i, j)
    assert np.array_equal(oracle.dgemm3(A, B, sA, sB, 7, full=full, Q=1), oracle.dgemm2(A, B, sA, sB, 7, full=full))


def test_a_single_level_holds_the_exact_sum_of_the_products():
    # t = 3: all diagonals of s = 9 and 12 fit one level, so nothing is rounded and C is the exact value of
    # eq. (c-prime) (a level that is exact in binary64 has exact partial sums too, so Q = 1 agrees)
    A, B = workloads.lognormal(6, 5, 9, 1.0, seed=5)
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    for s in (9, 12):
        want = to_float_matrix(ex.reduced_product_exact(Af, Bf, s, 3))
        assert np.array_equal(oracle.dgemm3(A, B, s, s, 3, Q=s), want)
        assert np.array_equal(oracle.dgemm3(A, B, s, s, 3, Q=1), want)


def test_a_level_that_is_not_exact_in_binary64_is_refused():
    # all slices at +-127, k = 64: a diagonal of 9 products has 9 * 64 * 127^2 ~ 2^23.1; six diagonals span
    # 35 more bits -> beyond 2^53 units
    x = 1.0 - 2.0 ** -53
    A = np.full((2, 64), x)
    B = np.full((64, 2), x)
    oracle.dgemm3(A, B, 9, 9, 7, Q=4)
    with pytest.raises(oracle.OracleError) as ei:
        oracle.dgemm3(A, B, 9, 9, 7, Q=6)
    assert ei.value.code == oracle.BAD_ARG


def test_levels_never_lose_accuracy_on_the_benchmark_distribution():
    # rounding errors only arise across levels (subsection "Accumulation in floating-point arithmetic"):
    # with fewer roundings the distance to the exact reduced product cannot grow on average
    A, B = workloads.lognormal(8, 8, 64, 0.5, seed=12)
    Af, Bf = ex.frac_matrix(A), ex.frac_matrix(B)
    want = ex.reduced_product_exact(Af, Bf, 10, 7)
    err = {}
    for Q in (1, 3):
        C = oracle.dgemm3(A, B, 10, 10, 7, Q=Q)
        err[Q] = sum(abs(Fraction(float(C[i, j])) - want[i][j]) for i in range(8) for j in range(8))
    assert err[3] <= err[1]
