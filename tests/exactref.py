"""Exact rational helpers for pinning the oracle.

Everything here works on ``fractions.Fraction`` values and follows the paper's
*definitions* (not the oracle's shift-and-mask route), so that an agreement between the two
is evidence and not a tautology.  Only for tiny inputs.
"""
from fractions import Fraction
import math


def frac_matrix(X):
    return [[Fraction(float(v)) for v in row] for row in X]


def scale_exponent(M):
    """Smallest integer e with 2**e > M  (eq. (alpha-def): alpha = 2**(floor(log2 M)+1)).
    M == 0 -> 0 (sentinel used by this build for an all-zero block)."""
    M = Fraction(M)
    if M == 0:
        return 0
    e = 0
    while Fraction(2) ** e <= M:
        e += 1
    while Fraction(2) ** (e - 1) > M:
        e -= 1
    return e


def block_exponents(side, X):
    """X: list of rows of Fractions. side 'A': per row; 'B': per column."""
    rows, cols = len(X), len(X[0]) if X else 0
    if side == "A":
        return [scale_exponent(max((abs(v) for v in X[i]), default=0)) for i in range(rows)]
    return [scale_exponent(max((abs(X[i][j]) for i in range(rows)), default=0)) for j in range(cols)]


def int_part(x):
    """[x]: floor for x >= 0, ceil for x < 0 (the operator under eq. (bit-splitting-alg))."""
    x = Fraction(x)
    return math.floor(x) if x >= 0 else math.ceil(x)


def slices_by_recursion(x, e, s, t):
    """Slices of one entry by the recursion of eq. (bit-splitting-alg):
    x_(l) = [2^{lt} (x / 2^e - sum_{r<l} 2^{-rt} x_(r))]."""
    y = Fraction(x) / Fraction(2) ** e
    out = []
    acc = Fraction(0)
    for l in range(1, s + 1):
        v = int_part(Fraction(2) ** (l * t) * (y - acc))
        out.append(v)
        acc += Fraction(v) / Fraction(2) ** (l * t)
    return out


def truncate(x, e, r, t):
    """x with everything below bit r*t of x / 2^e chopped (round toward zero); r = 0 gives 0."""
    if r <= 0:
        return Fraction(0)
    x = Fraction(x)
    q = Fraction(2) ** (e - r * t)
    return int_part(x / q) * q


def nearest(x, e, r, t):
    """x rounded to the nearest multiple of 2^{e - r t} (ties: the even multiple); r = 0 gives 0 for
    |x| < 2^{e-1}.  Python rounds a Fraction to the nearest integer with ties to even."""
    q = Fraction(2) ** (e - r * t)
    return round(Fraction(x) / q) * q


def slices_nearest(x, e, s, t):
    """Round-to-nearest slices relative to the scale 2^(e+1), by the closed form: the first l slices
    together are the nearest integer to x / 2^(e+1) * 2^(lt), so slice l is the difference between
    that integer and 2^t times the previous one."""
    y = Fraction(x) / Fraction(2) ** (e + 1)
    R = [round(y * Fraction(2) ** (l * t)) for l in range(0, s + 1)]
    return [R[l] - 2 ** t * R[l - 1] for l in range(1, s + 1)]


def matmul(A, B):
    m, k, n = len(A), len(B), len(B[0])
    return [[sum((A[i][kk] * B[kk][j] for kk in range(k)), Fraction(0)) for j in range(n)] for i in range(m)]


def absmat(A):
    return [[abs(v) for v in row] for row in A]


def diagonal_terms(A, B, s, t, full=False, sB=None, rounding=False):
    """Exact value of each diagonal's contribution alpha beta^T o 2^{-dt} sum_{l+h=d} A_(l) B^(h),
    written with truncation operators only:  2^{-lt} alpha A_(l) = T_l(A) - T_{l-1}(A)  (this is
    eq. (slices-eq) read backwards).  Returns {d: matrix of Fractions}.
    rounding: the round-to-nearest variant, scales 2^(e+1) and the nearest-multiple operator in
    place of truncation; the exponents returned are then e + 1."""
    m, k, n = len(A), len(B), len(B[0])
    sA, sB = s, (s if sB is None else sB)
    eA = block_exponents("A", A)
    eB = block_exponents("B", B)
    cut = truncate
    if rounding:
        eA = [e + 1 for e in eA]
        eB = [e + 1 for e in eB]
        cut = nearest
    dA = {l: [[cut(A[i][kk], eA[i], l, t) - cut(A[i][kk], eA[i], l - 1, t) for kk in range(k)]
              for i in range(m)] for l in range(1, sA + 1)}
    dB = {h: [[cut(B[kk][j], eB[j], h, t) - cut(B[kk][j], eB[j], h - 1, t) for j in range(n)]
              for kk in range(k)] for h in range(1, sB + 1)}
    out = {}
    dmax = sA + sB if full else max(sA, sB) + 1
    for d in range(2, dmax + 1):
        acc = [[Fraction(0)] * n for _ in range(m)]
        for l in range(1, sA + 1):
            h = d - l
            if h < 1 or h > sB:
                continue
            P = matmul(dA[l], dB[h])
            for i in range(m):
                for j in range(n):
                    acc[i][j] += P[i][j]
        out[d] = acc
    return out, eA, eB


def pair_terms(A, B, s, t):
    """Exact value of every single product's contribution alpha beta^T o 2^{-(l+h)t} A_(l) B^(h), l + h <= s + 1,
    from truncation operators only (as diagonal_terms).  Returns ({(l, h): matrix of Fractions}, eA, eB)."""
    m, k, n = len(A), len(B), len(B[0])
    eA = block_exponents("A", A)
    eB = block_exponents("B", B)
    dA = {l: [[truncate(A[i][kk], eA[i], l, t) - truncate(A[i][kk], eA[i], l - 1, t) for kk in range(k)]
              for i in range(m)] for l in range(1, s + 1)}
    dB = {h: [[truncate(B[kk][j], eB[j], h, t) - truncate(B[kk][j], eB[j], h - 1, t) for j in range(n)]
              for kk in range(k)] for h in range(1, s + 1)}
    return {(l, h): matmul(dA[l], dB[h]) for l in range(1, s + 1) for h in range(1, s + 2 - l)}, eA, eB


def accumulate_levels(terms, eA, eB, Q, i, j):
    """Entry (i, j) of C from the exact diagonal terms: the diagonals d = 2, 3, ... are taken Q at a
    time, each level summed exactly (asserted to be a binary64 number once the scales are taken
    out), the levels added one after the other in binary64.  Returns a float."""
    scale = Fraction(2) ** (eA[i] + eB[j])
    ds = sorted(terms)
    S = 0.0
    for start in range(0, len(ds), Q):
        level = sum((terms[d][i][j] for d in ds[start:start + Q]), Fraction(0)) / scale
        f = float(level)
        assert Fraction(f) == level, "level is not exact in binary64"
        S = S + f
    return math.ldexp(S, eA[i] + eB[j])


def reduced_product_exact(A, B, s, t, full=False, sB=None, rounding=False):
    """C' of eq. (c-prime) (or C-tilde of eq. (wtc-expr) when full) as exact Fractions;
    s slices of A and sB (default s) slices of B."""
    terms, _, _ = diagonal_terms(A, B, s, t, full, sB, rounding)
    m, n = len(A), len(B[0])
    C = [[Fraction(0)] * n for _ in range(m)]
    for d in sorted(terms):
        for i in range(m):
            for j in range(n):
                C[i][j] += terms[d][i][j]
    return C


def kappa(side, X):
    """2 * max over blocks of max|x| / min|x| over the nonzero entries of the block
    (eq. (a-bound-row-2), eq. (b-bound)); as a Fraction."""
    rows, cols = len(X), len(X[0])
    blocks = X if side == "A" else [[X[i][j] for i in range(rows)] for j in range(cols)]
    worst = Fraction(0)
    for blk in blocks:
        nz = [abs(v) for v in blk if v != 0]
        if nz:
            worst = max(worst, max(nz) / min(nz))
    return 2 * worst


def bit_spread_slices(side, X, t):
    """Minimum slice count that keeps every bit, by the 'bit spread' recipe of the block-LU
    experiment: per block, (largest exponent - smallest exponent) + widest significand spread,
    maximised over blocks, divided by t and rounded up.  X holds Python floats.
    This recipe is an upper estimate; the exact minimum is min_exact_slices()."""
    rows, cols = len(X), len(X[0])
    blocks = X if side == "A" else [[X[i][j] for i in range(rows)] for j in range(cols)]
    worst = 0
    for blk in blocks:
        nz = [v for v in blk if v != 0]
        if not nz:
            continue
        exps = [math.frexp(v)[1] for v in nz]
        spreads = []
        for v in nz:
            mant = int(abs(Fraction(v)) * Fraction(2) ** 1200)
            spreads.append(mant.bit_length() - ((mant & -mant).bit_length() - 1))
        worst = max(worst, max(exps) - min(exps) + max(spreads))
    return -(-worst // t)


def min_exact_slices(side, X, t):
    """s* of eq. (exact-splitting): smallest s with truncate(x, e, s) == x for all entries."""
    Xf = frac_matrix(X)
    e = block_exponents(side, Xf)
    rows, cols = len(Xf), len(Xf[0])
    s = 1
    while True:
        ok = all(truncate(Xf[i][j], e[i] if side == "A" else e[j], s, t) == Xf[i][j]
                 for i in range(rows) for j in range(cols))
        if ok:
            return s
        s += 1
