/*
 * CPU oracle for the integer-slice (Ootomo-Ozaki-Yokota) matrix product.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from the product path.
 *
 * It follows the paper's Algorithm 1 ("Matrix multiplication using an integer
 * MMA unit") step by step, in the paper's notation:
 *   alpha_i, beta_j   eq. (alpha-def), (beta-def)          -> oz_oracle_exponents
 *   A_(l), B^(h)      eq. (bit-splitting-alg), bit view     -> oz_oracle_split
 *                     the same recursion with round-to-nearest
 *                     (second tweak of the "Enhanced algorithm") -> oz_oracle_split_nearest
 *   A_(l) B^(h)       exact integer products, eq. (wtc-expr)-> oz_oracle_slice_product
 *   S, C              Alg. 1 accumulation and final scaling -> oz_oracle_dgemm, _dgemm2, _dgemm3
 *                     (by products, by diagonals, by levels of diagonals)
 *   kappa_A, kappa_B  eq. (a-bound-row-2), (b-bound)        -> oz_oracle_kappa
 *   slice estimate    eq. (err-bound) and the recipe of the
 *                     "Discussion" subsection of Sect. 4    -> oz_oracle_estimate_slices
 *
 * All matrices are column-major with BLAS-style leading dimensions.
 * Slices are stored one int8 per entry (t <= 7, so |slice| <= 2^t - 1 <= 127).
 * Integer products are formed in int64, so they are exact for every k an int
 * can hold (k * 127^2 < 2^63).  The only rounding anywhere is in the binary64
 * additions of the accumulation step.
 *
 * Parity status: every function here is pinned by tests/test_oracle_pins.py
 * (worked example of Sect. 3, exact rational arithmetic, closed forms).
 * Unpinned: the absolute error values plotted in the paper's figures (their
 * data files are not available) -- "parity unpinned" for those only.
 *
 * Build:  gcc -O2 -fopenmp -ffp-contract=off -fPIC -shared -o liboracle.so ozimmu_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define OZ_ORACLE_OK 0
#define OZ_ORACLE_BAD_ARG 1
#define OZ_ORACLE_NONFINITE 2
#define OZ_ORACLE_UNREACHABLE 4

#define OZ_ORACLE_MAX_SLICES 64

int oz_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* |x| = I * 2^q with I the integer significand (0 <= I < 2^53).  Sect. 2. */
static void decompose(double x, int *neg, uint64_t *I, int *q)
{
    uint64_t u;
    memcpy(&u, &x, 8);
    *neg = (int)(u >> 63);
    int E = (int)((u >> 52) & 0x7ff);
    uint64_t f = u & 0xfffffffffffffULL;
    if (E == 0) { *I = f; *q = -1074; }               /* subnormal or zero */
    else        { *I = f | (1ULL << 52); *q = E - 1075; }
}

/*
 * e = floor(log2 M) + 1, so that 2^e is the smallest power of two strictly
 * larger than M -- eq. (alpha-def).  Computed from the representation, never
 * through log2().  M = 0 gives the sentinel e = 0 (the paper assumes no zero
 * row; any scale works because every slice of such a row is zero).
 */
static int exponent_above(double M)
{
    if (M == 0.0) return 0;
    int e;
    (void)frexp(M, &e);          /* M = f * 2^e, 0.5 <= f < 1 */
    return e;
}

/*
 * Scale exponents.  side 'A': one per row of X (rows entries);
 * side 'B': one per column of X (cols entries).   alpha_i = 2^e[i].
 */
int oz_oracle_exponents(char side, int rows, int cols, const double *X, int ldx, int32_t *e)
{
    if ((side != 'A' && side != 'B') || rows < 0 || cols < 0 || ldx < (rows > 1 ? rows : 1)) return OZ_ORACLE_BAD_ARG;
    int nblk = side == 'A' ? rows : cols;
    int len = side == 'A' ? cols : rows;
    for (int b = 0; b < nblk; ++b) {
        double M = 0.0;
        for (int r = 0; r < len; ++r) {
            double x = side == 'A' ? X[b + (size_t)r * ldx] : X[r + (size_t)b * ldx];
            if (!isfinite(x)) return OZ_ORACLE_NONFINITE;
            if (fabs(x) > M) M = fabs(x);
        }
        e[b] = exponent_above(M);
    }
    return OZ_ORACLE_OK;
}

/*
 * Slice l (1-based) of x relative to the scale 2^e, with t bits per slice:
 * the bits of |x| / 2^e in positions (l-1)t+1 .. lt after the binary point,
 * carrying the sign of x -- bit-level view of eq. (bit-splitting-alg).
 * floor(|x| 2^{lt-e}) mod 2^t  with |x| = I 2^q  is a shift and a mask.
 */
static int slice_of(double x, int e, int l, int t)
{
    int neg, q;
    uint64_t I;
    decompose(x, &neg, &I, &q);
    long sh = (long)e - q - (long)l * t;     /* right shift that aligns bit lt with bit 0 */
    uint64_t v;
    if (sh >= 64) v = 0;
    else if (sh >= 0) v = I >> sh;
    else if (-sh >= t) v = 0;                /* all of I lies above this slice's window */
    else v = I << (-sh);
    int d = (int)(v & ((1u << t) - 1u));
    return neg ? -d : d;
}

/*
 * planes[(l-1) * rows * cols + r + c * rows] = slice l of X[r, c]  (l = 1..s),
 * each plane column-major with leading dimension rows.
 * e: the exponents from oz_oracle_exponents for the same side.
 */
int oz_oracle_split(char side, int rows, int cols, const double *X, int ldx, int s, int t,
                    const int32_t *e, int8_t *planes)
{
    if ((side != 'A' && side != 'B') || rows < 0 || cols < 0 || ldx < (rows > 1 ? rows : 1) ||
        s < 1 || s > OZ_ORACLE_MAX_SLICES || t < 1 || t > 7) return OZ_ORACLE_BAD_ARG;
    size_t plane = (size_t)rows * cols;
    for (int c = 0; c < cols; ++c)
        for (int r = 0; r < rows; ++r) {
            double x = X[r + (size_t)c * ldx];
            if (!isfinite(x)) return OZ_ORACLE_NONFINITE;
            int ex = side == 'A' ? e[r] : e[c];
            for (int l = 1; l <= s; ++l)
                planes[(size_t)(l - 1) * plane + r + (size_t)c * rows] = (int8_t)slice_of(x, ex, l, t);
        }
    return OZ_ORACLE_OK;
}

/*
 * Round-to-nearest splitting (second tweak of the "Enhanced algorithm" paragraph of Sect. 3).
 * The recursion of eq. (bit-splitting-alg),
 *     A_(l) = [ 2^{lt} ( x - sum_{r<l} 2^{-rt} A_(r) ) ],
 * with [.] = round to nearest (ties to even) instead of truncation.  Rounding up can carry into
 * the next higher slice, so the first slice may only use t-1 bits: the block is scaled by
 * 2^{e+1} instead of 2^e, x = a / 2^{e+1} lies in (-1/2, 1/2), and every slice lies in
 * [-2^{t-1}, 2^{t-1}].  The paper gives no formula for this variant; this is the reading taken.
 *
 * Exact arithmetic: the scaled residual rho = 2^{(l-1)t} (x - sum_{r<l} ...) is kept as the dyadic
 * number N / 2^G (N a signed integer).  One step: y = 2^t rho, A_(l) = round(y), rho <- y - A_(l).
 */
static void slices_nearest(double x, int e, int s, int t, int *out)
{
    int neg, q;
    uint64_t I;
    decompose(x, &neg, &I, &q);
    int64_t N = neg ? -(int64_t)I : (int64_t)I;
    long G = (long)e + 1 - q;                   /* x / 2^{e+1} = N / 2^G */
    for (int l = 1; l <= s; ++l) {
        long g = G - t;                         /* y = N / 2^g */
        int64_t A;
        if (N == 0) { A = 0; }
        else if (g <= 0) { A = N * ((int64_t)1 << (-g)); N = 0; }      /* y is an integer */
        else if (g >= 62) { A = 0; G = g; }                            /* |y| < 2^53 / 2^62 < 1/2 */
        else {
            uint64_t mag = (uint64_t)(N < 0 ? -N : N), D = (uint64_t)1 << g;
            uint64_t a = mag >> g, rem = mag & (D - 1), half = D >> 1;
            if (rem > half || (rem == half && (a & 1))) ++a;           /* nearest, ties to even */
            A = N < 0 ? -(int64_t)a : (int64_t)a;
            N -= A * (int64_t)D;
            G = g;
        }
        out[l - 1] = (int)A;
    }
}

/*
 * planes as in oz_oracle_split, slices by round-to-nearest relative to the scale 2^{e+1}:
 *     x ~ 2^{e+1} sum_l 2^{-lt} A_(l).     e: the exponents from oz_oracle_exponents.
 */
int oz_oracle_split_nearest(char side, int rows, int cols, const double *X, int ldx, int s, int t,
                            const int32_t *e, int8_t *planes)
{
    if ((side != 'A' && side != 'B') || rows < 0 || cols < 0 || ldx < (rows > 1 ? rows : 1) ||
        s < 1 || s > OZ_ORACLE_MAX_SLICES || t < 2 || t > 7) return OZ_ORACLE_BAD_ARG;
    size_t plane = (size_t)rows * cols;
    int sl[OZ_ORACLE_MAX_SLICES];
    for (int c = 0; c < cols; ++c)
        for (int r = 0; r < rows; ++r) {
            double x = X[r + (size_t)c * ldx];
            if (!isfinite(x)) return OZ_ORACLE_NONFINITE;
            slices_nearest(x, side == 'A' ? e[r] : e[c], s, t, sl);
            for (int l = 1; l <= s; ++l) planes[(size_t)(l - 1) * plane + r + (size_t)c * rows] = (int8_t)sl[l - 1];
        }
    return OZ_ORACLE_OK;
}

/* P = Al * Bh exactly, Al m-by-k (ld m), Bh k-by-n (ld k), P m-by-n (ld m), all column-major. */
int oz_oracle_slice_product(int m, int n, int k, const int8_t *Al, const int8_t *Bh, int64_t *P)
{
    if (m < 0 || n < 0 || k < 0) return OZ_ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < n; ++j) {
        int64_t *p = P + (size_t)j * m;
        for (int i = 0; i < m; ++i) p[i] = 0;
        for (int kk = 0; kk < k; ++kk) {
            int64_t b = Bh[kk + (size_t)j * k];
            const int8_t *a = Al + (size_t)kk * m;
            for (int i = 0; i < m; ++i) p[i] += (int64_t)a[i] * b;
        }
    }
    return OZ_ORACLE_OK;
}

/*
 * C ~ A B by Algorithm 1 with sA slices of A and sB slices of B, t bits each.
 *
 * Products computed (full = 0): A_(l) B^(h) with l <= sA, h <= sB and l + h <= max(sA, sB) + 1 --
 * Algorithm 1's rule l + h <= s + 1 in the extension to different slice counts stated at the
 * start of the subsection "Reduction in number of products".  full = 1: all sA * sB products
 * (subsection "Computation of all products").
 *
 * nearest = 0: slices by truncation (oz_oracle_split), scales 2^e.
 * nearest = 1: slices by round-to-nearest (oz_oracle_split_nearest), scales 2^{e+1}.
 *
 * order 0  "by diagonals" (the accumulation order analysed in the subsection
 *          "Accumulation in floating-point arithmetic" and the first tweak of
 *          the "Enhanced algorithm"): D_d = sum of A_(l) B^(d-l) over the
 *          computed pairs, exactly in integers.  The diagonals d = 2, 3, ... are
 *          taken Q at a time (a "level" of that subsection): the level's value
 *              sum_{d in level} 2^{-dt} D_d
 *          is formed exactly (as an integer multiple of 2^{-t dl}, dl the level's last
 *          diagonal; it must be below 2^53 units, else OZ_ORACLE_BAD_ARG: such a level is
 *          not exact in binary64), then S <- S + level, one binary64 rounding per level.
 *          Q = 1 is the plain diagonal order.
 * order 1  literal loop nest of Algorithm 1: l outer, h inner, one binary64
 *          addition per product (Q ignored).
 *
 * Final step: C = diag(alpha) S diag(beta), i.e. ldexp(S_ij, eA_i + eB_j) with the exponents
 * of the scales used (e or e + 1).  Optional outputs (may be NULL): eA[m], eB[n], those exponents.
 */
int oz_oracle_dgemm3(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                     double *C, int ldc, int sA, int sB, int t, int order, int full, int nearest, int Q,
                     int32_t *eA_out, int32_t *eB_out)
{
    if (m < 0 || n < 0 || k < 0 || sA < 1 || sA > OZ_ORACLE_MAX_SLICES || sB < 1 || sB > OZ_ORACLE_MAX_SLICES ||
        t < 1 || t > 7 || lda < (m > 1 ? m : 1) || ldb < (k > 1 ? k : 1) || ldc < (m > 1 ? m : 1) ||
        (order != 0 && order != 1) || (full != 0 && full != 1) || (nearest != 0 && nearest != 1) ||
        (nearest && t < 2) || Q < 1) return OZ_ORACLE_BAD_ARG;
    if (m == 0 || n == 0) return OZ_ORACLE_OK;

    int32_t *eA = malloc(sizeof(int32_t) * (size_t)m);
    int32_t *eB = malloc(sizeof(int32_t) * (size_t)n);
    int8_t *pa = malloc((size_t)sA * m * (k > 0 ? k : 1));
    int8_t *pb = malloc((size_t)sB * n * (k > 0 ? k : 1));
    int rc = OZ_ORACLE_BAD_ARG;
    if (!eA || !eB || !pa || !pb) goto done;
    if ((rc = oz_oracle_exponents('A', m, k, A, lda, eA))) goto done;
    if ((rc = oz_oracle_exponents('B', k, n, B, ldb, eB))) goto done;
    if (nearest) {
        if ((rc = oz_oracle_split_nearest('A', m, k, A, lda, sA, t, eA, pa))) goto done;
        if ((rc = oz_oracle_split_nearest('B', k, n, B, ldb, sB, t, eB, pb))) goto done;
        for (int i = 0; i < m; ++i) eA[i] += 1;
        for (int j = 0; j < n; ++j) eB[j] += 1;
    } else {
        if ((rc = oz_oracle_split('A', m, k, A, lda, sA, t, eA, pa))) goto done;
        if ((rc = oz_oracle_split('B', k, n, B, ldb, sB, t, eB, pb))) goto done;
    }

    const size_t planeA = (size_t)m * k, planeB = (size_t)k * n;
    const int smax = sA > sB ? sA : sB;
    const int dmax = full ? sA + sB : smax + 1;     /* largest l + h of a computed product */

    int inexact_level = 0;
#pragma omp parallel
    {
        int64_t *p = malloc(sizeof(int64_t) * (size_t)m);   /* one product column   */
        int64_t *D = malloc(sizeof(int64_t) * (size_t)m);   /* one diagonal column  */
        __int128 *L = malloc(sizeof(__int128) * (size_t)m); /* one level column, in units of 2^{-t d} */
        double *S = malloc(sizeof(double) * (size_t)m);
#pragma omp for schedule(dynamic, 1)
        for (int j = 0; j < n; ++j) {
            for (int i = 0; i < m; ++i) S[i] = 0.0;
            if (order == 0) {
                for (int i = 0; i < m; ++i) L[i] = 0;
                for (int d = 2; d <= dmax; ++d) {
                    for (int i = 0; i < m; ++i) D[i] = 0;
                    for (int l = 1; l <= sA; ++l) {
                        int h = d - l;
                        if (h < 1 || h > sB) continue;
                        const int8_t *al = pa + (size_t)(l - 1) * planeA;
                        const int8_t *bh = pb + (size_t)(h - 1) * planeB + (size_t)j * k;
                        for (int kk = 0; kk < k; ++kk) {
                            int64_t b = bh[kk];
                            const int8_t *a = al + (size_t)kk * m;
                            for (int i = 0; i < m; ++i) D[i] += (int64_t)a[i] * b;
                        }
                    }
                    /* level so far, now in units of 2^{-t d}:  L <- 2^t L + D_d  (exact) */
                    for (int i = 0; i < m; ++i) L[i] = L[i] * ((__int128)1 << t) + D[i];
                    if ((d - 1) % Q == 0 || d == dmax) {            /* d closes a level */
                        for (int i = 0; i < m; ++i) {
                            __int128 a = L[i] < 0 ? -L[i] : L[i];
                            if (a >= ((__int128)1 << 53)) {
#pragma omp atomic write
                                inexact_level = 1;
                            }
                            S[i] = S[i] + ldexp((double)(int64_t)L[i], -d * t);
                            L[i] = 0;
                        }
                    }
                }
            } else {
                for (int l = 1; l <= sA; ++l) {
                    for (int h = 1; h <= sB && l + h <= dmax; ++h) {
                        const int8_t *al = pa + (size_t)(l - 1) * planeA;
                        const int8_t *bh = pb + (size_t)(h - 1) * planeB + (size_t)j * k;
                        for (int i = 0; i < m; ++i) p[i] = 0;
                        for (int kk = 0; kk < k; ++kk) {
                            int64_t b = bh[kk];
                            const int8_t *a = al + (size_t)kk * m;
                            for (int i = 0; i < m; ++i) p[i] += (int64_t)a[i] * b;
                        }
                        for (int i = 0; i < m; ++i) S[i] = S[i] + ldexp((double)p[i], -(l + h) * t);
                    }
                }
            }
            for (int i = 0; i < m; ++i) C[i + (size_t)j * ldc] = ldexp(S[i], eA[i] + eB[j]);
        }
        free(p); free(D); free(L); free(S);
    }
    if (eA_out) memcpy(eA_out, eA, sizeof(int32_t) * (size_t)m);
    if (eB_out) memcpy(eB_out, eB, sizeof(int32_t) * (size_t)n);
    rc = inexact_level ? OZ_ORACLE_BAD_ARG : OZ_ORACLE_OK;
done:
    free(eA); free(eB); free(pa); free(pb);
    return rc;
}

/* Slices by truncation, accumulation diagonal by diagonal (or product by product). */
int oz_oracle_dgemm2(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                     double *C, int ldc, int sA, int sB, int t, int order, int full,
                     int32_t *eA_out, int32_t *eB_out)
{
    return oz_oracle_dgemm3(m, n, k, A, lda, B, ldb, C, ldc, sA, sB, t, order, full, 0, 1, eA_out, eB_out);
}

/* Algorithm 1 as printed: the same number s of slices for A and B. */
int oz_oracle_dgemm(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                    double *C, int ldc, int s, int t, int order, int full,
                    int32_t *eA_out, int32_t *eB_out)
{
    return oz_oracle_dgemm2(m, n, k, A, lda, B, ldb, C, ldc, s, s, t, order, full, eA_out, eB_out);
}

/*
 * Number of products the reduced variant computes,
 *   chi(sA, sB) = sm (2 sM - sm + 1) / 2,  sM = max, sm = min
 * (subsection "Reduction in number of products").
 */
int oz_oracle_chi(int sA, int sB)
{
    int sM = sA > sB ? sA : sB, sm = sA > sB ? sB : sA;
    return sm * (2 * sM - sm + 1) / 2;
}

/*
 * kappa = 2 max_blocks ( max |x| / min |x| ), eq. (a-bound-row-2) for side 'A'
 * (blocks = rows) and eq. (b-bound) for side 'B' (blocks = columns).  The
 * minimum runs over the nonzero entries of a block (a zero entry has no
 * conversion error); a block of zeros is skipped; no nonzero entry: kappa = 0.
 */
int oz_oracle_kappa(char side, int rows, int cols, const double *X, int ldx, double *kappa)
{
    if ((side != 'A' && side != 'B') || rows < 0 || cols < 0 || ldx < (rows > 1 ? rows : 1)) return OZ_ORACLE_BAD_ARG;
    int nblk = side == 'A' ? rows : cols;
    int len = side == 'A' ? cols : rows;
    double worst = 0.0;
    for (int b = 0; b < nblk; ++b) {
        double M = 0.0, mn = INFINITY;
        for (int r = 0; r < len; ++r) {
            double x = side == 'A' ? X[b + (size_t)r * ldx] : X[r + (size_t)b * ldx];
            if (!isfinite(x)) return OZ_ORACLE_NONFINITE;
            double ax = fabs(x);
            if (ax > M) M = ax;
            if (ax != 0.0 && ax < mn) mn = ax;
        }
        if (M == 0.0) continue;
        double ratio = M / mn;
        if (ratio > worst) worst = ratio;
    }
    *kappa = 2.0 * worst;
    return OZ_ORACLE_OK;
}

/*
 * Smallest s >= 1 (same count for A and B) with
 *     kappa_A 2^{-st} + kappa_B 2^{-st} <= tol,
 * the left-hand side of eq. (err-bound), evaluated for s = 1, 2, ... as the
 * "Discussion" subsection of Sect. 4 prescribes.  s_max: largest s tried;
 * if none meets tol the result is s_max and the return code says so.
 */
int oz_oracle_estimate_slices(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                              double tol, int t, int s_max, int *s_out, double *kappaA_out, double *kappaB_out)
{
    if (!(tol > 0.0) || t < 1 || t > 7 || s_max < 1) return OZ_ORACLE_BAD_ARG;
    double kA, kB;
    int rc;
    if ((rc = oz_oracle_kappa('A', m, k, A, lda, &kA))) return rc;
    if ((rc = oz_oracle_kappa('B', k, n, B, ldb, &kB))) return rc;
    if (kappaA_out) *kappaA_out = kA;
    if (kappaB_out) *kappaB_out = kB;
    for (int s = 1; s <= s_max; ++s) {
        double lhs = ldexp(kA, -s * t) + ldexp(kB, -s * t);
        if (lhs <= tol) { *s_out = s; return OZ_ORACLE_OK; }
    }
    *s_out = s_max;
    return OZ_ORACLE_UNREACHABLE;
}

/*
 * Slice counts (sA, sB), 1 <= sA, sB <= s_max, that meet
 *     kappa_A 2^{-sA t} + kappa_B 2^{-sB t} <= tol
 * with the fewest products chi(sA, sB): the recipe at the end of the "Discussion" subsection of
 * Sect. 4 (evaluate the left-hand side of eq. (err-bound) for small sA, sB and keep the
 * cheapest combination that delivers the bound).  Ties: smaller sA + sB, then smaller sA.
 * None feasible: (s_max, s_max) and the return code says so.
 */
int oz_oracle_estimate_slices2(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                               double tol, int t, int s_max, int *sA_out, int *sB_out,
                               double *kappaA_out, double *kappaB_out)
{
    if (!(tol > 0.0) || t < 1 || t > 7 || s_max < 1) return OZ_ORACLE_BAD_ARG;
    double kA, kB;
    int rc;
    if ((rc = oz_oracle_kappa('A', m, k, A, lda, &kA))) return rc;
    if ((rc = oz_oracle_kappa('B', k, n, B, ldb, &kB))) return rc;
    if (kappaA_out) *kappaA_out = kA;
    if (kappaB_out) *kappaB_out = kB;
    int best = 0, bA = s_max, bB = s_max;
    for (int sA = 1; sA <= s_max; ++sA)
        for (int sB = 1; sB <= s_max; ++sB) {
            double lhs = ldexp(kA, -sA * t) + ldexp(kB, -sB * t);
            if (!(lhs <= tol)) continue;
            int c = oz_oracle_chi(sA, sB);
            int better = !best || c < oz_oracle_chi(bA, bB) ||
                         (c == oz_oracle_chi(bA, bB) && (sA + sB < bA + bB || (sA + sB == bA + bB && sA < bA)));
            if (better) { best = 1; bA = sA; bB = sB; }
        }
    *sA_out = bA;
    *sB_out = bB;
    return best ? OZ_ORACLE_OK : OZ_ORACLE_UNREACHABLE;
}
