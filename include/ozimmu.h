/*
 * ozimmu -- binary64 matrix multiplication through int8 slices on MI355X (gfx950).
 *
 * C ~ A B for binary64 A (m-by-k) and B (k-by-n) by the integer-slice scheme of Ootomo,
 * Ozaki and Yokota as stated in Algorithm 1 of "Analysis of Floating-Point Matrix
 * Multiplication Computed via Integer Arithmetic" (Sect. 3), with the accumulation order
 * of the subsection "Accumulation in floating-point arithmetic" (Sect. 4) and the
 * slice-count estimate of the "Discussion" subsection of Sect. 4.
 *
 * Conventions for every entry point
 *   - Matrices are column-major with BLAS-style leading dimensions; D = A B (alpha = 1,
 *     beta = 0, no transposes), the GEMM form the paper's GPU benchmark uses.
 *   - A, B, C, X, planes, exps, workspace are DEVICE pointers owned by the caller.  The
 *     library allocates no device memory.  Pointers marked [host] are host pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on that stream unless stated otherwise.
 *   - Slices hold t = 7 bits (int8 storage, values in [-127, 127]); 1 <= s <= OZIMMU_MAX_SLICES.
 *   - Return value: one of the OZIMMU_* status codes; never throws or aborts.
 *   - Inputs must be finite.  NaN or +-Inf are outside the method's domain (Sect. 3,
 *     first paragraph of "Original algorithm"); they are detected, reported by
 *     ozimmu_check(), and the output is then unspecified (but no fault occurs).
 *     -0.0 is treated as +0.  An all-zero row of A / column of B gets exponent 0 and
 *     yields a zero row / column of C.
 *   - m, n or k equal to 0 is accepted (k = 0 gives C = 0).
 */
#ifndef OZIMMU_H
#define OZIMMU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OZIMMU_OK 0
#define OZIMMU_BAD_ARG 1      /* null pointer, negative size, ld too small, s out of range, workspace too small */
#define OZIMMU_NONFINITE 2    /* NaN or Inf met in A or B */
#define OZIMMU_HIP_ERROR 3    /* a HIP runtime call failed */
#define OZIMMU_UNREACHABLE 4  /* estimator: tolerance not met by any s <= OZIMMU_MAX_SLICES */
#define OZIMMU_TOO_LARGE 5    /* ozimmu_dgemm_static: the problem needs more than OZIMMU_STATIC_WORKSPACE_BYTES */

#define OZIMMU_MAX_SLICES 32
#define OZIMMU_SLICE_BITS 7

/* plane layouts for ozimmu_split */
#define OZIMMU_LAYOUT_PLAIN 0 /* plane l (0-based) at planes + l*rows*cols, column-major like X, ld = rows */
#define OZIMMU_LAYOUT_MFMA 1  /* tiled operand layout read by the GEMM kernel, see ozimmu_split */

/* how an operand is cut into slices (ozimmu_split2, ozimmu_dgemm3) */
#define OZIMMU_SPLIT_TRUNCATE 0 /* eq. (bit-splitting-alg): round towards zero, slices in [-127, 127], scale 2^e */
#define OZIMMU_SPLIT_NEAREST 1  /* second tweak of the "Enhanced algorithm" paragraph: round to nearest,
                                   slices in [-64, 64], scale 2^(e+1) */

/* Human-readable name of a status code (static storage). */
const char *ozimmu_status_string(int status);

/*
 * Bytes of device workspace ozimmu_dgemm / ozimmu_estimate_slices need for this problem:
 * scale exponents, per-row/column reductions, the int8 slice planes of A and B, and int64 totals of the
 * diagonals (8 bytes per diagonal and entry of a column panel of C, panels of about 1 GiB)
 *   - for up to 20 slices only when min(sA, sB) * k > 133144, i.e. when a diagonal's int32 sum could overflow and
 *     k has to be cut into blocks,
 *   - for product sets beyond those kernels (21 ... 32 equal counts; different counts with the larger above 18; all
 *     products of more than 9 slices) always: the products are formed group of slices by group of slices and meet
 *     in the totals; the planes then hold a whole number of groups of 7, 8 or 9 slices per operand (zero slices
 *     appended).
 * Returns 0 for invalid arguments.  Alignment required of the workspace pointer: 256 bytes.
 */
size_t ozimmu_workspace_bytes(int m, int n, int k, int s);

/* Bytes of the `planes` buffer ozimmu_split writes for the given layout (0 if invalid). */
size_t ozimmu_planes_bytes(char side, int rows, int cols, int s, int layout);

/*
 * Slice-count estimate (Sect. 4, eq. (a-bound-row-2), (b-bound), (err-bound)):
 *   kappa_A = 2 max_i ( max_j |a_ij| / min_j |a_ij| ),  kappa_B likewise over columns of B,
 *   minima over the nonzero entries; all-zero rows/columns skipped;
 *   *s_out = smallest s >= 1 with  kappa_A 2^{-7s} + kappa_B 2^{-7s} <= tol.
 * One pass over A and B on the device; SYNCHRONISES the stream to return the result.
 *   s_out  [host] receives s (OZIMMU_MAX_SLICES when unreachable)
 *   kappa  [host] optional (may be NULL): kappa[0] = kappa_A, kappa[1] = kappa_B
 * Returns OZIMMU_OK, OZIMMU_UNREACHABLE, OZIMMU_NONFINITE, OZIMMU_BAD_ARG (tol <= 0 or NaN,
 * workspace smaller than ozimmu_workspace_bytes(m, n, k, 1)) or OZIMMU_HIP_ERROR.
 */
int ozimmu_estimate_slices(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                           double tol, int *s_out, double *kappa,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * Scales and slices of one operand (Algorithm 1, the two scale loops and the two slicing
 * loops; eq. (alpha-def), (beta-def), (bit-splitting-alg)).
 *   side 'A': X is rows-by-cols = m-by-k; row i shares the scale 2^exps[i]; exps has `rows` entries.
 *   side 'B': X is rows-by-cols = k-by-n; column j shares the scale 2^exps[j]; exps has `cols` entries.
 *   exps[b] = floor(log2 max|x|) + 1 over the block (0 for an all-zero block).
 *   Slice l (1-based) of an entry x of a block with exponent e is
 *   sign(x) * ( floor(|x| 2^{7l - e}) mod 2^7 ).
 * layout OZIMMU_LAYOUT_PLAIN: planes[(l-1)*rows*cols + r + c*rows].
 * layout OZIMMU_LAYOUT_MFMA: the operand is viewed as R-by-K with R the scaled dimension
 *   (rows of A / columns of B) and K the contraction dimension, zero-padded to
 *   Rp = roundup(R, 128), Kp = roundup(K, 128), and cut into fragments of 32 (R) by 32 (K)
 *   entries.  Fragment (rb, kb) of slice l starts at byte
 *       (((size_t)rb * (Kp/32) + kb) * s + (l-1)) * 1024
 *   and entry (r, kk) of the fragment sits at byte  ((r + 32*(kk/16)) * 16 + kk%16)  in it:
 *   the 16 bytes lane (r + 32*(kk/16)) of a wavefront feeds to v_mfma_i32_32x32x32_i8.
 * `scratch`: device buffer of ozimmu_split_scratch_bytes(side, rows, cols) bytes, 256-byte
 * aligned, used for the reduction; a NaN/Inf in X is reported by ozimmu_check(scratch, stream).
 */
size_t ozimmu_split_scratch_bytes(char side, int rows, int cols);
int ozimmu_split(char side, int rows, int cols, const double *X, int ldx, int s,
                 int8_t *planes, int32_t *exps, int layout, void *scratch, void *stream);

/*
 * ozimmu_split with the way of slicing chosen by `splitting`.  OZIMMU_SPLIT_TRUNCATE is ozimmu_split.
 * OZIMMU_SPLIT_NEAREST (second tweak of the "Enhanced algorithm" paragraph of Sect. 3, which states the
 * idea -- round the fixed-point representation to nearest instead of truncating it, the first slice
 * then has t-1 bits -- but no formula; the reading implemented is the recursion of eq.
 * (bit-splitting-alg) with round-to-nearest, ties to even, in place of truncation):
 *   exps[b] = floor(log2 max|x|) + 2 over the block (1 for an all-zero block), i.e. the scale is doubled
 *   so that |x| / 2^exps < 1/2;  with R_l = the integer nearest to x 2^{7l - exps} and R_0 = 0,
 *   slice l = R_l - 128 R_{l-1}, a value in [-64, 64];  x ~ 2^exps sum_l 2^{-7l} slice_l  with an error
 *   of at most 2^{exps - 7s - 1}, zero when enough slices are taken.
 */
int ozimmu_split2(char side, int rows, int cols, const double *X, int ldx, int s, int splitting,
                  int8_t *planes, int32_t *exps, int layout, void *scratch, void *stream);

/*
 * C = A B through s int8 slices (Algorithm 1 with k-blocked exact integer accumulation):
 *   1. scale exponents of the rows of A and the columns of B,
 *   2. s slices of each operand,
 *   3. exact integer products A_(l) B^(h) for l + h <= s + 1 on the int8 matrix cores; the
 *      products of one diagonal l + h = d are added exactly in integer arithmetic
 *      (first tweak of the "Enhanced algorithm" paragraph of Sect. 3),
 *   4. S = sum over d = 2, ..., s+1 in this order of 2^{-7d} D_d, one binary64 rounding per
 *      addition; C_ij = 2^{eA_i + eB_j} S_ij.
 * C is m-by-n with leading dimension ldc >= max(1, m).  The result is deterministic
 * (bit-identical from run to run).  Non-finite input is reported by ozimmu_check().
 */
int ozimmu_dgemm(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                 double *C, int ldc, int s, void *workspace, size_t workspace_bytes, void *stream);

/*
 * ozimmu_dgemm for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace (scale exponents, slice planes,
 * split-k totals) is a static device array of OZIMMU_STATIC_WORKSPACE_BYTES inside the library, of which every
 * GPU the library runs on holds one copy until the process ends; the call allocates nothing and calls no
 * allocating routine.  Same result as ozimmu_dgemm, bit for bit.
 *   - Problems with ozimmu_workspace_bytes(m, n, k, s) > OZIMMU_STATIC_WORKSPACE_BYTES return OZIMMU_TOO_LARGE
 *     and touch nothing (64 MiB: e.g. 2048^3 with 7 slices, 1024^3 with 28).
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents (the kernels clear what
 *     they need cleared): calls that overlap on one GPU -- different streams, different threads -- race.  Calls on
 *     one stream are ordered and safe.
 *   - ozimmu_check() is not available for it (the array is not exposed); inputs must be finite.
 */
#define OZIMMU_STATIC_WORKSPACE_BYTES (64u << 20)
int ozimmu_dgemm_static(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                        double *C, int ldc, int s, void *stream);

/*
 * The same with sA slices of A and sB slices of B (Sect. 4, subsection "Reduction in number of
 * products": a well scaled operand needs fewer slices than a badly scaled one).  Products computed:
 *   all_products = 0:  l <= sA, h <= sB, l + h <= max(sA, sB) + 1   (chi(sA, sB) of them)
 *   all_products = 1:  all sA * sB                                   ("Computation of all products")
 * accumulated by diagonals l + h = 2, 3, ... as in ozimmu_dgemm; ozimmu_dgemm(s) equals
 * ozimmu_dgemm2(s, s, 0) bit for bit.  Workspace: ozimmu_workspace_bytes2(m, n, k, sA, sB, all_products).
 * (Counts that differ little are run as equal counts with zero slices appended to the short operand, which
 * leaves every diagonal sum and hence the result unchanged; the workspace size accounts for it.)
 */
size_t ozimmu_workspace_bytes2(int m, int n, int k, int sA, int sB, int all_products);
int ozimmu_dgemm2(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                  double *C, int ldc, int sA, int sB, int all_products,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * The two accuracy variants on top of ozimmu_dgemm2 (same workspace size):
 *   splitting        OZIMMU_SPLIT_TRUNCATE or OZIMMU_SPLIT_NEAREST (see ozimmu_split2); with the latter the
 *                    exponents ozimmu_get_exponents returns are those of the doubled scales.
 *   level_diagonals  Q >= 1: the binary64 accumulation takes the diagonals l + h = 2, 3, ... Q at a time
 *                    (the "levels" of the subsection "Accumulation in floating-point arithmetic" of
 *                    Sect. 4): the Q terms 2^{-7d} D_d of a level are added to each other without rounding
 *                    error, then the level is added to S with one rounding; the last level may be
 *                    shorter.  Q = 1 is the order of ozimmu_dgemm.  Q must not exceed
 *                    ozimmu_max_level_diagonals(k, sA, sB), the largest Q for which every level is
 *                    certain to be a binary64 number: min(sA, sB) k 127^2 (2^{7Q} - 1) / 127 < 2^53
 *                    (4 at k = 8192, 3 at k = 2^17 for 4 to 32 slices; 3 is the value the paper derives for a
 *                    full 31-bit accumulator); a larger Q returns OZIMMU_BAD_ARG.
 * ozimmu_dgemm3(..., all_products, OZIMMU_SPLIT_TRUNCATE, 1, ...) equals ozimmu_dgemm2 bit for bit.
 */
int ozimmu_max_level_diagonals(int k, int sA, int sB);
int ozimmu_dgemm3(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                  double *C, int ldc, int sA, int sB, int all_products, int splitting, int level_diagonals,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * Two-dimensional slice estimate ("Discussion" subsection of Sect. 4): among all 1 <= sA, sB <=
 * OZIMMU_MAX_SLICES with  kappa_A 2^{-7 sA} + kappa_B 2^{-7 sB} <= tol  the pair with the fewest
 * products chi(sA, sB) = sm (2 sM - sm + 1) / 2; ties go to the smaller sA + sB, then the smaller sA.
 * Arguments and return codes as ozimmu_estimate_slices; none feasible: both = OZIMMU_MAX_SLICES and
 * OZIMMU_UNREACHABLE.  SYNCHRONISES.
 */
int ozimmu_estimate_slices2(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                            double tol, int *sA_out, int *sB_out, double *kappa,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * Waits for the stream and returns OZIMMU_NONFINITE if the last ozimmu_dgemm /
 * ozimmu_estimate_slices that used this workspace met a NaN or Inf, else OZIMMU_OK.
 */
int ozimmu_check(void *workspace, void *stream);

/*
 * After ozimmu_dgemm(m, n, k, ..., s, workspace, ...) on the same stream: copies the scale
 * exponents it computed to eA[m] and eB[n] (device pointers, either may be NULL).
 */
int ozimmu_get_exponents(int m, int n, int k, int s, const void *workspace, int32_t *eA, int32_t *eB,
                         void *stream);

/* Benchmark aids (phase timing, calibration copy, sustained matrix-core rate) and the hooks of the parity
 * tests are declared in ozimmu_bench.h; nothing in this header depends on them. */

#ifdef __cplusplus
}
#endif
#endif
