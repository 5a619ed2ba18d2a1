/*
 * ozimmu_bench.h -- benchmark aids and test hooks of libozimmu.  Not part of the method's interface
 * (ozimmu.h): phase timing and calibration helpers used by the benchmark, and hooks with which the parity
 * tests read integer intermediates or steer the choice of kernel.
 *
 * Everything here that keeps host-side state (the phase timer, the two ozimmu_debug_* knobs) is process-wide:
 * the knobs are atomics (a change is seen by every later call of every thread), the phase timer is guarded by a
 * mutex, and both are meant to be driven from ONE thread while no other thread is inside ozimmu_dgemm*.
 */
#ifndef OZIMMU_BENCH_H
#define OZIMMU_BENCH_H

#include "ozimmu.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-phase timing of ozimmu_dgemm, for benchmarks.  Between ozimmu_profile_start(max_calls) and
 * ozimmu_profile_stop(), each ozimmu_dgemm call (up to max_calls <= 4096 of them) records HIP
 * events on its stream before and after its three phases; the calls stay asynchronous.
 * ozimmu_profile_stop waits for the recorded events and returns in phase_ms [host, 3 floats] the
 * average milliseconds per call of: [0] scale extraction (reductions), [1] splitting of A and B,
 * [2] the GEMM kernel (a single launch); *calls [host] receives the number of calls averaged.
 * One timer per process (guarded by a mutex; drive it from one thread); allocates no device memory.
 */
int ozimmu_profile_start(int max_calls);
int ozimmu_profile_stop(int *calls, float *phase_ms);

/*
 * Name, slice count and tile of the GEMM kernel the calling thread's last ozimmu_dgemm* call launched (for a call
 * made of several GEMM launches -- split-k panels, blocks of slice groups -- the path and its last launch), e.g.
 * "gemm_fused16_kernel<7> tile 128x64".  Static thread-local storage, valid until the thread's next call; "" before
 * the first one.  Written by the launchers themselves.
 */
const char *ozimmu_last_gemm_kernel(void);

/*
 * Benchmark aid: the int8 rate (TOP/s, written to *tops [host]) that a register-only loop of
 * v_mfma_i32_32x32x32_i8 sustains on the current device for some tens of milliseconds, with
 * constant (random_operands = 0) or pseudo-random (1) operand registers.  `sink`: device pointer
 * to one int (never written in practice).  Synchronises.  Context for the roofline fraction of the
 * GEMM kernel: the sustained clock of the matrix cores depends on the operand data.
 */
int ozimmu_measure_int8_ceiling(int random_operands, int *sink, float *tops, void *stream);
/* The same with the matrix instruction chosen: shape 0 = v_mfma_i32_32x32x32_i8, 1 = v_mfma_i32_16x16x64_i8 (the
 * one the GEMM kernel for 4 ... 9 slices uses; it spends less energy per product).  random_operands = 2: a
 * register tile of pseudo-random operands (4 x 4 fragments, 2 x 4 for 32x32x32), so that consecutive instructions
 * read different operands, as in a GEMM; other values: OZIMMU_BAD_ARG. */
int ozimmu_measure_int8_ceiling2(int random_operands, int shape, int *sink, float *tops, void *stream);

/*
 * Benchmark aid: the rate of the v_mfma_i32_16x16x64_i8 loop on pseudo-random operands WITH the data movement of the
 * GEMM kernel going on beside it and nothing else of that kernel (no barriers, no waits on the moving data):
 * `lds_reads` operand registers re-read from LDS per 16 matrix instructions (one iteration ahead of their use) and
 * `dma_copies_per_32` LDS-DMA copies of 1 KiB per wavefront per 32 matrix instructions from an L2-resident window of
 * `src` (device pointer, 16-byte aligned, at least 64 KiB, contents arbitrary).  Combinations built:
 * (0, 0), (4, 0), (0, 3), (4, 3) -- the ratios of the kernel for 7 slices --, (3, 2) -- close to those for 9 slices --,
 * (5, 4), (6, 4), (5, 3) -- close to those for 2, 3, 4 slices --, (2, 3), (4, 2), and (0, -3), (4, -3): the 3 copies
 * made through registers (vector load, LDS store) instead of LDS-DMA; others: OZIMMU_BAD_ARG.
 * Writes TOP/s to *tops [host]; synchronises.  Under the board's power cap this is what is left for the matrix cores
 * once the bytes move.
 */
int ozimmu_measure_int8_with_traffic(int lds_reads, int dma_copies_per_32, const void *src, size_t src_bytes,
                                     int *sink, float *tops, void *stream);

/*
 * Benchmark aid: a plain device-to-device copy kernel (`calibration_copy_kernel`) of `bytes` bytes (a multiple
 * of 16, both pointers 16-byte aligned), asynchronous on `stream`.  Its HBM traffic is known exactly -- `bytes`
 * read and `bytes` written -- so the FETCH_SIZE / WRITE_SIZE readings a profiler reports for it give the
 * factors by which the same counters have to be scaled for the other kernels.
 */
int ozimmu_calibration_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Test hooks (used by the parity tests to compare integer intermediates bit for bit).
 * Both read the MFMA-layout planes that ozimmu_dgemm(m, n, k, ..., s, workspace) left in
 * `workspace`, on the same stream.
 *
 * ozimmu_debug_diagonals: D[(d-2) * m * n + i + j*m] = sum_{l+h=d} (A_(l) B^(h))_ij as int32,
 *   d = 2..s+1, produced by the main loop of the fused GEMM kernel (needs
 *   s * k * 127^2 < 2^31 and s <= the fused kernel's limit, else OZIMMU_BAD_ARG).
 * ozimmu_debug_small_tile_limit: ozimmu_dgemm with equal slice counts up to 12 uses a 64 x 64 tile instead of
 *   the tile tabulated for the slice count where that finishes sooner by (rounds of the compute units) x (tile
 *   area) / (relative speed of the kernel); that rule is the default (-1).  0: never the small tile; n > 0: the
 *   small tile whenever the tabulated one would give fewer than n work-groups.  Process-wide host state; lets
 *   the tests run both kernels on the same small inputs.  Returns OZIMMU_BAD_ARG for a value below -1.
 * ozimmu_debug_tile_choice: with 2 ... 6 slices ozimmu_dgemm picks between the tabulated tile (256 x 128,
 *   256 x 128, 128 x 128, 128 x 128, 128 x 128) and an alternative (128 x 128, 128 x 128, 192 x 128, 128 x 64,
 *   128 x 64) by the number of rounds of the compute units each needs; 1 forces the tabulated tile, 2 the alternative, 0 (default) restores the choice.
 *   Process-wide host state.  Returns OZIMMU_BAD_ARG for other values.
 * ozimmu_debug_panel_bytes: when k has to be cut into blocks, C is computed one column panel after the other so
 *   that the int64 totals of a panel take about `bytes` (default 1 GiB; <= 0: all of C at once).  Changes what
 *   ozimmu_workspace_bytes* return: set it before sizing the workspace.  Process-wide host state.
 * ozimmu_debug_slice_product: P[i + j*m] = sum_{kk = k0}^{k1-1} A_(l)[i,kk] B^(h)[kk,j] as int32
 *   for one pair (l, h), 1-based, over the contraction range [k0, k1) with k0 a multiple of 32
 *   and (k1-k0) * 127^2 < 2^31, produced by the generic (pair-by-pair) GEMM kernel.
 */
int ozimmu_debug_diagonals(int m, int n, int k, int s, const void *workspace, int32_t *D, void *stream);
int ozimmu_debug_small_tile_limit(long long tiles);
int ozimmu_debug_tile_choice(int choice);
int ozimmu_debug_panel_bytes(long long bytes);
int ozimmu_debug_slice_product(int m, int n, int k, int s, const void *workspace, int l, int h,
                               int k0, int k1, int32_t *P, void *stream);

#ifdef __cplusplus
}
#endif
#endif
