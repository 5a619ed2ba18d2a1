// Internal declarations shared by the HIP translation units of libozimmu.
// (Nothing here is used by, or shared with, the CPU oracle.)
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/ozimmu.h"
#include "../../include/ozimmu_bench.h"

namespace oz {

constexpr int kSliceBits = OZIMMU_SLICE_BITS;   // t = 7: INT8 = I_7 in the paper's notation
constexpr int kFrag = 32;                       // fragment edge: 32 (R) x 32 (K) int8 = 1 KiB
constexpr int kFragBytes = 1024;
constexpr int kPad = 128;                       // R and K are zero-padded to multiples of this
// largest contraction length whose int8 x int8 products sum without int32 overflow:
// k * 127^2 <= 2^31 - 1  (accumulator-width discussion of Sect. 3, with the true constant)
constexpr long long kMaxInt32K = 2147483647LL / (127LL * 127LL);   // 133144

inline int round_up(int x, int q) { return (x + q - 1) / q * q; }

// Name and shape of the GEMM kernel the calling thread launched last (reported by ozimmu_last_gemm_kernel for
// benchmarks and profiles; written by the launchers themselves, so it cannot drift from the routing).
void note_gemm_kernel(const char *fmt, ...);
const char *last_gemm_kernel();

// Lets a kernel use `bytes` of dynamic LDS (more than the 64 KiB default), once per device: `done` holds one
// bit per device ordinal.  (Two first calls racing on a device both set the attribute: harmless.)
inline hipError_t allow_dynamic_lds(const void *kernel, int bytes, std::atomic<unsigned long long> &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && (done.load(std::memory_order_acquire) >> dev & 1ULL)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 64) done.fetch_or(1ULL << dev, std::memory_order_release);
    return e;
}

bool fused_handles(int sA, int sB, bool all_products, int m, int n, int k);
size_t fused_totals_bytes(int sA, int sB, bool all_products, int m, int n, int k);
size_t banded_totals_bytes(int sA, int sB, int k);
int fused_max_slices();
// Product sets beyond the fused kernels, run as blocks of the (l, h) grid through the fused kernels: group size and
// slices per entry the planes of A and B hold (the counts rounded up to whole groups, the surplus written as
// zeros).  blocks_plan() is false where the band kernel is the cheaper choice; call it only for product sets
// the fused kernels do not take.  blocks_totals_bytes(): bytes of int64 totals the path needs.
struct BlocksPlan {
    int G, spA, spB;
    long long cost, needed;      // products the blocks compute / products of the requested set
};
bool blocks_plan(int sA, int sB, bool all_products, BlocksPlan *plan);
size_t blocks_totals_bytes(int sA, int sB, bool all_products, int m, int n, int k);

// Slice counts the GEMM runs with.  Different counts that differ little run as EQUAL counts, the short operand
// getting zero slices appended by the slicing kernel: a product with a zero slice adds nothing, so every diagonal
// sum -- and with it the result -- is the one of the product set l <= s_A, h <= s_B, l + h <= max(s_A, s_B) + 1
// (subsection "Reduction in number of products" of Sect. 4), while the kernels for equal counts are faster by more
// than the d (d + 1) / 2 surplus products cost (d = the difference of the counts).  Thresholds from timings at
// 8192^3: (7,8) 14.7 -> 12.2 ms, (5,8) 12.7 -> 12.0, (4,8) 11.6 stays (12.1 as (8,8)), (9,12) 26.5 stays (27.8),
// (12,16) 48.8 -> 47.0, (17,18) 112 -> 64 and (19,20) 128 -> 83 ms (beyond 16 the kernels for different counts read part of the long operand on demand,
// beyond 18 only the band kernel is left).
inline void gemm_slice_counts(int sA, int sB, bool all_products, int &cA, int &cB)
{
    cA = sA;
    cB = sB;
    if (sA == sB) return;
    const int S = sA > sB ? sA : sB, d = S - (sA < sB ? sA : sB);
    if (all_products) {
        // all s_A s_B products: the fused kernel takes equal counts up to 9 (about twice the rate of the band
        // kernel, which serves different counts), so zero slices pay while they at most double the products
        if (S <= 9 && 2 * sA * sB >= S * S) cA = cB = S;
        return;
    }
    const int full = S * (S + 1) / 2, surplus = d * (d + 1) / 2;
    const bool pad = S > 20   ? false
                     : S >= 17 ? 5 * surplus <= 2 * full
                     : S >= 13 ? 10 * surplus <= full
                     : S >= 10 ? 14 * surplus <= full
                               : 5 * surplus <= full;
    if (pad) cA = cB = S;
}

// Which GEMM path takes a product set, and with how many slices per entry in the planes: the fused kernels (cA, cB
// from gemm_slice_counts), else blocks of slice groups (whole groups), else the band kernel (the counts as they are).
enum GemmPath { kPathFused, kPathBlocks, kPathBand };
inline GemmPath gemm_path(int sA, int sB, bool all_products, int m, int n, int k, int &cA, int &cB)
{
    gemm_slice_counts(sA, sB, all_products, cA, cB);
    BlocksPlan p;
    // Different counts with the larger one from 13 on run in the four-wavefront shape of the fused kernel (2450-2580
    // TOP/s at 8192^3); where the groups of the block path fit them with at most 18 % surplus products, that path is
    // the faster one: (7,14) 2450 -> 2950, (8,16) 2560 -> 3095, (6,14) 2440 -> 2680, (9,16) 2580 -> 2780 TOP/s of
    // useful products (and (7,12), 22 % surplus, against the eight-wavefront shape: 2870 -> 2430, so not there).
    const bool blocks_first = !all_products && cA != cB && (cA > cB ? cA : cB) >= 13 && blocks_plan(sA, sB, false, &p) &&
                              100 * p.cost <= 118 * p.needed;
    if (!blocks_first && fused_handles(cA, cB, all_products, m, n, k)) return kPathFused;
    if (blocks_plan(sA, sB, all_products, &p)) {
        cA = cB = p.spA > p.spB ? p.spA : p.spB;       // the block kernel wants the same number of slices per entry in both
        return kPathBlocks;
    }
    cA = sA;
    cB = sB;
    return kPathBand;
}

// Workspace carve-up (all offsets multiples of 256 bytes).
struct Workspace {
    int mp, np, kp;                 // padded extents
    int cA, cB;                     // slices per entry in the planes (gemm_path)
    int path;                       // GemmPath
    size_t off_header;              // 256 B: [0] u32 non-finite flag, [8] u64 kappa_A bits, [16] u64 kappa_B bits
    size_t off_maxA, off_minA;      // u64[mp]: integer view of max |a_ij| / min nonzero |a_ij| per row
    size_t off_maxB, off_minB;      // u64[np]
    size_t off_expA, off_expB;      // i32[mp], i32[np]
    size_t off_planesA, off_planesB;
    size_t off_totals;              // int64 per-tile diagonal totals of the k-blocked fused GEMM (may be empty)
    size_t total;
};

inline Workspace carve(int m, int n, int k, int sA, int sB, bool all_products = false)
{
    Workspace w;
    w.mp = round_up(m > 0 ? m : 1, kPad);
    w.np = round_up(n > 0 ? n : 1, kPad);
    w.kp = round_up(k > 0 ? k : 1, kPad);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
    w.off_header = take(256);
    w.off_maxA = take(8 * (size_t)w.mp);
    w.off_minA = take(8 * (size_t)w.mp);
    w.off_maxB = take(8 * (size_t)w.np);
    w.off_minB = take(8 * (size_t)w.np);
    w.off_expA = take(4 * (size_t)w.mp);
    w.off_expB = take(4 * (size_t)w.np);
    w.path = gemm_path(sA, sB, all_products, m, n, k, w.cA, w.cB);
    w.off_planesA = take((size_t)w.cA * w.mp * w.kp);
    w.off_planesB = take((size_t)w.cB * w.np * w.kp);
    w.off_totals = take(w.path == kPathBlocks  ? blocks_totals_bytes(sA, sB, all_products, m, n, k)
                        : w.path == kPathFused ? fused_totals_bytes(w.cA, w.cB, all_products, m, n, k)
                                               : banded_totals_bytes(w.cA, w.cB, k));
    w.total = off;
    return w;
}

// ---- launchers implemented in reduce.hip -------------------------------------------------
// side 'A': per-row reduction of a rows x cols matrix; side 'B': per-column.
// maxbits/minbits: u64 per block (bit pattern of max |x| and of the smallest nonzero |x|;
// minbits may be null).  flags: u32, bit 0 set when a NaN/Inf is met.
hipError_t launch_reduce(char side, int rows, int cols, const double *X, int ldx,
                         unsigned long long *maxbits, unsigned long long *minbits,
                         unsigned int *flags, hipStream_t st);
// exps[b] from maxbits[b], plus `bias` (1 for round-to-nearest slices, whose scale is twice as large);
// entries b in [nblk, nblk_padded) get 0.  If kappa_bits is non-null (needs minbits) also folds
// 2*max/min into *kappa_bits with an integer atomic max.
hipError_t launch_finalize(const unsigned long long *maxbits, const unsigned long long *minbits,
                           int32_t *exps, int nblk, int nblk_padded, unsigned long long *kappa_bits,
                           int bias, hipStream_t st);
hipError_t launch_clear_header(void *header, hipStream_t st);
// the whole scale extraction of ozimmu_dgemm in three launches: clear, reduce both operands, exponents of both
hipError_t launch_scales_fused(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                               unsigned long long *hdr, unsigned long long *maxA, unsigned long long *maxB,
                               int32_t *expA, int mp, int32_t *expB, int np, int bias, bool finalize, hipStream_t st);

// e = floor(log2 M) + 1 from the bit pattern of M >= 0 (eq. (alpha-def)); the exponent-field
// shortcut described after eq. (beta-def) for normal numbers, leading-zero count for
// subnormal ones, 0 for M = 0.
__device__ __forceinline__ int exponent_above(unsigned long long bits)
{
    if (bits == 0) return 0;
    int E = (int)(bits >> 52);
    if (E) return E - 1022;
    return (64 - __clzll((long long)bits)) - 1074;
}

// ---- launchers implemented in split.hip --------------------------------------------------
// nearest: slices by round-to-nearest (exps must then hold the biased exponents), else by truncation
hipError_t launch_split(char side, int rows, int cols, const double *X, int ldx, int s,
                        const int32_t *exps, int8_t *planes, int layout, bool nearest, hipStream_t st);

// slices of both operands (MFMA layout) in one launch; the planes have room for cA >= sA and cB >= sB slices per
// entry, the slices beyond sA (sB) are written as zeros
// (the exponents are formed here from the maxima of launch_scales_fused -- bit patterns of max |x| per row of A /
// column of B -- and stored to eA, eB, their padding as zeros)
hipError_t launch_split_both(int m, int n, int k, const double *A, int lda, const double *B, int ldb, int sA, int sB,
                             int cA, int cB, const unsigned long long *maxA, const unsigned long long *maxB,
                             int32_t *eA, int32_t *eB, int8_t *pA, int8_t *pB, bool nearest, hipStream_t st);

// ---- launchers implemented in gemm.hip ---------------------------------------------------
// largest s the fused (all diagonals in registers) kernel handles
int fused_max_slices();
// problems with fewer tiles of the tabulated shape than this use the 64 x 64 tile (default 256; 0: never)
void fused_set_small_tile_limit(long long tiles);
// bytes of split-k totals per column panel of C (default 1 GiB; <= 0: no panels); affects fused_totals_bytes
void fused_set_panel_bytes(long long bytes);
// true when the routing gives this product set to the fused kernels: the reduced set with equal counts <=
// fused_max_slices() (20; not 18, which runs faster as two groups of 9) or different counts <= 18, or all products of
// equal counts with 2 s - 1 <= 18 diagonals
bool fused_handles(int sA, int sB, bool all_products, int m, int n, int k);
// true when it can keep the whole contraction in int32 (min(sA, sB) * k * 127^2 < 2^31)
bool fused_single_block(int sA, int sB, int k);
// bytes of int64 per-tile totals the fused kernel needs when it has to cut k into blocks (else 0)
size_t fused_totals_bytes(int sA, int sB, bool all_products, int m, int n, int k);
// dump != null: write int32 diagonal sums (single block only); totals != null: k-blocked mode.
// Q (all GEMM launchers): diagonals per exactly summed level of the binary64 accumulation, 1 <= Q <= 8.
hipError_t launch_gemm_fused(int m, int n, int kp, int sA, int sB, bool all_products, const int8_t *pA,
                             const int8_t *pB, const int32_t *eA, const int32_t *eB, double *C, int ldc,
                             int32_t *dump, long long *totals, int Q, hipStream_t st);
// the same fused computation on v_mfma_i32_16x16x64_i8, for the slice counts where it is faster (gemm_fused16.hip)
bool fused16_preferred(int s, bool split_k);
void fused16_tile(int s, int &tm, int &tn);
// k-blocks of the 16x16x64 kernel's split-k mode when each gets an int32 slot of its own (2 ... kMaxSplitKSlots), else 0
constexpr int kMaxSplitKSlots = 14;   // (16 slots at 8 slices, 2048 x 2048 x 262144, were 1-2 % behind the totals)
int fused16_split_k_slots(int s, int kp);
// (rounds of the compute units) x (tile area) of a launch with that tile, a measure of its duration; for the
// 16x16x64 kernel with the tile it would choose (4 slices: the cheaper of its two, the alternative's speed counted in)
// (a partly filled last round counts 0.8 of a full one plus 0.2 of its share: the fit over 99 measured pairs of
// launches, sizes 512 ... 6000 and 2 ... 12 slices, picks the faster kernel in all but one, which it misses by 4 %)
inline double launch_cost(int m, int n, int tm, int tn, int cus)
{
    const long long tiles = (long long)((m + tm - 1) / tm) * ((n + tn - 1) / tn);
    const double exact = (double)tiles / cus, whole = (double)((tiles + cus - 1) / cus);
    return (0.8 * whole + 0.2 * exact) * tm * tn;
}
double fused16_launch_cost(int s, int m, int n, int cus);
inline int device_cus()
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return 256;
    return cus;
}
void fused16_set_tile_choice(int choice);   // test knob: 0 automatic, 1 tabulated tile, 2 alternative tile (4 slices)
// (kslots: split-k with an int32 slot per k-block -- fused16_split_k_slots() of them -- instead of int64 totals)
hipError_t launch_gemm_fused16(int m, int n, int kp, int s, const int8_t *pA, const int8_t *pB,
                               const int32_t *eA, const int32_t *eB, double *C, int ldc,
                               int32_t *dump, long long *totals, int Q, bool kslots, hipStream_t st);
// product sets beyond the fused kernels (planes with the slices per entry of blocks_plan); totals: blocks_totals_bytes()
hipError_t launch_gemm_blocks(int m, int n, int kp, int sA, int sB, bool all_products, const int8_t *pA,
                              const int8_t *pB, const int32_t *eA, const int32_t *eB, double *C, int ldc,
                              long long *totals, int Q, hipStream_t st);
// general product band (any sA, sB, any k); totals: scratch of banded_totals_bytes() or null when that is 0
hipError_t launch_gemm_banded(int m, int n, int kp, int sA, int sB, int dmax, const int8_t *pA, const int8_t *pB,
                              const int32_t *eA, const int32_t *eB, double *C, int ldc, long long *totals,
                              int Q, hipStream_t st);
hipError_t launch_gemm_generic(int m, int n, int kp, int s, const int8_t *pA, const int8_t *pB,
                               const int32_t *eA, const int32_t *eB, double *C, int ldc,
                               int pair_l, int pair_h, int kb_begin, int kb_end, int32_t *dump,
                               hipStream_t st);

}  // namespace oz
