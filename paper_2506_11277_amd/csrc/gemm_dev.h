// Device-side helpers shared by the GEMM translation units (HIP only; nothing of the oracle).
#pragma once
#include "oz_common.h"

namespace oz {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// kPlain: whole contraction in int32.  kDump: as kPlain but write the int32 diagonal sums (test hook).
// kBlocked: one work-group per (tile, k-block), diagonal sums added into int64 totals with atomics.
enum FusedMode { kPlain = 0, kDump = 1, kBlocked = 2 };

// XCD-aware tile order.  Work-groups are dealt round-robin to the 8 XCDs (id % 8), each with
// its own L2.  Renumber so that an XCD owns a contiguous run of tiles, and walk the run in
// groups of GM tile-rows so that tiles resident at the same time share A and B panels in L2.
__device__ __forceinline__ void tile_of_block(int b, int nb, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int xcd = b & 7, idx = b >> 3;
    const int q = nb >> 3, rem = nb & 7;
    const int lin = xcd * q + (xcd < rem ? xcd : rem) + idx;
    constexpr int GM = 4;
    const int group = GM * tiles_n;
    const int g = lin / group, in = lin - g * group;
    const int first = g * GM;
    const int gm = tiles_m - first < GM ? tiles_m - first : GM;
    tm = first + in % gm;
    tn = in / gm;
}

// Two-dimensional variant for the fused kernels: the 8 XCDs form a 4 (m) x 2 (n) grid over the tile grid, each
// owning a quarter of the tile rows and half of the tile columns, walked in groups of GM tile rows as above.  At
// any time the XCDs then stream 4 different A panels and 2 different B panels from beyond their L2s instead of 8
// and 1, and an XCD's A panels stay in the memory-side cache while it walks its columns (8192^3, s = 7: +2.7 %).
// The regions can differ in size by a tile row or column, so the grid is padded to 8 x the largest region and
// the surplus work-groups leave at once (tile_of_block_xcd returns false); where that padding would exceed 4 %
// (small or very flat grids) the one-dimensional order above is kept.  Host and device decide by the same rule.
// (Not in split-k mode, where the work-groups of all k-blocks of a tile share its panels anyway: there the 2-D
// order measured 3 % slower at 2048 x 2048 x 262144.)
__host__ __device__ inline bool tile_order_2d(int tiles_m, int tiles_n, bool split_k)
{
    const long long bm = (tiles_m + 3) / 4, bn = (tiles_n + 1) / 2;
    return !split_k && 8 * bm * bn * 100 <= (long long)tiles_m * tiles_n * 104;
}

__host__ __device__ inline long long tile_order_blocks(int tiles_m, int tiles_n, bool split_k)
{
    return tile_order_2d(tiles_m, tiles_n, split_k) ? 8LL * ((tiles_m + 3) / 4) * ((tiles_n + 1) / 2)
                                                    : (long long)tiles_m * tiles_n;
}

__device__ __forceinline__ bool tile_of_block_xcd(int b, int tiles_m, int tiles_n, bool split_k, int &tm, int &tn)
{
    if (!tile_order_2d(tiles_m, tiles_n, split_k)) {
        tile_of_block(b, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
        return true;
    }
    const int x = b & 7, idx = b >> 3;
    const int xm = x & 3, xn = x >> 2;
    const int r0 = (int)((long long)tiles_m * xm / 4), r1 = (int)((long long)tiles_m * (xm + 1) / 4);
    const int c0 = (int)((long long)tiles_n * xn / 2), c1 = (int)((long long)tiles_n * (xn + 1) / 2);
    const int cols = c1 - c0;
    if (idx >= (r1 - r0) * cols) return false;
    constexpr int GM = 4;
    const int group = GM * cols;
    const int g = idx / group, in = idx - g * group;
    const int first = r0 + g * GM;
    const int gm = r1 - first < GM ? r1 - first : GM;
    tm = first + in % gm;
    tn = c0 + in / gm;
    return true;
}

// Window of the planes one launch of the 16x16x64 kernel works on, and where its diagonals go in split-k totals
// (blocks of slice groups: slice counts beyond the accumulator budget are multiplied group by group).  Both planes
// hold `stride` slices per entry; local slice l (0-based) of A is plane slice baseA + dirA * l, of B likewise
// (dir = -1 walks a group backwards, which turns the products l' + h' >= G + 2 of a pair of groups into a reduced
// set); local diagonal a is diagonal abase + adir * a of the na_tot diagonals the totals hold per entry.
struct Window16 {
    int stride, baseA, dirA, baseB, dirB, abase, adir, na_tot;
};
// Several blocks in ONE launch (blockIdx.z picks the window): a block on a column panel is only a couple of rounds of
// tiles, and a launch of its own would pay the ramp-up and the half-empty last round once per block.
constexpr int kMaxWindows16 = 16;
struct WindowList16 {
    Window16 w[kMaxWindows16];
};

// (gemm_fused16.hip) nwin <= kMaxWindows16 blocks in one launch, each: the reduced product set of s in {7, 8, 9}
// slices on a window, k-blocked, int32 diagonal sums added to `totals` (layout of the 128 x 64 tile) with integer
// atomics; and the finishing kernel.
// With `slots` (one k-block only: s * kp within the int32 range) nothing is added: window z stores its s int32
// diagonal sums per entry into a slot of its own, slot z of `totals` read as int32 (a slot: tiles * s * 128 * 64
// values, windows' na_tot = s), nothing has to be cleared, and launch_finish_slots16 adds what belongs to each
// diagonal.  (The atomics of nine blocks cost 14 % of the time of 24 slices at 8192^3, 27 % at 4096^3, 36 % at 2048^3.)
hipError_t launch_fused16_windows(int s, int m, int n, int kp, const int8_t *pA, const int8_t *pB, long long *totals,
                                  const WindowList16 &wins, int nwin, bool slots, hipStream_t st);
hipError_t launch_finish_blocks16(const long long *totals, const int32_t *eA, const int32_t *eB, double *C, int ldc,
                                  int m, int n, int Q, int diagonals, int na_tot, hipStream_t st);
// Which slot values add up to each diagonal: the terms of diagonal d are term[first[d]] ... term[first[d + 1] - 1],
// each (slot index) * 16 + (local diagonal).  Slots 0 ... nf - 1 hold G diagonals per entry (the reduced sets of the
// blocks), the slots from nf on G - 1 (the reversed sets of the whole blocks), one after the other.
constexpr int kMaxSlotDiagonals = 2 * OZIMMU_MAX_SLICES + 8;
struct SlotTerms {
    unsigned short first[kMaxSlotDiagonals + 1];
    unsigned short term[kMaxWindows16 * 9 + kMaxWindows16 * 8];
};
hipError_t launch_finish_slots16(const int32_t *slots, int nf, int G, const SlotTerms &terms, const int32_t *eA,
                                 const int32_t *eB, double *C, int ldc, int m, int n, int Q, int diagonals, hipStream_t st);

// 16 bytes per lane: global (sbase + voff)  ->  LDS (ldsaddr + lane * 16); ldsaddr is wavefront-uniform.
// (global_load_lds: the LDS-DMA form of the vector load, 1 KiB per wavefront instruction; issued
// from inline asm, so the waits on these loads (vmcnt) are placed by hand, and so is the wait state between the
// scalar write of m0 and its use)
__device__ __forceinline__ void lds_dma16(const void *sbase, unsigned voff, unsigned ldsaddr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(ldsaddr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

// The same copy with the LDS address given as wavefront-uniform base + compile-time constant (one scalar add
// straight into m0).
template <int IMM>
__device__ __forceinline__ void lds_dma16_at(const void *sbase, unsigned voff, unsigned ldsbase)
{
    asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3" ::"s"(ldsbase), "n"(IMM), "v"(voff), "s"(sbase)
                 : "memory", "m0", "scc");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

constexpr int kLdsBytes = 160 * 1024;

// Binary64 accumulation of the scaled diagonal sums 2^{-7d} D_d, d ascending, in levels of Q
// consecutive diagonals (subsection "Accumulation in floating-point arithmetic" of Sect. 4): the
// terms of a level are added to each other first, then the level to S.  The host admits only Q for
// which every partial sum of a level is a binary64 number, so the additions inside a level do not
// round and S is rounded once per level.  Q = 1: S <- S + (0 + term), the plain diagonal order.
struct LevelSum {
    double S = 0.0, L = 0.0;
    int cnt = 0;
    __device__ __forceinline__ void add(double term, int Q, bool last)
    {
        L = L + term;
        if (++cnt == Q || last) {
            S = S + L;
            L = 0.0;
            cnt = 0;
        }
    }
};

}  // namespace oz
