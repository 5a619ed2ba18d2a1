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
