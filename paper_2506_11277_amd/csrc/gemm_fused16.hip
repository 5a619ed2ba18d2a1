// Fused slice-product kernel built on v_mfma_i32_16x16x64_i8 (equal slice counts 2 ... 9).
//
// Same computation as gemm_fused_kernel in gemm.hip (all s(s+1)/2 products of Algorithm 1, Sect. 3,
// per-diagonal int32 sums, binary64 accumulation by ascending diagonal), same plane layout, same
// LDS-DMA staging.  The difference is the matrix instruction: on MI355X the 16x16x64 shape sustains
// about 24 % more int8 op/s than 32x32x32 on random operands (the chip is power-limited on real
// data, and the deeper reduction per accumulator update costs less energy per product).  Inside the
// whole kernel the gain is smaller and not uniform: see fused16_preferred() below for where it is used.
//
// A 16x16x64 operand is 16 rows x 64 k: it is assembled from two consecutive 32x32 fragments of the
// plane layout (lane l: row l%16 of the half, k-group l/16 -> fragment (l/16)/2, its lane slot
// row + 32*((l/16)%2)), the same way for A and B, so the k positions of both operands match.
// A stage therefore holds 64 k, which for s >= 7 no longer fits twice into the 160 KiB of LDS.
// For those slice counts the stage is split: the slices l >= L0 of the A tile sit in a
// single-buffered region and are multiplied FIRST; a barrier then frees that region and the next
// stage's copy of it is issued, to land while the remaining products run.  The rest of the stage
// (A slices l < L0, all of B) is double-buffered as before.
//
// Main loop, software-pipelined by hand with a compile-time schedule (Sched16): the matrix instructions of a
// stage are numbered in execution order and every operand is read from LDS a fixed number of them ahead of its
// first use -- the first ones of the NEXT stage behind the end-of-stage barrier, which stands before the products
// of the last slice (all reads of the stage are issued by then), as the mid-stage barrier stands before the
// products of slice L0; the copies of the next stage are issued one at a time behind single matrix instructions,
// two instructions each (source addresses formed once per wavefront, the stage in the 32-bit lane offset, the LDS
// address one scalar add into m0); the loop body has no branch but a ragged last copy.  (A plain loop -- copies
// issued at the top of the stage, operands read where they are used, barriers behind the last product -- left
// the matrix pipe idle 30 % of the cycles at s = 7; this one 15 %, at a clock that the board's power cap lowers
// accordingly.)
//
// The kernel also serves slice counts beyond the accumulator budget: a launch works on a window of planes that hold
// more slices per entry (Window16 in gemm_dev.h; blockIdx.z picks one of up to 16 windows) and adds its int32
// diagonal sums to shared int64 totals at a diagonal offset (launch_fused16_windows; the plan is in gemm.hip,
// launch_gemm_blocks).
#include <type_traits>

#include "gemm_dev.h"

namespace oz {

namespace {

template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// Compile-time schedule of a stage of the 16x16x64 kernel: the matrix instructions are numbered in execution order
// (slices of A from the last to the first, within a slice the slices of B upwards -- downwards for slice 0 --, MPP
// instructions per product); an operand first needed by instruction q is read D instructions ahead.
template <int S, int MPP, int HP, int D, int DO>
struct Sched16 {
    static constexpr int NM = MPP * S * (S + 1) / 2;
    static constexpr int gs(int l) { return MPP * ((S - 1 - l) * (S - l) / 2); }              // first instruction of slice l
    static constexpr int pidx(int l, int h) { return gs(l) + MPP * (l == 0 ? S - 1 - h : h); }  // ... of product (l, h)
    static constexpr int needB(int h) { return pidx(S - 1 - h, h); }                          // first use of B slice h
    static constexpr int slice_of(int e)
    {
        int l = S - 1;
        while (l > 0 && gs(l - 1) <= e) --l;
        return l;
    }
    static constexpr int h_of(int e)
    {
        const int l = slice_of(e), p = (e - gs(l)) / MPP;
        return l == 0 ? S - 1 - p : p;
    }
    // a read needed at instruction q is issued before instruction q - D of the same stage, or, if that lies before
    // the stage, in the stage before: behind its end-of-stage barrier (before instruction EB) at the earliest
    static constexpr bool wrapped(int q) { return q - D < 0; }
    static constexpr int issue_at(int q, int EB) { return q - D >= 0 ? q - D : (NM + q - D > EB ? NM + q - D : EB); }
    static constexpr bool any_read(int e, int EB)
    {
        for (int l = 0; l < S; ++l)
            if (issue_at(gs(l), EB) == e) return true;
        for (int h = 0; h < HP; ++h)
            if (issue_at(needB(h), EB) == e) return true;
        for (int l = 0; l < S; ++l)
            for (int h = HP; h < S - l; ++h)
                if (pidx(l, h) - DO == e) return true;
        return false;
    }
};

// Experiments: -DOZ_EXP_S=<s> overrides the shape tabulated for that slice count with OZ_EXP_WVM/WVN/WMF/WNF
// (wavefront grid and 32 x 32 fragments per wavefront), OZ_EXP_L0, OZ_EXP_D, OZ_EXP_HP.
#ifndef OZ_EXP_S
#define OZ_EXP_S -1
#define OZ_EXP_WVM 4
#define OZ_EXP_WVN 2
#define OZ_EXP_WMF 1
#define OZ_EXP_WNF 1
#endif
#ifndef OZ_EXP_L0
#define OZ_EXP_L0 -1
#endif
#ifndef OZ_EXP_D
#define OZ_EXP_D -1
#endif
#ifndef OZ_EXP_HP
#define OZ_EXP_HP -1
#endif
#ifndef OZ_EXP_NSTG
#define OZ_EXP_NSTG -1
#endif

template <int S, int ALT = 0>
struct Cfg16 {
    static constexpr bool EXP = S == OZ_EXP_S && ALT == 0;
    // s = 2, 3: tile 256 x 128 (4 x 2 wavefronts of 64 x 64: 64 accumulator registers per diagonal; s = 3: 192
    // accumulator registers, so one slice of B held and operands read one instruction ahead, or the loop spills);
    // tile 128 x 128 (2 x 4 wavefronts of 64 x 32) while 32 * S accumulator registers are affordable and the
    // stages fit (s = 5: two 80 KiB stages, all of LDS; s = 6: 192 accumulator registers, B and one slice of A
    // double-buffered, five slices of A single-buffered: 152 KiB), else 128 x 64 (4 x 2 wavefronts of 32 x 32).
    // ALT = 1 (s = 4 only): tile 192 x 128 (2 x 4 wavefronts of 96 x 32, 192 accumulator registers, two 80 KiB
    // stages): 17 % fewer L2 -> LDS bytes and 11 % fewer LDS reads per product than 128 x 128; the launcher takes
    // it where the tile grid of the problem does not lose more in partial rounds than that gains.
    // ALT = 2 (s = 2, 3): tile 128 x 128 with a ring of three stages, for problems of a few thousand rows and
    // columns whose 256 x 128 tiles would leave most of a round of the compute units empty.
    // ALT = 3 (s = 5, 6): tile 128 x 64, whole stage double-buffered, for the same purpose.
    static_assert(ALT == 0 || (ALT == 1 && S == 4) || (ALT == 2 && (S == 2 || S == 3)) || (ALT == 3 && (S == 5 || S == 6)),
                  "no such alternative tile");
    static constexpr bool HUGE = (S == 2 || S == 3) && ALT != 2, WIDE = ((S >= 4 && S <= 6) || ALT == 2) && ALT != 3;
    static constexpr int WVM = EXP ? OZ_EXP_WVM : WIDE ? 2 : 4, WVN = EXP ? OZ_EXP_WVN : WIDE ? 4 : 2;
    static constexpr int WMF = EXP ? OZ_EXP_WMF : ALT == 1 ? 3 : (WIDE || HUGE) ? 2 : 1, WNF = EXP ? OZ_EXP_WNF : HUGE ? 2 : 1;
    static constexpr int FA = WVM * WMF, FB = WVN * WNF;          // 32-row fragment rows of the tile
    // A slices [0, L0) are double-buffered with B; A slices [L0, S) single-buffered (L0 == S: no split)
    // (from a sweep at 8192^3: s = 7 runs 2820 / 2960 / 2905 / 2840 / 2795 TOP/s for L0 = 2 / 3 / 4 / 5 / 6, s = 8
    // 2985 / 3150 / 3120 for L0 = 2 / 3 / 4 -- and 3230 against 3110 with split-k --, s = 9 2925 / 3100 for L0 = 1 / 2;
    // s = 6 on the 128 x 128 tile: L0 = 1 with two slices of B held 3055-3065, L0 = 2 spills, against 2905 for the
    // 128 x 64 tile without split, same box)
    static constexpr int L0 = EXP && OZ_EXP_L0 >= 0 ? OZ_EXP_L0 : (S <= 5 || ALT == 3) ? S : S == 6 ? 1 : S <= 8 ? 3 : 2;
    static constexpr int P1 = (FA * L0 + FB * S) * 2 * kFragBytes;    // double-buffered part of a 64-k stage
    static constexpr int P2 = FA * (S - L0) * 2 * kFragBytes;         // single-buffered part
    // ring depth of the double-buffered part.  Few slices make a stage short (s = 2: 48 matrix instructions per
    // wavefront): a copy issued one stage ahead would have to land within a few hundred cycles, less than the
    // latency of the L2.  With a ring of three the copies of stage st + 2 are issued while stage st is multiplied
    // and only those of stage st + 1 are waited for.
    // Measured at 8192^3: s = 2 (tile 256 x 128) 2150 -> 2370 TOP/s, s = 3 (tile 128 x 128) 2500 -> 2640 against the
    // 32x32x32 kernel with its ring of three; with a ring of two the same tiles gain nothing (matrix pipe busy half
    // of the cycles).  From 4 slices on three stages of a 128 x 128 tile do not fit.
    // s = 3 on the 256 x 128 tile has stages as long as those of s = 7 (96 matrix instructions per wavefront) and
    // runs with two: 2800 against 2670 TOP/s for the 128 x 128 tile with its ring of three, same box.
    static constexpr int NSTG = EXP && OZ_EXP_NSTG >= 0 ? OZ_EXP_NSTG : (S == 2 || ALT == 2) ? 3 : 2;
    static_assert(NSTG == 2 || (NSTG == 3 && L0 == S), "a ring of three only without the split stage");
    static constexpr int LDS = NSTG * P1 + P2;
    static_assert(LDS <= kLdsBytes, "stages do not fit LDS");
    // operands are read D matrix instructions ahead of their first use (DO: the B slices that are not held in
    // registers, ahead of each use).  Measured at s = 7, 8192^3: 3250 / 3200 / 3310 / 3140 / 3240 / 3205 TOP/s for
    // D = 4 / 6 / 8 / 10 / 12 / 16 (reads one slice ahead, the earlier scheme: 3215); s = 4 is indifferent up to 24.
    // (s = 3 on 256 x 128 and s = 4 on 192 x 128 spill with any longer read-ahead: 2190 against 2800 TOP/s at s = 3)
    static constexpr int D = EXP && OZ_EXP_D >= 0 ? OZ_EXP_D : ((S == 3 && ALT == 0) || ALT == 1) ? 1 : S == 4 ? 24 : 8, DO = 4;
    // slices of B held in registers for the whole stage (the others are read when needed)
    static constexpr int HP = EXP && OZ_EXP_HP >= 0 ? OZ_EXP_HP : S >= 9 ? 7 : ((S == 6 && ALT == 0) || ALT == 1) ? 2 : (S == 3 && ALT == 0) ? 1 : S;
};

template <int S, int MODE, int ALT = 0>
__global__ __launch_bounds__((64 * Cfg16<S, ALT>::WVM * Cfg16<S, ALT>::WVN)) void gemm_fused16_kernel(
    const int8_t *__restrict__ pA, const int8_t *__restrict__ pB, const int32_t *__restrict__ eA,
    const int32_t *__restrict__ eB, double *__restrict__ C, int ldc, int m, int n, int KB, int tiles_m, int tiles_n,
    int32_t *__restrict__ dump, long long *__restrict__ totals, int stages_per_block, int Q, long long slot_stride,
    WindowList16 wins)
{
    using G = Cfg16<S, ALT>;
    const Window16 win = wins.w[blockIdx.z];
    constexpr int WVM = G::WVM, WVN = G::WVN, WMF = G::WMF, WNF = G::WNF, FA = G::FA, FB = G::FB, L0 = G::L0;
    constexpr int NW = WVM * WVN;
    constexpr bool SPLIT = L0 < S;
    constexpr int NS2 = SPLIT ? S - L0 : 1;                         // slices in the single-buffered region
    constexpr bool DUMP = MODE == kDump;
    // 1 KiB copy units of a stage.  P1: A rows c < FA, slices l < L0, k-halves kk < 2, then B rows, all slices,
    // kk.  P2: A rows, slices l >= L0, kk.  The two k-halves of a (row, slice) are neighbours in LDS, so one
    // per-lane offset serves all three regions.
    constexpr int U1A = FA * 2 * L0, U1 = U1A + FB * 2 * S, U2 = FA * 2 * (S - L0);
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
    constexpr int Z = G::NSTG * G::P1;                                   // offset of the single-buffered region

    int tm, tn;
    if (!tile_of_block_xcd(blockIdx.x, tiles_m, tiles_n, MODE == kBlocked, tm, tn)) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % WVM, wn = wave / WVM;
    const size_t row_bytes = (size_t)KB * ((size_t)win.stride * kFragBytes);
    // fragment rows of the planes (padded to kPad entries): a tile taller or wider than the padding may reach
    // beyond them at the edge; such rows are read from the last valid fragment row instead (their outputs lie
    // beyond m resp. n and are never stored)
    const int frA = (m + kPad - 1) / kPad * (kPad / kFrag), frB = (n + kPad - 1) / kPad * (kPad / kFrag);
    auto rowA_of = [&](int c) { const int r = tm * FA + c; return pA + (size_t)(r < frA ? r : frA - 1) * row_bytes; };
    auto rowB_of = [&](int c) { const int r = tn * FB + c; return pB + (size_t)(r < frB ? r : frB - 1) * row_bytes; };

    // accumulators: per diagonal a and 32x32 fragment (i, j) four 16x16 blocks (i2, j2)
    v4i acc[S][WMF][WNF][4];
#pragma unroll
    for (int a = 0; a < S; ++a)
#pragma unroll
        for (int i = 0; i < WMF; ++i)
#pragma unroll
            for (int j = 0; j < WNF; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][i][j][b] = v4i{0, 0, 0, 0};

    const int nst_all = KB / 2;
    const int st0 = MODE == kBlocked ? (int)blockIdx.y * stages_per_block : 0;
    const int nst = MODE == kBlocked && st0 + stages_per_block < nst_all ? st0 + stages_per_block : nst_all;

    // Copy units of this wavefront: unit u = wave + i * NW of a region, its source address for the first stage of
    // this work-group formed once here (a stage advances every source by STG bytes, which the copies carry in their
    // 32-bit lane offset: a k-block is a few MiB of a fragment row at most, whatever k).
    constexpr int NU1 = (U1 + NW - 1) / NW, NU2 = SPLIT ? (U2 + NW - 1) / NW : 0;
    const size_t STG = (size_t)2 * win.stride * kFragBytes;      // bytes of a 64-k stage in a fragment row of the planes
    const int8_t *src1[NU1], *src2[NU2 ? NU2 : 1];
#pragma unroll
    for (int i = 0; i < NU1; ++i) {
        const int u = wave + i * NW;
        if (u < U1A) {
            const int c = u / (2 * L0), l = (u / 2) % L0, kk = u % 2;
            src1[i] = rowA_of(c) + (size_t)st0 * STG + (size_t)(kk * win.stride + win.baseA + win.dirA * l) * kFragBytes;
        } else {
            const int v = u - U1A;
            const int c = v / (2 * S), h = (v / 2) % S, kk = v % 2;
            src1[i] = rowB_of(c) + (size_t)st0 * STG + (size_t)(kk * win.stride + win.baseB + win.dirB * h) * kFragBytes;
        }
    }
#pragma unroll
    for (int i = 0; i < NU2; ++i) {
        const int u = wave + i * NW;
        const int c = u / (2 * NS2), l = L0 + (u / 2) % NS2, kk = u % 2;
        src2[i] = rowA_of(c) + (size_t)st0 * STG + (size_t)(kk * win.stride + win.baseA + win.dirA * l) * kFragBytes;
    }
    // Unit I of the double-buffered part (issue1) / of the single-buffered part (issue2): `voff` carries the stage
    // (lane * 16 + (stage - first stage) * STG), `ldsbuf` the ring buffer and the wavefront.  Two instructions per
    // copy.
    const unsigned ldsw = lds0 + wave * kFragBytes;
    auto issue1 = [&](auto I, unsigned voff, unsigned ldsbuf) {
        constexpr int i = decltype(I)::value;
        if (i < U1 / NW || wave < U1 % NW) lds_dma16_at<i * NW * kFragBytes>(src1[i], voff, ldsbuf);
    };
    auto issue2 = [&](auto I, unsigned voff) {
        constexpr int i = decltype(I)::value;
        if (i < U2 / NW || wave < U2 % NW) lds_dma16_at<Z + i * NW * kFragBytes>(src2[i], voff, ldsw);
    };
    // (compile-time dispatch on the unit number)
    auto issue1_n = [&](int i, unsigned voff, unsigned ldsbuf) {
        switch (i) {
#define OZ_U(N_) case N_: if constexpr (N_ < NU1) issue1(std::integral_constant<int, N_>{}, voff, ldsbuf); break;
            OZ_U(0) OZ_U(1) OZ_U(2) OZ_U(3) OZ_U(4) OZ_U(5) OZ_U(6) OZ_U(7) OZ_U(8) OZ_U(9) OZ_U(10) OZ_U(11)
            OZ_U(12) OZ_U(13) OZ_U(14) OZ_U(15) OZ_U(16) OZ_U(17) OZ_U(18) OZ_U(19) OZ_U(20) OZ_U(21) OZ_U(22) OZ_U(23)
#undef OZ_U
        }
    };
    auto issue2_n = [&](int i, unsigned voff) {
        switch (i) {
#define OZ_U(N_) case N_: if constexpr (N_ < NU2) issue2(std::integral_constant<int, N_>{}, voff); break;
            OZ_U(0) OZ_U(1) OZ_U(2) OZ_U(3) OZ_U(4) OZ_U(5) OZ_U(6) OZ_U(7) OZ_U(8) OZ_U(9) OZ_U(10) OZ_U(11)
            OZ_U(12) OZ_U(13) OZ_U(14) OZ_U(15) OZ_U(16) OZ_U(17) OZ_U(18) OZ_U(19) OZ_U(20) OZ_U(21) OZ_U(22) OZ_U(23)
#undef OZ_U
        }
    };
    static_assert(NU1 <= 24 && NU2 <= 24, "unit dispatch");

    constexpr int NSTG = G::NSTG;
    // (ring of three: every wavefront issues the same number of copies per stage, so that "all but the copies of
    // the last stage issued" is one compile-time count)
    static_assert(NSTG == 2 || U1 % NW == 0, "ring of three: copies must divide evenly among the wavefronts");
    {
        const unsigned v0 = lane * 16;
#pragma unroll
        for (int i = 0; i < NU1; ++i) issue1_n(i, v0, ldsw);
#pragma unroll
        for (int i = 0; i < NU2; ++i) issue2_n(i, v0);
        if constexpr (NSTG == 3) {
            // second stage of the work-group (the first one again if there is no other: nobody reads it)
            const unsigned v1 = v0 + (st0 + 1 < nst ? (unsigned)STG : 0u);
#pragma unroll
            for (int i = 0; i < NU1; ++i) issue1_n(i, v1, ldsw + G::P1);
        }
        if constexpr (NSTG == 3) wait_vmcnt<NU1>(); else wait_vmcnt<0>();
    }
    __syncthreads();

    // this lane's part of a 16x64 operand: row lane%16 of the half, k-group g = lane/16
    // -> fragment kk = g / 2 of the pair, lane slot (row + 32 * (g % 2)) in it
    const int lofs = ((lane >> 4) >> 1) * kFragBytes + ((lane & 15) + 32 * ((lane >> 4) & 1)) * 16;
    auto readA = [&](int l, const unsigned char *stage, int i, int i2) -> v4i {
        return l >= L0 ? *(const v4i *)(lds + Z + (((wm * WMF + i) * NS2 + (l - L0)) * 2) * kFragBytes + lofs + i2 * 256)
                       : *(const v4i *)(stage + (((wm * WMF + i) * L0 + l) * 2) * kFragBytes + lofs + i2 * 256);
    };
    auto readB = [&](int h, const unsigned char *stage, int j, int j2) -> v4i {
        return *(const v4i *)(stage + (U1A + ((wn * WNF + j) * S + h) * 2) * kFragBytes + lofs + j2 * 256);
    };

    // Schedule of a stage.  The slices of A go from the last to the first (the single-buffered ones, l >= L0,
    // first); within a slice the slices of B go upwards, for slice 0 downwards.  Every operand is read G::D matrix
    // instructions ahead of its first use.  Before the products of slice L0 nobody needs the single-buffered region
    // any more (mid-stage barrier); before the products of slice 0 -- after the B slices that are read on demand,
    // s = 9: only HP slices of B are held in registers -- every read of the stage is issued: the end-of-stage
    // barrier stands there, and the operands of the first instructions of the NEXT stage are read behind it.  The
    // copies of the next stage go one at a time behind single matrix instructions (double-buffered part from the
    // start of the stage, the single-buffered part from the mid-stage barrier on).
    constexpr int HP = G::HP;
    constexpr int NSLOT = S * (S - 1) / 2;                                  // products of the slices l > 0
    constexpr int NPRE = SPLIT ? (S - L0 - 1) * (S - L0) / 2 : NSLOT;        // ... of them before the mid-stage barrier
    constexpr int MPP = 4 * WMF * WNF;                                       // matrix instructions per product
    static_assert(NU1 <= NPRE * MPP && (!SPLIT || NU2 <= (NSLOT - NPRE) * MPP), "too few products to issue the copies behind");
    static_assert(NSTG == 2 || NU1 <= MPP * NSLOT, "ring of three: the copies of a stage are issued before its end-of-stage barrier");
    using T = Sched16<S, MPP, HP, G::D, G::DO>;
    // (a B slice that is not held is first needed in slice S - 1 - HP or later: its read-ahead stays inside the stage)
    static_assert(HP == S || T::pidx(S - 1 - HP, HP) >= G::DO, "on-demand reads must not precede the stage");
    constexpr int NM = T::NM;                           // matrix instructions of a stage, numbered in execution order
    constexpr int EB = MPP * (NSLOT + (S - HP));        // the end-of-stage barrier stands before this one
    constexpr int MB = MPP * NPRE;                      // the mid-stage barrier before this one

    v4i A_[S][WMF][2], B_[HP][WNF][2], An_[S][WMF][2], Bn_[HP][WNF][2], Bo[S][S - HP + 1][WNF][2];
    auto loadA = [&](v4i (&dst)[WMF][2], int l, const unsigned char *stage) {
#pragma unroll
        for (int i = 0; i < WMF; ++i)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) dst[i][i2] = readA(l, stage, i, i2);
    };
    auto loadB = [&](v4i (&dst)[WNF][2], int h, const unsigned char *stage) {
#pragma unroll
        for (int j = 0; j < WNF; ++j)
#pragma unroll
            for (int j2 = 0; j2 < 2; ++j2) dst[j][j2] = readB(h, stage, j, j2);
    };
    // the wrapped reads of the first stage
    static_for<0, S>([&](auto L) {
        constexpr int l = decltype(L)::value;
        if constexpr (T::wrapped(T::gs(l))) loadA(A_[l], l, lds);
    });
    static_for<0, HP>([&](auto H) {
        constexpr int h = decltype(H)::value;
        if constexpr (T::wrapped(T::needB(h))) loadB(B_[h], h, lds);
    });

    int buf = 0;
    for (int st = st0; st < nst; ++st) {
        // (in the last stage the copies and the reads ahead go on, of that stage again: nobody uses them, and
        // the loop stays free of branches)
        const int ahead = st + NSTG - 1 < nst ? st + NSTG - 1 : nst - 1;
        const unsigned vnext = lane * 16 + (unsigned)(ahead - st0) * (unsigned)STG;
        const int buf1 = buf + 1 == NSTG ? 0 : buf + 1;                       // holds stage st + 1
        const int bufc = NSTG == 2 ? buf1 : (buf1 + 1 == NSTG ? 0 : buf1 + 1);   // receives stage st + NSTG - 1
        const unsigned ldsnext = ldsw + bufc * G::P1;
        const unsigned char *cur = lds + buf * G::P1, *nxt = lds + buf1 * G::P1;
        static_for<0, NM>([&](auto E) {
            constexpr int e = decltype(E)::value;
            constexpr int l = T::slice_of(e), h = T::h_of(e), inner = e % MPP;
            constexpr int j2 = inner % 2, i2 = (inner / 2) % 2, j = (inner / 4) % WNF, i = inner / 4 / WNF;
            constexpr bool pin = T::any_read(e, EB) || e == EB || (SPLIT && e == MB);
            if constexpr (pin) __builtin_amdgcn_sched_barrier(0);
            // reads of this stage due before instruction e
            if constexpr (T::any_read(e, EB)) {
                static_for<0, S>([&](auto L2) {
                    constexpr int l2 = decltype(L2)::value;
                    if constexpr (!T::wrapped(T::gs(l2)) && T::issue_at(T::gs(l2), EB) == e) loadA(A_[l2], l2, cur);
                });
                static_for<0, HP>([&](auto H2) {
                    constexpr int h2 = decltype(H2)::value;
                    if constexpr (!T::wrapped(T::needB(h2)) && T::issue_at(T::needB(h2), EB) == e) loadB(B_[h2], h2, cur);
                });
                static_for<0, S>([&](auto L2) {
                    constexpr int l2 = decltype(L2)::value;
                    static_for<HP, S>([&](auto H2) {
                        constexpr int h2 = decltype(H2)::value;
                        if constexpr (h2 < S - l2 && T::pidx(l2, h2) - G::DO == e) loadB(Bo[l2][h2 - HP], h2, cur);
                    });
                });
            }
            if constexpr (SPLIT && e == MB) __syncthreads();      // nobody reads the single-buffered region any more
            if constexpr (e == EB) {
                // nothing of this stage is left to read, and the next one must have landed (ring of three: the
                // copies issued during this stage, of the stage after the next, may stay in flight)
                if constexpr (NSTG == 3) wait_vmcnt<NU1>(); else wait_vmcnt<0>();
                __syncthreads();
            }
            // reads for the first instructions of the next stage
            if constexpr (T::any_read(e, EB)) {
                static_for<0, S>([&](auto L2) {
                    constexpr int l2 = decltype(L2)::value;
                    if constexpr (T::wrapped(T::gs(l2)) && T::issue_at(T::gs(l2), EB) == e) loadA(An_[l2], l2, nxt);
                });
                static_for<0, HP>([&](auto H2) {
                    constexpr int h2 = decltype(H2)::value;
                    if constexpr (T::wrapped(T::needB(h2)) && T::issue_at(T::needB(h2), EB) == e) loadB(Bn_[h2], h2, nxt);
                });
            }
            if constexpr (pin) __builtin_amdgcn_sched_barrier(0);

            const v4i bv = h < HP ? B_[h < HP ? h : 0][j][j2] : Bo[l][h >= HP ? h - HP : 0][j][j2];
            acc[l + h][i][j][i2 * 2 + j2] =
                __builtin_amdgcn_mfma_i32_16x16x64_i8(bv, A_[l][i][i2], acc[l + h][i][j][i2 * 2 + j2], 0, 0, 0);
            // one copy of the next stage behind each of the first matrix instructions of the stage
            // (double-buffered part) / after the mid-stage barrier (the rest)
            if constexpr (e < NU1) issue1(std::integral_constant<int, (e < NU1 ? e : 0)>{}, vnext, ldsnext);
            if constexpr (SPLIT && e >= MB && e - MB < NU2)
                issue2(std::integral_constant<int, (e >= MB && e - MB < NU2 ? e - MB : 0)>{}, vnext);
        });
        static_for<0, S>([&](auto L) {
            constexpr int l = decltype(L)::value;
            if constexpr (T::wrapped(T::gs(l))) {
#pragma unroll
                for (int i = 0; i < WMF; ++i)
#pragma unroll
                    for (int i2 = 0; i2 < 2; ++i2) A_[l][i][i2] = An_[l][i][i2];
            }
        });
        static_for<0, HP>([&](auto H) {
            constexpr int h = decltype(H)::value;
            if constexpr (T::wrapped(T::needB(h))) {
#pragma unroll
                for (int j = 0; j < WNF; ++j)
#pragma unroll
                    for (int j2 = 0; j2 < 2; ++j2) B_[h][j][j2] = Bn_[h][j][j2];
            }
        });
        buf = buf1;
    }

    // element of accumulator block (i2, j2), register r: m_local = 16*i2 + lane%16, n_local = 16*j2 + 4*(lane/16) + r
    const int m0 = (tm * FA + wm * WMF) * 32, n0 = (tn * FB + wn * WNF) * 32;
    if (MODE == kBlocked) {
        const size_t e0 = ((size_t)(tm * tiles_n + tn) * NW + wave) * (size_t)(win.na_tot * WMF * WNF * 16 * 64) + lane;
        if (slot_stride) {
            // exactly two k-blocks: plain int32 stores into this block's slot, nothing cleared, nothing added
            // (blocks of slice groups with a slot per window: blockIdx.z picks the slot)
            int *slot = (int *)totals + (size_t)(blockIdx.y + gridDim.y * blockIdx.z) * (size_t)slot_stride + e0;
#pragma unroll
            for (int a = 0; a < S; ++a) {
                int *sa = slot + (size_t)a * (WMF * WNF * 16 * 64);
                asm volatile("" : "+v"(sa));
#pragma unroll
                for (int i = 0; i < WMF; ++i)
#pragma unroll
                    for (int j = 0; j < WNF; ++j)
#pragma unroll
                        for (int b = 0; b < 4; ++b)
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                sa[(((size_t)i * WNF + j) * 16 + b * 4 + r) * 64] = acc[a][i][j][b][r];
                asm volatile("" ::: "memory");
            }
            return;
        }
        long long *tot = totals + e0;
#pragma unroll
        for (int a = 0; a < S; ++a)
#pragma unroll
            for (int i = 0; i < WMF; ++i)
#pragma unroll
                for (int j = 0; j < WNF; ++j)
#pragma unroll
                    for (int b = 0; b < 4; ++b)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            __hip_atomic_fetch_add(tot + ((((size_t)(win.abase + win.adir * a) * WMF + i) * WNF + j) * 16 + b * 4 + r) * 64,
                                                   (long long)acc[a][i][j][b][r], __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
#pragma unroll
    for (int i = 0; i < WMF; ++i)
#pragma unroll
        for (int i2 = 0; i2 < 2; ++i2) {
            const int mi = m0 + i * 32 + i2 * 16 + (lane & 15);
            if (mi >= m) continue;
            const int ea = DUMP ? 0 : eA[mi];
#pragma unroll
            for (int j = 0; j < WNF; ++j)
#pragma unroll
                for (int j2 = 0; j2 < 2; ++j2)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int nj = n0 + j * 32 + j2 * 16 + 4 * (lane >> 4) + r;
                        if (nj >= n) continue;
                        if (DUMP) {
#pragma unroll
                            for (int a = 0; a < S; ++a)
                                dump[(size_t)a * m * n + mi + (size_t)nj * m] = acc[a][i][j][i2 * 2 + j2][r];
                        } else {
                            LevelSum sum;
#pragma unroll
                            for (int a = 0; a < S; ++a)
                                sum.add((double)acc[a][i][j][i2 * 2 + j2][r] * __builtin_ldexp(1.0, -kSliceBits * (a + 2)),
                                        Q, a == S - 1);
                            // (streaming store: C is not read again here, and keeping its 8 m n bytes out of the caches
                            // leaves the reduction of the next call 8 % faster -- 0.202 -> 0.185 ms at 8192^3)
                            __builtin_nontemporal_store(ldexp(sum.S, ea + eB[nj]), &C[mi + (size_t)nj * ldc]);
                        }
                    }
        }
}

// Second step of the k-blocked mode: binary64 accumulation from the int64 totals, same element
// mapping and order of additions as the epilogue above.
template <int S>
__global__ __launch_bounds__(64 * Cfg16<S>::WVM * Cfg16<S>::WVN) void finish_blocked16_kernel(
    const long long *__restrict__ totals, const int32_t *__restrict__ eA, const int32_t *__restrict__ eB,
    double *__restrict__ C, int ldc, int m, int n, int tiles_n, int Q, long long slot_stride, int nslot)
{
    using G = Cfg16<S>;
    constexpr int WVM = G::WVM, WVN = G::WVN, WMF = G::WMF, WNF = G::WNF, FA = G::FA, FB = G::FB, NW = WVM * WVN;
    const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WVM, wn = wave / WVM;
    const size_t e0 = ((size_t)blockIdx.x * NW + wave) * (size_t)(S * WMF * WNF * 16 * 64) + lane;
    const long long *tot = totals + e0;
    const int *slot = (const int *)totals + e0;      // slot_stride != 0: nslot int32 slots (one per k-block) instead of int64 totals
    const int m0 = (tm * FA + wm * WMF) * 32, n0 = (tn * FB + wn * WNF) * 32;
    // blockIdx.y picks one 16 x 16 block of the wavefront's fragments (i, j, i2, j2): WMF * WNF * 4 times the wavefronts
    // of the tile grid, and the four entries of a lane (registers r) go together, so that the loads are independent
    const int blk = blockIdx.y, f = blk >> 2, i = f / WNF, j = f % WNF, i2 = (blk >> 1) & 1, j2 = blk & 1;
    LevelSum sum[4];
#pragma unroll
    for (int a = 0; a < S; ++a) {
        const size_t e = ((((size_t)a * WMF + i) * WNF + j) * 16 + (i2 * 2 + j2) * 4) * 64;
        long long v[4] = {0, 0, 0, 0};
        if (slot_stride) {
            for (int y = 0; y < nslot; ++y) {
                const int *p = slot + (size_t)y * (size_t)slot_stride + e;
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] += p[r * 64];
            }
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = tot[e + r * 64];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
            sum[r].add((double)v[r] * __builtin_ldexp(1.0, -kSliceBits * (a + 2)), Q, a == S - 1);   // exact conversion
    }
    const int mi = m0 + i * 32 + i2 * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int nj = n0 + j * 32 + j2 * 16 + 4 * (lane >> 4) + r;
        if (mi < m && nj < n) C[mi + (size_t)nj * ldc] = ldexp(sum[r].S, eA[mi] + eB[nj]);
    }
}

// Binary64 accumulation after the block launches of launch_gemm_blocks: the totals hold na_tot diagonals per entry in
// the layout of the 128 x 64 tile (4 x 2 wavefronts), the first `diagonals` of them are added in ascending order.
__global__ __launch_bounds__(512) void finish_blocks16_kernel(const long long *__restrict__ totals,
                                                              const int32_t *__restrict__ eA,
                                                              const int32_t *__restrict__ eB, double *__restrict__ C,
                                                              int ldc, int m, int n, int tiles_n, int Q, int diagonals,
                                                              int na_tot)
{
    constexpr int WVM = 4, NW = 8;
    const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WVM, wn = wave / WVM;
    const long long *tot = totals + ((size_t)blockIdx.x * NW + wave) * (size_t)(na_tot * 16 * 64) + lane;
    const int m0 = (tm * 4 + wm) * 32, n0 = (tn * 2 + wn) * 32;
    // blockIdx.y picks one of the lane's four 16 x 16 blocks (i2, j2): four times the wavefronts of the tile grid
    const int blk = blockIdx.y, i2 = blk >> 1, j2 = blk & 1;
    LevelSum sum[4];
    for (int a = 0; a < diagonals; ++a) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const long long v = tot[((size_t)a * 16 + blk * 4 + r) * 64];
            sum[r].add(ldexp((double)v, -kSliceBits * (a + 2)), Q, a == diagonals - 1);      // exact: |v| < 2^53
        }
    }
    const int mi = m0 + i2 * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int nj = n0 + j2 * 16 + 4 * (lane >> 4) + r;
        if (mi < m && nj < n) C[mi + (size_t)nj * ldc] = ldexp(sum[r].S, eA[mi] + eB[nj]);
    }
}

// The same after block launches that stored a slot per window (launch_fused16_windows with `slots`): the int32 values
// that belong to a diagonal are added exactly in int64, the diagonals then in ascending order as everywhere.
__global__ __launch_bounds__(512) void finish_slots16_kernel(const int32_t *__restrict__ slots, int nf, int G,
                                                             long long stride_f, long long stride_r, SlotTerms terms,
                                                             const int32_t *__restrict__ eA,
                                                             const int32_t *__restrict__ eB, double *__restrict__ C,
                                                             int ldc, int m, int n, int tiles_n, int Q, int diagonals)
{
    constexpr int WVM = 4, NW = 8;
    const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WVM, wn = wave / WVM;
    const int32_t *base_f = slots + ((size_t)blockIdx.x * NW + wave) * (size_t)(G * 16 * 64) + lane;
    const int32_t *base_r = slots + (size_t)nf * (size_t)stride_f + ((size_t)blockIdx.x * NW + wave) * (size_t)((G - 1) * 16 * 64) + lane;
    const int m0 = (tm * 4 + wm) * 32, n0 = (tn * 2 + wn) * 32;
    // blockIdx.y picks one of the lane's four 16 x 16 blocks (i2, j2); its four entries (registers r: value
    // el = (i2 * 2 + j2) * 4 + r of a local diagonal) go together, so that the loads of a term are independent, and the
    // launch has four times the wavefronts of the GEMM's tile grid to hide their latency
    const int blk = blockIdx.y, i2 = blk >> 1, j2 = blk & 1;
    LevelSum sum[4];
    for (int d = 0; d < diagonals; ++d) {
        long long v[4] = {0, 0, 0, 0};
        for (int t = terms.first[d]; t < terms.first[d + 1]; ++t) {
            const int q = terms.term[t] >> 4, a = terms.term[t] & 15;
            const int32_t *p = (q < nf ? base_f + (size_t)q * (size_t)stride_f : base_r + (size_t)(q - nf) * (size_t)stride_r) +
                               a * (16 * 64) + blk * (4 * 64);
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] += p[r * 64];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
            sum[r].add(ldexp((double)v[r], -kSliceBits * (d + 2)), Q, d == diagonals - 1);      // exact: |v| < 2^53
    }
    const int mi = m0 + i2 * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int nj = n0 + j2 * 16 + 4 * (lane >> 4) + r;
        if (mi < m && nj < n) C[mi + (size_t)nj * ldc] = ldexp(sum[r].S, eA[mi] + eB[nj]);
    }
}

__global__ void zero16_i64_kernel(long long *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

template <int S, int MODE, int ALT = 0>
hipError_t launch16_s(int m, int n, int kp, const int8_t *pA, const int8_t *pB, const int32_t *eA, const int32_t *eB,
                      double *C, int ldc, int32_t *dump, long long *totals, int Q, bool kslots, hipStream_t st)
{
    using G = Cfg16<S, ALT>;
    static_assert(ALT == 0 || MODE != kBlocked, "split-k keeps the tabulated tile: the totals are laid out for it");
    constexpr int TM = 32 * G::FA, TN = 32 * G::FB, THREADS = 64 * G::WVM * G::WVN;
    auto kern = gemm_fused16_kernel<S, MODE, ALT>;
    static std::atomic<unsigned long long> configured{0};
    if (hipError_t e = allow_dynamic_lds((const void *)kern, G::LDS, configured); e != hipSuccess) return e;
    const int tiles_m = (m + TM - 1) / TM, tiles_n = (n + TN - 1) / TN;
    const int KB = kp / kFrag;
    note_gemm_kernel("gemm_fused16_kernel<%d> tile %dx%d%s%s", S, TM, TN, G::NSTG == 3 ? " ring of 3" : "",
                     MODE == kBlocked ? " split-k" : "");
    if (MODE != kBlocked) {
        kern<<<(unsigned)tile_order_blocks(tiles_m, tiles_n, false), THREADS, G::LDS, st>>>(pA, pB, eA, eB, C, ldc, m, n, KB, tiles_m, tiles_n, dump,
                                                         nullptr, 0, Q, 0, WindowList16{{Window16{S, 0, 1, 0, 1, 0, 1, S}}});
        return hipGetLastError();
    }
    // longest k-block (in 64-k stages) whose s products per diagonal cannot overflow int32; equally long blocks
    const int max_stages = (int)(kMaxInt32K / S / (2 * kFrag));
    const int nst = KB / 2;
    const int nblocks = (nst + max_stages - 1) / max_stages;
    const int stages_per_block = (nst + nblocks - 1) / nblocks;
    // two k-blocks, or up to kMaxSplitKSlots where the caller has the buffer for it (`kslots`): an int32 slot per block,
    // nothing to clear and no atomics (which cost 4-9 % of the launch at 2048 x 2048 x 65536 ... 262144); else int64
    // totals shared through atomics
    const size_t nslots = (size_t)tiles_m * tiles_n * S * TM * TN;
    const long long slot_stride = nblocks == 2 || (kslots && fused16_split_k_slots(S, kp)) ? (long long)nslots : 0;
    if (!slot_stride) zero16_i64_kernel<<<2048, 256, 0, st>>>(totals, nslots);
    dim3 grid((unsigned)tile_order_blocks(tiles_m, tiles_n, true), nblocks);
    kern<<<grid, THREADS, G::LDS, st>>>(pA, pB, eA, eB, C, ldc, m, n, KB, tiles_m, tiles_n, nullptr, totals,
                                        stages_per_block, Q, slot_stride, WindowList16{{Window16{S, 0, 1, 0, 1, 0, 1, S}}});
    finish_blocked16_kernel<S><<<dim3(tiles_m * tiles_n, G::WMF * G::WNF * 4), THREADS, 0, st>>>(totals, eA, eB, C, ldc, m, n, tiles_n, Q, slot_stride, nblocks);
    return hipGetLastError();
}

// Blocks of slice groups: for each of the nwin windows the reduced product set of S slices on that window of the
// planes, k-blocked, its int32 diagonal sums added to the totals with integer atomics (nothing cleared, nothing
// finished here).
template <int S, int ALT = 0>
hipError_t launch16_windows(int m, int n, int kp, const int8_t *pA, const int8_t *pB, long long *totals,
                            const WindowList16 &wins, int nwin, bool slots, hipStream_t st)
{
    using G = Cfg16<S, ALT>;
    constexpr int TM = 32 * G::FA, TN = 32 * G::FB, THREADS = 64 * G::WVM * G::WVN;
    static_assert(TM == 128 && TN == 64 && G::WVM == 4 && G::WVN == 2, "blocks share the totals layout of the 128 x 64 tile");
    auto kern = gemm_fused16_kernel<S, kBlocked, ALT>;
    static std::atomic<unsigned long long> configured{0};
    if (hipError_t e = allow_dynamic_lds((const void *)kern, G::LDS, configured); e != hipSuccess) return e;
    const int tiles_m = (m + TM - 1) / TM, tiles_n = (n + TN - 1) / TN;
    const int max_stages = (int)(kMaxInt32K / S / (2 * kFrag));
    const int nst = kp / kFrag / 2;
    const int nblocks = (nst + max_stages - 1) / max_stages;
    const int stages_per_block = (nst + nblocks - 1) / nblocks;
    if (slots && nblocks != 1) return hipErrorInvalidValue;
    const long long slot_stride = slots ? (long long)tiles_m * tiles_n * S * TM * TN : 0;
    dim3 grid((unsigned)tile_order_blocks(tiles_m, tiles_n, true), nblocks, nwin);
    kern<<<grid, THREADS, G::LDS, st>>>(pA, pB, nullptr, nullptr, nullptr, 0, m, n, kp / kFrag, tiles_m, tiles_n, nullptr,
                                        totals, stages_per_block, 1, slot_stride, wins);
    return hipGetLastError();
}

// Alternative tiles.  4 slices: the 192 x 128 tile runs its products about 6.5 % faster than the 128 x 128 tile
// (8192^3: +3.3 % although its 43 x 64 tiles make 10.75 rounds of the 256 CUs, 3 % more padded work than the 16 whole
// rounds of 128 x 128).  2 and 3 slices: the 128 x 128 tile with a ring of three stages runs at 0.87 and 0.95 of the
// 256 x 128 tile's rate at 8192^3, but a problem of a few thousand rows and columns fills the compute units with it
// where 256 x 128 tiles leave half of them idle (2048^3, s = 3: 43 us against 66 us, and 51 us for the 64 x 64 tile).
// 5 and 6 slices: the 128 x 64 tile (0.82-0.90 and 0.94 of the 128 x 128 tile's rate) likewise (2304^3, s = 6: 183 us
// against 223 us).
std::atomic<int> g_tile_choice{0};      // test knob: 0 by cost, 1 always the tabulated tile, 2 always the alternative

constexpr double kAltSpeed = 1.065;                  // 192 x 128 against 128 x 128, 4 slices
constexpr double kMidSpeed[7] = {0, 0, 0.87, 0.95, 0, 0.88, 0.94};   // 128 x 128 (ring of three) against 256 x 128 for 2 and 3 slices, 128 x 64 against 128 x 128 for 5 and 6

// Which tile a launch without split-k takes: 0 the tabulated one, 1 the 192 x 128 tile (4 slices), 2 the 128 x 128 tile
// (2, 3 slices), 3 the 128 x 64 tile (5, 6 slices), by the launch cost of oz_common.h divided by the relative speed of the shape.
int alt_tile(int s, int m, int n)
{
    if (s < 2 || s > 6 || s == OZ_EXP_S) return 0;
    const int other = s == 4 ? 1 : s <= 3 ? 2 : 3;
    const int choice = g_tile_choice.load();
    if (choice) return choice == 2 ? other : 0;
    const int cus = device_cus();
    if (s == 4) return launch_cost(m, n, 192, 128, cus) / kAltSpeed < launch_cost(m, n, 128, 128, cus) ? 1 : 0;
    if (s >= 5) return launch_cost(m, n, 128, 64, cus) / kMidSpeed[s] < launch_cost(m, n, 128, 128, cus) ? 3 : 0;
    return launch_cost(m, n, 128, 128, cus) / kMidSpeed[s] < launch_cost(m, n, 256, 128, cus) ? 2 : 0;
}

template <int MODE>
hipError_t dispatch16(int s, int m, int n, int kp, const int8_t *pA, const int8_t *pB, const int32_t *eA,
                      const int32_t *eB, double *C, int ldc, int32_t *dump, long long *totals, int Q, bool kslots,
                      hipStream_t st)
{
    if constexpr (MODE != kBlocked) {
        const int alt = alt_tile(s, m, n);
        if (alt == 1) return launch16_s<4, MODE, 1>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, kslots, st);
        if (alt == 2 && s == 2) return launch16_s<2, MODE, 2>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, kslots, st);
        if (alt == 2 && s == 3) return launch16_s<3, MODE, 2>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, kslots, st);
        if (alt == 3 && s == 5) return launch16_s<5, MODE, 3>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, kslots, st);
        if (alt == 3 && s == 6) return launch16_s<6, MODE, 3>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, kslots, st);
    }
    switch (s) {
#define OZ_CASE(S_) \
    case S_: return launch16_s<S_, MODE>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, kslots, st);
        OZ_CASE(2) OZ_CASE(3) OZ_CASE(4) OZ_CASE(5) OZ_CASE(6) OZ_CASE(7) OZ_CASE(8) OZ_CASE(9)
#undef OZ_CASE
    }
    return hipErrorInvalidValue;
}

}  // namespace

// Slice counts for which this kernel is the faster one at 8192^3 (s = 2: +10 % and s = 3: +6 % with the ring of
// three stages, s = 4: +10 %, s = 5: +7.5 % with the wide tile, s = 6: +16 % with the wide tile and the split stage,
// s = 7 ... 9 with the pipelined schedule: +17 % over the 32x32x32 kernel).  With split-k (long contractions) the
// 32x32x32 kernel keeps s = 2, 3 (not measured there); s = 6 is 9-11 % faster here with split-k as well (2048 x 2048
// x 262144: 3465 against 3170 TOP/s).  Beyond 9 a 64-deep stage of a 128 x 64 tile does not fit LDS.  Only the
// preferred ones are instantiated.
bool fused16_preferred(int s, bool split_k) { return s >= 2 && s <= 9 && !(s <= 3 && split_k); }

hipError_t launch_fused16_windows(int s, int m, int n, int kp, const int8_t *pA, const int8_t *pB, long long *totals,
                                  const WindowList16 &wins, int nwin, bool slots, hipStream_t st)
{
    if (m <= 0 || n <= 0 || nwin <= 0) return hipSuccess;
    if (nwin > kMaxWindows16) return hipErrorInvalidValue;
    switch (s) {
#define OZ_CASE(S_) case S_: return launch16_windows<S_>(m, n, kp, pA, pB, totals, wins, nwin, slots, st);
        case 6: return launch16_windows<6, 3>(m, n, kp, pA, pB, totals, wins, nwin, slots, st);   // (its 128 x 64 tile)
        OZ_CASE(7) OZ_CASE(8) OZ_CASE(9)      // groups of 7, 8 or 9 slices and their reversed sets of 6, 7 or 8
#undef OZ_CASE
    }
    return hipErrorInvalidValue;
}

hipError_t launch_finish_blocks16(const long long *totals, const int32_t *eA, const int32_t *eB, double *C, int ldc,
                                  int m, int n, int Q, int diagonals, int na_tot, hipStream_t st)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    const int tiles_m = (m + 127) / 128, tiles_n = (n + 63) / 64;
    finish_blocks16_kernel<<<dim3(tiles_m * tiles_n, 4), 512, 0, st>>>(totals, eA, eB, C, ldc, m, n, tiles_n, Q, diagonals, na_tot);
    return hipGetLastError();
}

hipError_t launch_finish_slots16(const int32_t *slots, int nf, int G, const SlotTerms &terms, const int32_t *eA,
                                 const int32_t *eB, double *C, int ldc, int m, int n, int Q, int diagonals, hipStream_t st)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    if (diagonals < 1 || diagonals > kMaxSlotDiagonals || G < 7 || G > 9) return hipErrorInvalidValue;
    const int tiles_m = (m + 127) / 128, tiles_n = (n + 63) / 64;
    const long long tile_values = (long long)tiles_m * tiles_n * 128 * 64;
    finish_slots16_kernel<<<dim3(tiles_m * tiles_n, 4), 512, 0, st>>>(slots, nf, G, tile_values * G, tile_values * (G - 1), terms, eA,
                                                             eB, C, ldc, m, n, tiles_n, Q, diagonals);
    return hipGetLastError();
}

double fused16_launch_cost(int s, int m, int n, int cus)
{
    const int alt = alt_tile(s, m, n);
    if (alt == 1) return launch_cost(m, n, 192, 128, cus) / kAltSpeed;
    if (alt == 2) return launch_cost(m, n, 128, 128, cus) / kMidSpeed[s];
    if (alt == 3) return launch_cost(m, n, 128, 64, cus) / kMidSpeed[s];
    int tm, tn;
    fused16_tile(s, tm, tn);
    return launch_cost(m, n, tm, tn, cus);
}

int fused16_split_k_slots(int s, int kp)
{
    if (s < 2 || s > 9) return 0;
    const int max_stages = (int)(kMaxInt32K / s / (2 * kFrag)), nst = kp / (2 * kFrag);
    const int nblocks = (nst + max_stages - 1) / max_stages;
    return nblocks >= 2 && nblocks <= kMaxSplitKSlots ? nblocks : 0;
}

void fused16_set_tile_choice(int choice) { g_tile_choice.store(choice < 0 || choice > 2 ? 0 : choice); }

void fused16_tile(int s, int &tm, int &tn)
{
    tm = s <= 3 ? 256 : 128;
    tn = s <= 6 ? 128 : 64;
    if (s == OZ_EXP_S) {
        tm = 32 * OZ_EXP_WVM * OZ_EXP_WMF;
        tn = 32 * OZ_EXP_WVN * OZ_EXP_WNF;
    }
}

hipError_t launch_gemm_fused16(int m, int n, int kp, int s, const int8_t *pA, const int8_t *pB, const int32_t *eA,
                               const int32_t *eB, double *C, int ldc, int32_t *dump, long long *totals, int Q,
                               bool kslots, hipStream_t st)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    if (dump) return dispatch16<kDump>(s, m, n, kp, pA, pB, eA, eB, C, ldc, dump, nullptr, Q, false, st);
    if (totals) return dispatch16<kBlocked>(s, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, totals, Q, kslots, st);
    return dispatch16<kPlain>(s, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, nullptr, Q, false, st);
}

}  // namespace oz
