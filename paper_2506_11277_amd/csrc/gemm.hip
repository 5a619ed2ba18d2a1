// Slice-pair products on the int8 matrix cores with the binary64 accumulation fused in.
//
// What is computed (Algorithm 1 of Sect. 3, lines "E <- A_(l) B^(h)" and "S <- S + 2^{-(l+h)t} E",
// in the by-diagonal order of the subsection "Accumulation in floating-point arithmetic"):
//   D_d  = sum_{l+h=d, l,h<=s} A_(l) B^(h)          exact, int32 (k-blocked: int64)
//   S    = ((2^{-2t} D_2 + 2^{-3t} D_3) + 2^{-4t} D_4) + ...      one binary64 rounding per "+"
//   C_ij = 2^{eA_i + eB_j} S_ij
//
// Operand planes are stored as 1 KiB fragments of 32 (R) x 32 (K) int8, byte (lane*16 + b)
// of a fragment being what lane `lane` feeds to v_mfma_i32_32x32x32_i8 (lane%32 = row or
// column inside the fragment, lane/32 and b select the K position).  The K position -> (lane/32, b)
// map is the same for both operands, which is all an integer dot product needs.
//
// The MFMA is issued "transposed": the B-plane fragment is the first operand and the A-plane
// fragment the second, so that in the 32x32 result lane%32 runs along m.  C is column-major, so
// each accumulator register then stores 32 consecutive doubles of a column: 256 B segments.
#include <type_traits>

#include "gemm_dev.h"

namespace oz {

namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));   // 16-byte copy unit

constexpr int kThreads = 256;   // generic kernel: 4 wavefronts, 2 (m) x 2 (n)

// =============================== fused kernel ===========================================
// All s diagonals live in int32 accumulators for the whole contraction; needs
// s * k * 127^2 < 2^31.  Per k-step every slice of the A tile and of the B tile is staged
// once in LDS and feeds all s(s+1)/2 products.
//
// Work-group: WVM x WVN wavefronts (two per SIMD when 8), each owning WMF x WNF fragments of
// 32 x 32 outputs for every diagonal.  Operand stages are copied HBM/L2 -> LDS by the
// global_load_lds (LDS-DMA) form of the vector load, 1 KiB per wavefront instruction, into a
// ring of NSTAGE buffers: no staging registers, no ds_write, and the loads of stage st+NSTAGE-1
// are in flight while stage st is multiplied.  The loads are issued from inline asm, so the
// waits on them (vmcnt) are placed by hand below.
//   S      slices (compile time: the pair loop is fully unrolled)
//   KB32   32-deep k-blocks per LDS stage
//   MODE   kPlain: whole contraction in int32 (needs s * k * 127^2 < 2^31)
//          kDump:  as kPlain, but write the int32 diagonal sums instead of C (test hook)
//          kBlocked: any k.  The contraction is cut into k-blocks short enough for int32, one work-group
//                  per (tile, k-block) (blockIdx.y = k-block).  Each adds its int32 diagonal sums into
//                  int64 totals in HBM with integer atomics -- exact, so the totals do not depend on
//                  the order of arrival and the result stays bit-reproducible; finish_blocked_kernel
//                  then does the binary64 accumulation.  With exactly two k-blocks (slot_stride != 0) nothing
//                  has to be added on the way: each block stores its int32 sums into a slot of its own (the two
//                  slots fill the same buffer), no clearing, no atomics, and the finish kernel adds the two
//   PSET   product set.  0: both operands have S slices, products l + h <= S + 1.  3: both have S slices, ALL
//          S * S products ("Computation of all products", Sect. 4): 2 S - 1 diagonals, so 2 S - 1 accumulator
//          sets (S <= 9).  1 / 2: different slice counts (subsection "Reduction in number
//          of products" of Sect. 4): S is the LARGER count, the operand A (1) or B (2) has only `sm` < S
//          slices (run time), and the products are l + h <= S + 1 with the short operand's index <= sm.  The
//          pair loop stays fully unrolled over the long operand; the short operand's loop is the outer one and
//          simply ends after sm slices, so no product needs a test of its own.  LDS keeps the layout for S
//          slices of both operands (the short one's upper slots stay unused).
//          3 takes its S slices from a WINDOW of planes that hold more slices per entry (SliceWindow below).

// Where a launch finds its S slices in the planes and where its diagonals go in the split-k totals: the planes
// hold strA / strB slices per entry and the launch multiplies slices offA + 1 ... offA + S of A and
// offB + 1 ... offB + S of B (PSET == 3 only); its diagonal a is diagonal a + a0 of the na_tot diagonals the totals
// hold per entry.
struct SliceWindow {
    int strA, strB, offA, offB, a0, na_tot;
};
// several windows in one launch (blockIdx.z picks one): see WindowList16
struct SliceWindowList {
    SliceWindow w[kMaxWindows16];
};

template <int S, int WVM, int WVN, int WMF, int WNF, int KB32, int NSTAGE, int MODE, int PSET>
__global__ __launch_bounds__(64 * WVM * WVN) void gemm_fused_kernel(const int8_t *__restrict__ pA,
                                                                    const int8_t *__restrict__ pB,
                                                                    const int32_t *__restrict__ eA,
                                                                    const int32_t *__restrict__ eB,
                                                                    double *__restrict__ C, int ldc, int m, int n,
                                                                    int KB, int tiles_m, int tiles_n,
                                                                    int32_t *__restrict__ dump,
                                                                    long long *__restrict__ totals,
                                                                    int stages_per_block, int Q, int sm,
                                                                    long long slot_stride, SliceWindowList wins)
{
    const SliceWindow win = wins.w[blockIdx.z];
    static_assert(PSET == 0 || (NSTAGE == 2 && MODE != kDump), "other product sets: ring of two, no dump");
    constexpr bool DUMP = MODE == kDump;
    constexpr int NA = PSET == 3 ? 2 * S - 1 : S;      // diagonals = accumulator sets
    constexpr int NW = WVM * WVN;                      // wavefronts
    constexpr int FA = WVM * WMF, FB = WVN * WNF;      // fragment rows per work-group tile along m / n
    constexpr int CHUNK = KB32 * S * kFragBytes;       // bytes of one fragment row per stage (contiguous in HBM)
    constexpr int STAGE = (FA + FB) * CHUNK;
    constexpr int UNITS = STAGE / kFragBytes;          // 1 KiB copy units per stage
    constexpr int UPW = UNITS / NW, UREM = UNITS % NW; // units per wavefront (+1 for the first UREM wavefronts)
    static_assert(NSTAGE == 2 || NSTAGE == 3, "ring depth");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;

    int tm, tn;
    if (!tile_of_block_xcd(blockIdx.x, tiles_m, tiles_n, MODE == kBlocked, tm, tn)) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % WVM, wn = wave / WVM;
    const int sA = PSET == 1 ? sm : S, sB = PSET == 2 ? sm : S;                 // slices in the planes of A / B
    const int plA = PSET == 3 ? win.strA : sA, plB = PSET == 3 ? win.strB : sB;  // slices per entry in the planes
    const size_t row_bytesA = (size_t)KB * plA * kFragBytes;    // one fragment row of an operand, all k
    const size_t row_bytesB = (size_t)KB * plB * kFragBytes;
    const int8_t *rowA = pA + (size_t)tm * FA * row_bytesA;
    const int8_t *rowB = pB + (size_t)tn * FB * row_bytesB;
    const bool extra = wave < UREM;

    // copy of stage `st` into ring buffer `buf`: unit u = wave + i*NW  ->  fragment row c = u / (KB32*S)
    // part < 0: all units of the stage; else the units i with i % NPART == part (see SPREAD below)
    constexpr int NPART = S < 4 ? S : 4;
    auto issue_stage = [&](int st, int buf, int part = -1) {
#pragma unroll
        for (int i = 0; i < UPW + (UREM ? 1 : 0); ++i) {
            if (i == UPW && !extra) break;
            if (part >= 0 && i % NPART != part) continue;
            const int u = wave + i * NW;
            const int c = u / (KB32 * S), o = u % (KB32 * S);
            const int8_t *src;
            if (PSET == 0) {
                src = (c < FA ? rowA + (size_t)c * row_bytesA : rowB + (size_t)(c - FA) * row_bytesB) +
                      (size_t)st * CHUNK + (size_t)o * kFragBytes;
            } else {
                const int kbl = o / S, sl = o % S;                          // LDS slot (k-block, slice)
                const int cnt = c < FA ? sA : sB;
                if (sl >= cnt) continue;                                    // the short operand has no such slice
                const int pl = c < FA ? plA : plB, off = PSET == 3 ? (c < FA ? win.offA : win.offB) : 0;
                src = (c < FA ? rowA + (size_t)c * row_bytesA : rowB + (size_t)(c - FA) * row_bytesB) +
                      ((size_t)(st * KB32 + kbl) * pl + off + sl) * kFragBytes;
            }
            lds_dma16(src, lane * 16, lds0 + buf * STAGE + u * kFragBytes);
        }
    };
    // wait until at most `keep` stages issued by this wavefront are still in flight
    auto wait_keep1 = [&]() {
        if (extra) wait_vmcnt<UPW + 1>(); else wait_vmcnt<UPW>();
    };

    v16i acc[NA][WMF][WNF];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int i = 0; i < WMF; ++i)
#pragma unroll
            for (int j = 0; j < WNF; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][i][j][r] = 0;

    // stages of this work-group: everything, or k-block blockIdx.y
    const int nst_all = KB / KB32;
    const int st0 = MODE == kBlocked ? (int)blockIdx.y * stages_per_block : 0;
    const int nst = MODE == kBlocked && st0 + stages_per_block < nst_all ? st0 + stages_per_block : nst_all;
    // PIPE: the main loop software-pipelined by hand, for equal slice counts 5 ... 11 with one 32-deep k-block per
    // stage and a ring of two.  The slices of A go from the last to the first; the operands of slice l - 1 (its A
    // fragments, the one B slice it needs beyond those of slice l) are read while the products of slice l run; the
    // end-of-stage barrier stands at the START of the products of slice 0 (every read of the stage is issued by
    // then) and the first operands of the next stage are read behind it while those products run; the copies of
    // the next stage are issued one at a time behind single matrix instructions, two instructions each (source
    // addresses formed once per wavefront, the stage in the 32-bit lane offset relative to the work-group's first
    // stage, the LDS address one scalar add into m0), so that the loop body has no branch but a ragged last copy.
    // Measured: 8192^3 s = 10 / 11 +4 %; 2048 x 2048 x 262144 s = 6 / 10 / 11 +2 ... 4 %; the 64 x 64 tile of small
    // problems -12 % time at 512^3 s = 9 (no gain below 7 slices there).  From 12 slices on (and for the
    // four-wavefront shape of 13 ... 20 slices) it brings nothing over the loop below with its copies issued in
    // portions, and with part of B read on demand (17 ... 20) it is slower.
    constexpr bool PIPE = PSET == 0 && NSTAGE == 2 && KB32 == 1 && S >= 5 && S <= 11 && (NW == 8 || S >= 7);
    if constexpr (PIPE) {
        constexpr int NU = (UNITS + NW - 1) / NW;
        const int8_t *src[NU];
#pragma unroll
        for (int i = 0; i < NU; ++i) {
            const int u = wave + i * NW;
            const int c = u / S, o = u % S;
            src[i] = (c < FA ? rowA + (size_t)c * row_bytesA : rowB + (size_t)(c - FA) * row_bytesB) +
                     (size_t)st0 * CHUNK + (size_t)o * kFragBytes;
        }
        const unsigned ldsw = lds0 + wave * kFragBytes;
        auto issue = [&](auto I, unsigned voff, unsigned ldsbuf) {
            constexpr int i = decltype(I)::value;
            if (i < UNITS / NW || wave < UNITS % NW) lds_dma16_at<i * NW * kFragBytes>(src[i], voff, ldsbuf);
        };
        auto issue_n = [&](int i, unsigned voff, unsigned ldsbuf) {
            switch (i) {
#define OZ_U(N_) case N_: if constexpr (N_ < NU) issue(std::integral_constant<int, N_>{}, voff, ldsbuf); break;
                OZ_U(0) OZ_U(1) OZ_U(2) OZ_U(3) OZ_U(4) OZ_U(5) OZ_U(6) OZ_U(7) OZ_U(8) OZ_U(9) OZ_U(10) OZ_U(11)
                OZ_U(12) OZ_U(13) OZ_U(14) OZ_U(15) OZ_U(16) OZ_U(17) OZ_U(18) OZ_U(19)
#undef OZ_U
            }
        };
        static_assert(NU <= 20, "unit dispatch");
#pragma unroll
        for (int i = 0; i < NU; ++i) issue_n(i, lane * 16, ldsw);
        wait_vmcnt<0>();
        __syncthreads();

        auto readA = [&](int l, const unsigned char *stage, int i) -> v4i {
            return *(const v4i *)(stage + (wm * WMF + i) * CHUNK + l * kFragBytes + lane * 16);
        };
        auto readB = [&](int h, const unsigned char *stage, int j) -> v4i {
            return *(const v4i *)(stage + (FA + wn * WNF + j) * CHUNK + h * kFragBytes + lane * 16);
        };
        // beyond 16 slices only the first HP slices of B are held in registers, the others are read when needed
        // (at slice 0 they are needed first, so that the barrier still follows the last read of the stage)
        constexpr int HP = S > 18 ? 4 : S > 16 ? 8 : S;
        constexpr int MPP = WMF * WNF, NSLOT = S * (S - 1) / 2;
        static_assert(NU <= NSLOT * MPP, "too few products to issue the copies behind");
        v4i bf[HP][WNF], af[WMF];
#pragma unroll
        for (int i = 0; i < WMF; ++i) af[i] = readA(S - 1, lds, i);
#pragma unroll
        for (int j = 0; j < WNF; ++j) bf[0][j] = readB(0, lds, j);

        int buf = 0;
        for (int st = st0; st < nst; ++st) {
            // (in the last stage the copies and the reads ahead go on, of that stage again: nobody uses them)
            const bool more = st + 1 < nst;
            const unsigned vnext = lane * 16 + (unsigned)((more ? st + 1 : st) - st0) * (unsigned)CHUNK;
            const unsigned ldsnext = ldsw + (buf ^ 1) * STAGE;
            const unsigned char *cur = lds + buf * STAGE, *nxt = lds + (buf ^ 1) * STAGE;
            v4i afn[WMF], bfn[WNF];
            int slot = 0;
#pragma unroll
            for (int l = S - 1; l >= 0; --l) {
                if (l > 0) {
#pragma unroll
                    for (int i = 0; i < WMF; ++i) afn[i] = readA(l - 1, cur, i);
                    if (S - l < HP) {
#pragma unroll
                        for (int j = 0; j < WNF; ++j) bf[S - l < HP ? S - l : 0][j] = readB(S - l, cur, j);
                    }
                    __builtin_amdgcn_sched_barrier(0);      // (the reads stay ahead of the products they hide behind)
                }
#pragma unroll
                for (int hh = 0; hh < S - l; ++hh) {
                    const int h = l == 0 ? S - 1 - hh : hh;
                    if (l == 0 && h == HP - 1) {
                        // nothing of this stage is left to read, and the next one must have landed
                        wait_vmcnt<0>();
                        __syncthreads();
#pragma unroll
                        for (int i = 0; i < WMF; ++i) afn[i] = readA(S - 1, nxt, i);
#pragma unroll
                        for (int j = 0; j < WNF; ++j) bfn[j] = readB(0, nxt, j);
                    }
#pragma unroll
                    for (int i = 0; i < WMF; ++i)
#pragma unroll
                        for (int j = 0; j < WNF; ++j) {
                            const v4i bv = h < HP ? bf[h < HP ? h : 0][j] : readB(h, cur, j);
                            acc[l + h][i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bv, af[i], acc[l + h][i][j], 0, 0, 0);
                            const int e = slot * MPP + i * WNF + j;
                            if (e < NU && l > 0) issue_n(e, vnext, ldsnext);
                        }
                    ++slot;
                }
                __builtin_amdgcn_sched_barrier(0);          // (and no product of the next slice moves up to wait for them)
#pragma unroll
                for (int i = 0; i < WMF; ++i) af[i] = afn[i];
            }
#pragma unroll
            for (int j = 0; j < WNF; ++j) bf[0][j] = bfn[j];
            buf ^= 1;
        }
    } else {
        issue_stage(st0, 0);
        if (NSTAGE == 3 && nst - st0 > 1) {
            issue_stage(st0 + 1, 1);
            wait_keep1();
        } else {
            wait_vmcnt<0>();
        }
        __syncthreads();

        int buf = 0;
        for (int st = st0; st < nst; ++st) {
            const bool ahead = st + NSTAGE - 1 < nst;
            // SPREAD: the copies of the next stage are not issued all at once at the top of the stage but in NPART
            // portions, one before each of the first NPART slices of the outer loop.  Measured at 8192^3: +7.5 % for
            // the four-wavefront shape (s = 13: 2855 -> 3075, s = 16: 3087 -> 3316 TOP/s), +2 % at s = 12, nothing at
            // 10 and 11, -3.5 % at s = 6: used from 12 accumulator sets on.
            // (Not for different slice counts: with few slices in the outer loop the late portions find no products
            // left to hide behind, and deciding that at run time costs more than spreading gains.)
            constexpr bool SPREAD = NSTAGE == 2 && KB32 == 1 && NA >= 12 && (PSET == 0 || PSET == 3);
            const int nbuf = buf == 0 ? NSTAGE - 1 : buf - 1;
            if (ahead && !SPREAD) issue_stage(st + NSTAGE - 1, nbuf);
            const unsigned char *cur = lds + buf * STAGE;
#pragma unroll
            for (int kbl = 0; kbl < KB32; ++kbl) {
                // beyond 16 slices only the first HP slices of the preloaded operand are held for the whole stage,
                // the others are read when needed
                constexpr int HP = S > 18 ? 4 : S > 16 ? 8 : S;
                if (PSET != 2) {
                    v4i bf[HP][WNF];
#pragma unroll
                    for (int h = 0; h < HP; ++h)
#pragma unroll
                        for (int j = 0; j < WNF; ++j)
                            bf[h][j] = *(const v4i *)(cur + (FA + wn * WNF + j) * CHUNK + (kbl * S + h) * kFragBytes + lane * 16);
#pragma unroll
                    for (int l = 0; l < S; ++l) {
                        if (SPREAD && ahead && l < NPART) issue_stage(st + NSTAGE - 1, nbuf, l);
                        if (PSET == 1 && l >= sm) continue;     // (not `break`: the loop must stay fully unrollable)
                        v4i af[WMF];
#pragma unroll
                        for (int i = 0; i < WMF; ++i)
                            af[i] = *(const v4i *)(cur + (wm * WMF + i) * CHUNK + (kbl * S + l) * kFragBytes + lane * 16);
#pragma unroll
                        for (int h = 0; h < (PSET == 3 ? S : S - l); ++h)
#pragma unroll
                            for (int i = 0; i < WMF; ++i)
#pragma unroll
                                for (int j = 0; j < WNF; ++j) {
                                    const v4i bv = h < HP ? bf[h < HP ? h : 0][j]
                                                          : *(const v4i *)(cur + (FA + wn * WNF + j) * CHUNK +
                                                                           (kbl * S + h) * kFragBytes + lane * 16);
                                    acc[l + h][i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bv, af[i], acc[l + h][i][j], 0, 0, 0);
                                }
                    }
                } else {
                    // B is the short operand: its slices form the outer loop, those of A are held
                    v4i af[HP][WMF];
#pragma unroll
                    for (int l = 0; l < HP; ++l)
#pragma unroll
                        for (int i = 0; i < WMF; ++i)
                            af[l][i] = *(const v4i *)(cur + (wm * WMF + i) * CHUNK + (kbl * S + l) * kFragBytes + lane * 16);
#pragma unroll
                    for (int h = 0; h < S; ++h) {
                        if (h >= sm) continue;
                        v4i bf[WNF];
#pragma unroll
                        for (int j = 0; j < WNF; ++j)
                            bf[j] = *(const v4i *)(cur + (FA + wn * WNF + j) * CHUNK + (kbl * S + h) * kFragBytes + lane * 16);
#pragma unroll
                        for (int l = 0; l < S - h; ++l)
#pragma unroll
                            for (int i = 0; i < WMF; ++i)
#pragma unroll
                                for (int j = 0; j < WNF; ++j) {
                                    const v4i av = l < HP ? af[l < HP ? l : 0][i]
                                                          : *(const v4i *)(cur + (wm * WMF + i) * CHUNK +
                                                                           (kbl * S + l) * kFragBytes + lane * 16);
                                    acc[l + h][i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf[j], av, acc[l + h][i][j], 0, 0, 0);
                                }
                    }
                }
            }
            // stage st+1 must have landed before anyone reads it: with a ring of 3 the stage issued in
            // this iteration may stay in flight, otherwise everything has to be back
            if (NSTAGE == 3 && ahead) wait_keep1(); else wait_vmcnt<0>();
            __syncthreads();
            buf = buf + 1 == NSTAGE ? 0 : buf + 1;
        }
    }

    if (MODE == kBlocked) {
        // this k-block's diagonal sums -> int64 totals of the tile, [tile][wavefront][a][i][j][r][lane]
        const size_t e0 = ((size_t)(tm * tiles_n + tn) * NW + wave) * (size_t)(win.na_tot * WMF * WNF * 16 * 64) + lane;
        if (slot_stride) {
            // two k-blocks: plain int32 stores into this block's slot
            int *slot = (int *)totals + (size_t)blockIdx.y * (size_t)slot_stride + e0;
#pragma unroll
            for (int a = 0; a < NA; ++a) {
                int *sa = slot + (size_t)a * (WMF * WNF * 16 * 64);
                asm volatile("" : "+v"(sa));
#pragma unroll
                for (int i = 0; i < WMF; ++i)
#pragma unroll
                    for (int j = 0; j < WNF; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) sa[(((size_t)i * WNF + j) * 16 + r) * 64] = acc[a][i][j][r];
                asm volatile("" ::: "memory");
            }
            return;
        }
        long long *tot = totals + e0 + (size_t)win.a0 * (WMF * WNF * 16 * 64);
#pragma unroll
        for (int a = 0; a < NA; ++a) {
            // (one diagonal at a time, its base address formed here: otherwise all 16 * S slot addresses are
            // built up front and spill)
            long long *ta = tot + (size_t)a * (WMF * WNF * 16 * 64);
            asm volatile("" : "+v"(ta));
#pragma unroll
            for (int i = 0; i < WMF; ++i)
#pragma unroll
                for (int j = 0; j < WNF; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int v = acc[a][i][j][r];
                        asm volatile("" : "+v"(v));     // (keeps the widening to 64 bits next to its use)
                        __hip_atomic_fetch_add(ta + (((size_t)i * WNF + j) * 16 + r) * 64, (long long)v,
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
            asm volatile("" ::: "memory");
        }
        return;
    }

    // epilogue: accumulator register r of lane holds  (n_local, m_local) = (8*(r/4) + 4*(lane/32) + r%4, lane%32)
    const int m0 = (tm * FA + wm * WMF) * 32, n0 = (tn * FB + wn * WNF) * 32;
#pragma unroll
    for (int i = 0; i < WMF; ++i) {
        const int mi = m0 + i * 32 + (lane & 31);
        if (mi >= m) continue;
        const int ea = DUMP ? 0 : eA[mi];
#pragma unroll
        for (int j = 0; j < WNF; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int nj = n0 + j * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (nj >= n) continue;
                if (DUMP) {
#pragma unroll
                    for (int a = 0; a < NA; ++a) dump[(size_t)a * m * n + mi + (size_t)nj * m] = acc[a][i][j][r];
                } else {
                    LevelSum sum;
#pragma unroll
                    for (int a = 0; a < NA; ++a)
                        sum.add((double)acc[a][i][j][r] * __builtin_ldexp(1.0, -kSliceBits * (a + 2)), Q, a == NA - 1);
                    __builtin_nontemporal_store(ldexp(sum.S, ea + eB[nj]), &C[mi + (size_t)nj * ldc]);   // (streaming: as in gemm_fused16_kernel)
                }
            }
        }
    }
}

// Second step of the k-blocked mode: binary64 accumulation from the int64 totals, same element
// mapping and the same order of additions as the epilogue of gemm_fused_kernel.  (S: number of diagonals.)
template <int S, int WVM, int WVN, int WMF, int WNF>
__global__ __launch_bounds__(64 * WVM * WVN) void finish_blocked_kernel(const long long *__restrict__ totals,
                                                                        const int32_t *__restrict__ eA,
                                                                        const int32_t *__restrict__ eB,
                                                                        double *__restrict__ C, int ldc, int m, int n,
                                                                        int tiles_n, int Q, long long slot_stride)
{
    constexpr int NW = WVM * WVN, FA = WVM * WMF, FB = WVN * WNF;
    const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WVM, wn = wave / WVM;
    const size_t e0 = ((size_t)blockIdx.x * NW + wave) * (size_t)(S * WMF * WNF * 16 * 64) + lane;
    const long long *tot = totals + e0;
    const int *slot = (const int *)totals + e0;      // slot_stride != 0: two int32 slots instead of int64 totals
    const int m0 = (tm * FA + wm * WMF) * 32, n0 = (tn * FB + wn * WNF) * 32;
    for (int i = 0; i < WMF; ++i) {
        const int mi = m0 + i * 32 + (lane & 31);
        if (mi >= m) continue;
        const int ea = eA[mi];
        for (int j = 0; j < WNF; ++j)
            for (int r = 0; r < 16; ++r) {
                const int nj = n0 + j * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (nj >= n) continue;
                LevelSum sum;
#pragma unroll
                for (int a = 0; a < S; ++a) {
                    const size_t e = ((((size_t)a * WMF + i) * WNF + j) * 16 + r) * 64;
                    const long long v = slot_stride ? (long long)slot[e] + (long long)slot[(size_t)slot_stride + e] : tot[e];
                    // (exact conversion: |v| < 2^53)
                    sum.add((double)v * __builtin_ldexp(1.0, -kSliceBits * (a + 2)), Q, a == S - 1);
                }
                C[mi + (size_t)nj * ldc] = ldexp(sum.S, ea + eB[nj]);
            }
    }
}

__global__ void zero_i64_kernel(long long *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

// =============================== generic kernel =========================================
// Any s and any k: one slice pair at a time.  Each pair's product is accumulated in int32 over
// k-blocks short enough not to overflow, k-block results are added exactly into an int64
// diagonal sum, and after the last pair of a diagonal the sum is converted (exactly, since
// s * k * 127^2 < 2^53) and added to S in binary64.  Work-group tile 128 (m) x 64 (n).
// With dump != null it instead writes the int32 product of the single pair (pair_l, pair_h)
// over k-blocks [kb_begin, kb_end).
__global__ __launch_bounds__(kThreads) void gemm_generic_kernel(const int8_t *__restrict__ pA,
                                                                const int8_t *__restrict__ pB,
                                                                const int32_t *__restrict__ eA,
                                                                const int32_t *__restrict__ eB,
                                                                double *__restrict__ C, int ldc, int m, int n, int s,
                                                                int KB, int tiles_m, int tiles_n, int kblk32,
                                                                int pair_l, int pair_h, int kb_begin, int kb_end,
                                                                int32_t *__restrict__ dump)
{
    constexpr int WMF = 2, FA = 4, FB = 2, KB32 = 4;
    __shared__ __attribute__((aligned(16))) unsigned char lds[(FA + FB) * KB32 * kFragBytes];
    int tm, tn;
    tile_of_block(blockIdx.x, gridDim.x, tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    double sum[WMF][16];
#pragma unroll
    for (int i = 0; i < WMF; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[i][r] = 0.0;

    const int d_lo = dump ? pair_l + pair_h : 2, d_hi = dump ? pair_l + pair_h : s + 1;
    for (int d = d_lo; d <= d_hi; ++d) {
        long long D[WMF][16];
#pragma unroll
        for (int i = 0; i < WMF; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) D[i][r] = 0;
        int l_lo = d - s > 1 ? d - s : 1, l_hi = d - 1 < s ? d - 1 : s;
        if (dump) l_lo = l_hi = pair_l;
        for (int l = l_lo; l <= l_hi; ++l) {
            const int h = d - l;
            for (int kb0 = kb_begin; kb0 < kb_end; kb0 += kblk32) {
                const int kb1 = kb0 + kblk32 < kb_end ? kb0 + kblk32 : kb_end;
                v16i acc[WMF];
#pragma unroll
                for (int i = 0; i < WMF; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][r] = 0;
                for (int kb = kb0; kb < kb1; kb += KB32) {
                    // stage: (FA + FB) fragment rows x KB32 k-blocks of this pair's two slices
                    // 6 * 4 * 64 = 1536 units of 16 B: 6 per thread
#pragma unroll
                    for (int i = 0; i < (FA + FB) * KB32 * 64 / kThreads; ++i) {
                        const int u = tid + i * kThreads;
                        const int c = u / (KB32 * 64), rest = u % (KB32 * 64);
                        const int kbl = rest / 64, o = rest % 64;
                        v4u v = {0u, 0u, 0u, 0u};
                        if (kb + kbl < kb1) {
                            const int8_t *base =
                                c < FA ? pA + (((size_t)(tm * FA + c) * KB + kb + kbl) * s + (l - 1)) * kFragBytes
                                       : pB + (((size_t)(tn * FB + c - FA) * KB + kb + kbl) * s + (h - 1)) * kFragBytes;
                            v = ((const v4u *)base)[o];
                        }
                        *(v4u *)(lds + u * 16) = v;
                    }
                    __syncthreads();
#pragma unroll
                    for (int kbl = 0; kbl < KB32; ++kbl) {
                        const v4i bf = *(const v4i *)(lds + ((FA + wn) * KB32 + kbl) * kFragBytes + lane * 16);
#pragma unroll
                        for (int i = 0; i < WMF; ++i) {
                            const v4i af = *(const v4i *)(lds + ((wm * WMF + i) * KB32 + kbl) * kFragBytes + lane * 16);
                            acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf, af, acc[i], 0, 0, 0);
                        }
                    }
                    __syncthreads();
                }
#pragma unroll
                for (int i = 0; i < WMF; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) D[i][r] += (long long)acc[i][r];
            }
        }
        if (!dump) {
#pragma unroll
            for (int i = 0; i < WMF; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) sum[i][r] = sum[i][r] + ldexp((double)D[i][r], -kSliceBits * d);
        } else {
            const int m0 = tm * FA * 32 + wm * WMF * 32, n0 = tn * FB * 32 + wn * 32;
#pragma unroll
            for (int i = 0; i < WMF; ++i) {
                const int mi = m0 + i * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int nj = n0 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (mi < m && nj < n) dump[mi + (size_t)nj * m] = (int32_t)D[i][r];
                }
            }
        }
    }
    if (dump) return;
    const int m0 = tm * FA * 32 + wm * WMF * 32, n0 = tn * FB * 32 + wn * 32;
#pragma unroll
    for (int i = 0; i < WMF; ++i) {
        const int mi = m0 + i * 32 + (lane & 31);
        if (mi >= m) continue;
        const int ea = eA[mi];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int nj = n0 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (nj < n) C[mi + (size_t)nj * ldc] = ldexp(sum[i][r], ea + eB[nj]);
        }
    }
}

// ------------------------------- launch tables --------------------------------------------
// Tile shapes per slice count, picked from a sweep at 8192^3 on random slices (all candidates
// land within a few percent of each other: the kernel is limited by the chip's power budget
// once the matrix cores are kept fed, not by a single pipe).
//   WIDE: 8 wavefronts as 2 (m) x 4 (n), each 64 x 32 outputs: tile 128 x 128 (fewer L2->LDS bytes
//         per product; fits the 256 registers of a two-per-SIMD wavefront while 32*S <= 192)
//   else: 8 wavefronts as 4 (m) x 2 (n), each 32 x 32 outputs: tile 128 x 64
//   BIG (s > 12): 4 wavefronts as 2 x 2, ONE per SIMD, each 32 x 32 outputs: tile 64 x 64.  A lone wavefront
//         may use all 512 registers of its SIMD lane (256 of them accumulation registers), which holds
//         16 * s accumulators up to s = 20; the products per staged byte grow with s, so the small tile
//         still feeds the matrix cores (3.0 POP/s at s = 16, where the band kernel reaches 1.8).
template <int S>
struct FusedCfg {
    static constexpr bool BIG = S > 12;
    static constexpr bool WIDE = S <= 4 || S == 6;
    static constexpr int WVM = BIG ? 2 : WIDE ? 2 : 4, WVN = BIG ? 2 : WIDE ? 4 : 2, WMF = WIDE ? 2 : 1, WNF = 1;
    static constexpr int FR = WVM * WMF + WVN * WNF;
    static constexpr int KB32 = S == 4 ? 2 : 1;
    static constexpr int NSTAGE = S <= 3 ? 3 : 2;
};

// Shape for problems too small to fill the chip with the tabulated tile: 4 wavefronts, tile 64 x 64 (four times
// as many work-groups as 128 x 128).  Equal counts up to 12, whole contraction in int32.
struct FusedCfgSmall {
    static constexpr int WVM = 2, WVN = 2, WMF = 1, WNF = 1, FR = 4, KB32 = 1, NSTAGE = 2;
};
constexpr int kSmallMaxS = 12;
std::atomic<long long> g_small_below_tiles{-1};           // test hook: -1 the cost rule below, 0 never, n: below n tiles

constexpr int kFusedMaxUneq = 18; // most accumulator sets for different slice counts and for all products
constexpr int kFusedMaxS = 20;   // 16 accumulator registers per diagonal: 12 fit 256 registers, 20 fit 512 (BIG);
                                 // two 32-deep stages of a 64 x 64 tile with 20 slices fill the 160 KiB of LDS

// Tile geometry of the fused kernel for a slice count (used for the size of the k-block totals).
template <int S>
void fused_tile(int &tm, int &tn)
{
    tm = 32 * FusedCfg<S>::WVM * FusedCfg<S>::WMF;
    tn = 32 * FusedCfg<S>::WVN * FusedCfg<S>::WNF;
}

// sm: slices of the short operand (PSET = 1: A, 2: B); PSET = 0, 3: sm = S.  The work-group shape is the one
// tabulated for the number of accumulator sets NA.
template <int S, int MODE, int PSET, bool SMALL = false>
hipError_t launch_fused_s(int m, int n, int kp, const int8_t *pA, const int8_t *pB, const int32_t *eA,
                          const int32_t *eB, double *C, int ldc, int32_t *dump, long long *totals, int Q, int sm,
                          hipStream_t st)
{
    constexpr int NA = PSET == 3 ? 2 * S - 1 : S;
    using Cfg = typename std::conditional<SMALL, FusedCfgSmall, FusedCfg<NA>>::type;
    constexpr int TM = 32 * Cfg::WVM * Cfg::WMF, TN = 32 * Cfg::WVN * Cfg::WNF;
    constexpr int STAGE = Cfg::FR * Cfg::KB32 * S * kFragBytes;
    constexpr int NSTAGE = PSET ? 2 : Cfg::NSTAGE;
    static_assert(NSTAGE * STAGE <= kLdsBytes, "LDS ring too large");
    static_assert(kPad % TM == 0 && kPad % TN == 0 && (kPad / kFrag) % Cfg::KB32 == 0, "tiles must divide the padding");
    auto kern = gemm_fused_kernel<S, Cfg::WVM, Cfg::WVN, Cfg::WMF, Cfg::WNF, Cfg::KB32, NSTAGE, MODE, PSET>;
    static std::atomic<unsigned long long> configured{0};
    if (hipError_t e = allow_dynamic_lds((const void *)kern, NSTAGE * STAGE, configured); e != hipSuccess) return e;
    const int tiles_m = (m + TM - 1) / TM, tiles_n = (n + TN - 1) / TN;
    note_gemm_kernel("gemm_fused_kernel<%d> %s tile %dx%d, %d wavefronts%s", S,
                     PSET == 0 ? "equal counts" : PSET == 3 ? "all products" : "different counts", TM, TN,
                     Cfg::WVM * Cfg::WVN, MODE == kBlocked ? ", split-k" : "");
    if (MODE != kBlocked) {
        kern<<<(unsigned)tile_order_blocks(tiles_m, tiles_n, false), 64 * Cfg::WVM * Cfg::WVN, NSTAGE * STAGE, st>>>(
            pA, pB, eA, eB, C, ldc, m, n, kp / kFrag, tiles_m, tiles_n, dump, nullptr, 0, Q, sm, 0,
            SliceWindowList{{SliceWindow{S, S, 0, 0, 0, NA}}});
        return hipGetLastError();
    }
    // longest k-block whose sm products per diagonal cannot overflow int32, in whole stages; the blocks are
    // then made equally long
    const int max_stages = (int)(kMaxInt32K / sm / kFrag) / Cfg::KB32;
    const int nst = kp / kFrag / Cfg::KB32;
    const int nblocks = (nst + max_stages - 1) / max_stages;
    const int stages_per_block = (nst + nblocks - 1) / nblocks;
    const size_t nslots = (size_t)tiles_m * tiles_n * NA * TM * TN;
    // exactly two k-blocks: an int32 slot per block (together the size of the int64 totals), nothing to clear
    const long long slot_stride = nblocks == 2 ? (long long)nslots : 0;
    if (!slot_stride) zero_i64_kernel<<<2048, 256, 0, st>>>(totals, nslots);
    dim3 grid((unsigned)tile_order_blocks(tiles_m, tiles_n, true), nblocks);
    kern<<<grid, 64 * Cfg::WVM * Cfg::WVN, NSTAGE * STAGE, st>>>(pA, pB, eA, eB, C, ldc, m, n, kp / kFrag, tiles_m,
                                                                  tiles_n, nullptr, totals, stages_per_block, Q, sm,
                                                                  slot_stride, SliceWindowList{{SliceWindow{S, S, 0, 0, 0, NA}}});
    finish_blocked_kernel<NA, Cfg::WVM, Cfg::WVN, Cfg::WMF, Cfg::WNF>
        <<<tiles_m * tiles_n, 64 * Cfg::WVM * Cfg::WVN, 0, st>>>(totals, eA, eB, C, ldc, m, n, tiles_n, Q, slot_stride);
    return hipGetLastError();
}

template <int MODE, int PSET>
hipError_t dispatch_fused(int s, int m, int n, int kp, const int8_t *pA, const int8_t *pB, const int32_t *eA,
                          const int32_t *eB, double *C, int ldc, int32_t *dump, long long *totals, int Q, int sm,
                          hipStream_t st)
{
    switch (s) {
    // (equal counts 2 ... 9 run in the 16x16x64 kernel -- 2 and 3 except in split-k mode -- and are not
    // instantiated here)
#define OZ_CASE(S_) \
    case S_: \
        if constexpr (PSET != 0 || S_ < 2 || S_ > 9 || (S_ <= 3 && MODE == kBlocked)) \
            return launch_fused_s<S_, MODE, PSET>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, sm, st); \
        break;
        OZ_CASE(2) OZ_CASE(3) OZ_CASE(4) OZ_CASE(5) OZ_CASE(6) OZ_CASE(7) OZ_CASE(8) OZ_CASE(9) OZ_CASE(10) OZ_CASE(11) OZ_CASE(12) OZ_CASE(13) OZ_CASE(14) OZ_CASE(15) OZ_CASE(16) OZ_CASE(17) OZ_CASE(18)
#undef OZ_CASE
        // equal counts only (a single slice: nothing to distinguish; 19 and 20: the variants for different counts
        // would spill inside the pair loop)
        case 1:
            if (PSET == 0) return launch_fused_s<1, MODE, 0>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, sm, st);
            break;
        case 19:
            if (PSET == 0) return launch_fused_s<19, MODE, 0>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, sm, st);
            break;
        case 20:
            if (PSET == 0) return launch_fused_s<20, MODE, 0>(m, n, kp, pA, pB, eA, eB, C, ldc, dump, totals, Q, sm, st);
            break;
    }
    return hipErrorInvalidValue;
}

// equal counts, whole contraction in int32, small tile
hipError_t dispatch_fused_small(int s, int m, int n, int kp, const int8_t *pA, const int8_t *pB, const int32_t *eA,
                                const int32_t *eB, double *C, int ldc, int Q, hipStream_t st)
{
    switch (s) {
#define OZ_CASE(S_) \
    case S_: return launch_fused_s<S_, kPlain, 0, true>(m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, nullptr, Q, S_, st);
        OZ_CASE(1) OZ_CASE(2) OZ_CASE(3) OZ_CASE(4) OZ_CASE(5) OZ_CASE(6) OZ_CASE(7) OZ_CASE(8) OZ_CASE(9) OZ_CASE(10) OZ_CASE(11) OZ_CASE(12)
#undef OZ_CASE
    }
    return hipErrorInvalidValue;
}

// all S * S products, equal counts: 2 S - 1 <= kFusedMaxS accumulator sets
template <int MODE>
hipError_t dispatch_fused_all(int s, int m, int n, int kp, const int8_t *pA, const int8_t *pB, const int32_t *eA,
                              const int32_t *eB, double *C, int ldc, long long *totals, int Q, hipStream_t st)
{
    switch (s) {
#define OZ_CASE(S_) \
    case S_: return launch_fused_s<S_, MODE, 3>(m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, totals, Q, S_, st);
        OZ_CASE(2) OZ_CASE(3) OZ_CASE(4) OZ_CASE(5) OZ_CASE(6) OZ_CASE(7) OZ_CASE(8) OZ_CASE(9)
#undef OZ_CASE
    }
    return hipErrorInvalidValue;
}

// ---- slice counts beyond the accumulator budget, as blocks of the (l, h) grid -------------------------------
// The slices of each operand are taken in groups of G (zero slices appended by the slicing kernel where a count is
// not a multiple of G, and to the operand with fewer groups, so that both planes hold the same number of slices per
// entry): NGA groups of A, NGB of B.  Block (I, J) -- slices I G + 1 ... (I + 1) G of A times slices
// J G + 1 ... (J + 1) G of B -- is the work of the 16x16x64 kernel on a window of the planes.  Reduced product set
// (l + h <= SP + 1 with SP = G max(NGA, NGB)): all G^2 products for I + J < NG - 1, the reduced set l' + h' <= G + 1
// for I + J = NG - 1, nothing beyond (NG = max(NGA, NGB)); all products: every block whole.  Local diagonal a of a
// block is diagonal a + G (I + J); the finishing kernel adds the diagonals of the REQUESTED product set in order.
// (Appended zero slices add nothing; the diagonals beyond the requested ones, which hold products outside the
// requested set, are not read.)
//
// The kernel computes reduced sets only (tile 128 x 64, two wavefronts per SIMD), so a whole
// block is two launches: the reduced set l' + h' <= G + 1 of the pair of groups, and the rest l' + h' >= G + 2, which
// is the reduced set of G - 1 slices once both groups are walked backwards from their last slice (l'' = G + 1 - l',
// h'' = G + 1 - h': l'' + h'' <= G, l'', h'' <= G - 1), its diagonals descending from the block's last one.
// Windows of the plan: nf blocks in all (each contributes the reduced set of G slices), nr of them whole (they also
// contribute the reversed reduced set of G - 1 slices).
inline void blocks_window_counts(const BlocksPlan &plan, bool all_products, int &nf, int &nr)
{
    const int G = plan.G, NGA = plan.spA / G, NGB = plan.spB / G, NG = NGA > NGB ? NGA : NGB;
    nf = nr = 0;
    for (int I = 0; I < NGA; ++I)
        for (int J = 0; J < NGB; ++J) {
            if (!all_products && I + J > NG - 1) continue;
            ++nf;
            if (all_products || I + J < NG - 1) ++nr;
        }
}

// A slot of int32 diagonal sums per window instead of int64 totals shared through atomics: when the contraction is
// one k-block for G slices and the windows fit one launch of each kind.
inline bool blocks_slots(const BlocksPlan &plan, bool all_products, int kp)
{
    int nf, nr;
    blocks_window_counts(plan, all_products, nf, nr);
    return nf <= kMaxWindows16 && nr <= kMaxWindows16 && kp / (2 * kFrag) <= (int)(kMaxInt32K / plan.G / (2 * kFrag));
}

inline hipError_t launch_blocks16_slots(int m, int n, int kp, const BlocksPlan &plan, bool all_products, int diagonals,
                                        const int8_t *pA, const int8_t *pB, const int32_t *eA, const int32_t *eB,
                                        double *C, int ldc, long long *totals, int Q, hipStream_t st)
{
    const int G = plan.G, NGA = plan.spA / G, NGB = plan.spB / G, NG = NGA > NGB ? NGA : NGB;
    const int stride = plan.spA > plan.spB ? plan.spA : plan.spB;      // slices per entry in both planes
    const int tiles_m = (m + 127) / 128, tiles_n = (n + 63) / 64;
    WindowList16 fwd, rev;
    int abase_f[kMaxWindows16], abase_r[kMaxWindows16];
    int nf = 0, nr = 0;
    for (int I = 0; I < NGA; ++I)
        for (int J = 0; J < NGB; ++J) {
            if (!all_products && I + J > NG - 1) continue;
            const int d0 = G * (I + J);                                       // first diagonal of the block
            if (nf >= kMaxWindows16 || nr >= kMaxWindows16) return hipErrorInvalidValue;
            abase_f[nf] = d0;
            fwd.w[nf++] = Window16{stride, I * G, 1, J * G, 1, 0, 1, G};
            if (all_products || I + J < NG - 1) {
                abase_r[nr] = d0 + 2 * G - 2;
                rev.w[nr++] = Window16{stride, I * G + G - 1, -1, J * G + G - 1, -1, 0, 1, G - 1};
            }
        }
    if (diagonals > kMaxSlotDiagonals) return hipErrorInvalidValue;
    // the terms of each requested diagonal: local diagonal a of a block is diagonal d0 + a, local diagonal a of its
    // reversed set diagonal d0 + 2 G - 2 - a
    SlotTerms terms;
    int nt = 0;
    for (int d = 0; d < diagonals; ++d) {
        terms.first[d] = (unsigned short)nt;
        for (int q = 0; q < nf; ++q)
            if (d >= abase_f[q] && d < abase_f[q] + G) terms.term[nt++] = (unsigned short)(q * 16 + (d - abase_f[q]));
        for (int q = 0; q < nr; ++q)
            if (d <= abase_r[q] && d > abase_r[q] - (G - 1)) terms.term[nt++] = (unsigned short)((nf + q) * 16 + (abase_r[q] - d));
    }
    for (int d = diagonals; d <= kMaxSlotDiagonals; ++d) terms.first[d] = (unsigned short)nt;
    const size_t tile_values = (size_t)tiles_m * tiles_n * 128 * 64;
    int32_t *slots = (int32_t *)totals;
    if (hipError_t e = launch_fused16_windows(G, m, n, kp, pA, pB, totals, fwd, nf, true, st); e != hipSuccess) return e;
    if (hipError_t e = launch_fused16_windows(G - 1, m, n, kp, pA, pB, (long long *)(slots + (size_t)nf * tile_values * G), rev, nr,
                                              true, st);
        e != hipSuccess)
        return e;
    return launch_finish_slots16(slots, nf, G, terms, eA, eB, C, ldc, m, n, Q, diagonals, st);
}

inline hipError_t launch_blocks16(int m, int n, int kp, const BlocksPlan &plan, bool all_products, int diagonals,
                                  int na_tot, const int8_t *pA, const int8_t *pB, const int32_t *eA, const int32_t *eB,
                                  double *C, int ldc, long long *totals, int Q, hipStream_t st)
{
    if (blocks_slots(plan, all_products, kp))
        return launch_blocks16_slots(m, n, kp, plan, all_products, diagonals, pA, pB, eA, eB, C, ldc, totals, Q, st);
    const int G = plan.G, NGA = plan.spA / G, NGB = plan.spB / G, NG = NGA > NGB ? NGA : NGB;
    const int stride = plan.spA > plan.spB ? plan.spA : plan.spB;
    const int tiles_m = (m + 127) / 128, tiles_n = (n + 63) / 64;
    zero_i64_kernel<<<2048, 256, 0, st>>>(totals, (size_t)tiles_m * tiles_n * na_tot * 128 * 64);
    // all blocks of the panel in two launches: the reduced sets of G slices (every block), the reversed reduced sets of
    // G - 1 slices (the whole blocks); more than kMaxWindows16 of a kind go in several launches
    WindowList16 fwd, rev;
    int nf = 0, nr = 0;
    auto flush = [&](int s_, WindowList16 &list, int &cnt) {
        const hipError_t e = launch_fused16_windows(s_, m, n, kp, pA, pB, totals, list, cnt, false, st);
        cnt = 0;
        return e;
    };
    for (int I = 0; I < NGA; ++I)
        for (int J = 0; J < NGB; ++J) {
            if (!all_products && I + J > NG - 1) continue;
            const int d0 = G * (I + J);                                       // first diagonal of the block
            fwd.w[nf++] = Window16{stride, I * G, 1, J * G, 1, d0, 1, na_tot};
            if (nf == kMaxWindows16)
                if (hipError_t e = flush(G, fwd, nf); e != hipSuccess) return e;
            if (all_products || I + J < NG - 1) {
                rev.w[nr++] = Window16{stride, I * G + G - 1, -1, J * G + G - 1, -1, d0 + 2 * G - 2, -1, na_tot};
                if (nr == kMaxWindows16)
                    if (hipError_t e = flush(G - 1, rev, nr); e != hipSuccess) return e;
            }
        }
    if (hipError_t e = flush(G, fwd, nf); e != hipSuccess) return e;
    if (hipError_t e = flush(G - 1, rev, nr); e != hipSuccess) return e;
    return launch_finish_blocks16(totals, eA, eB, C, ldc, m, n, Q, diagonals, na_tot, st);
}

}  // namespace

int fused_max_slices() { return kFusedMaxS; }

void fused_set_small_tile_limit(long long tiles) { g_small_below_tiles = tiles; }

// what the fused kernels CAN compute ...
static bool fused_capable(int sA, int sB, bool all_products)
{
    if (sA < 1 || sB < 1) return false;
    if (all_products) return sA == sB && 2 * sA - 1 <= kFusedMaxUneq;
    return sA == sB ? sA <= kFusedMaxS : (sA > sB ? sA : sB) <= kFusedMaxUneq;
}

// ... and what the routing gives them: all of it but 17, 18 and 20 equal slices where the groups of the block path
// serve them better.  18 slices are two groups of 9 and run faster as blocks through the 16x16x64 kernel than in the
// four-wavefront shape: 8192^3 (two k-blocks there) 66.7 -> 52.8 ms, 4096^3 8.0 -> 7.4 ms, the same at 2048^3, slower
// below.  17 (as 18, one zero slice) and 20 (as three groups of 7) gain where the contraction needs two k-blocks in
// the fused kernel: 8192^3 55.6 -> 52.8 ms and 81.6 -> 78.4 ms.  (14 and 16 slices, two groups of 7 and 8, gain 2-3 %
// at 8192^3 and lose as much at 4096^3: they stay; 19 as 21 would lose.)
bool fused_handles(int sA, int sB, bool all_products, int m, int n, int k)
{
    if (!all_products && sA == sB) {
        const bool two_k_blocks = (long long)sA * (k > 0 ? k : 1) > kMaxInt32K;
        if ((sA == 17 || sA == 18 || sA == 20) && two_k_blocks) return false;
        if (sA == 18 && (long long)m * n >= 2048LL * 2048LL) return false;
    }
    return fused_capable(sA, sB, all_products);
}

bool fused_single_block(int sA, int sB, int k)
{
    // the longest diagonal has min(sA, sB) products of k terms each, every term at most 127^2 in magnitude
    const int sm = sA < sB ? sA : sB;
    return fused_capable(sA, sB, false) && (long long)sm * (long long)(k > 0 ? k : 1) <= kMaxInt32K;
}

// Whether a product set runs as blocks of slice groups, and how: every set the fused kernels do not take (after
// gemm_slice_counts has tried equal counts), unless the zero slices that fill the last groups would cost more
// than 60 % extra products (then the band kernel, at about two thirds of the rate, is the cheaper one -- small
// different counts with all products).  G in {7, 8, 9} (all products of a block need 2 G - 1 <= 18 accumulator sets)
// is the one with the fewest products to compute.
bool blocks_plan(int sA, int sB, bool all_products, BlocksPlan *plan)
{
    if (sA < 1 || sB < 1 || sA > OZIMMU_MAX_SLICES || sB > OZIMMU_MAX_SLICES) return false;
    const int sM = sA > sB ? sA : sB, sm = sA > sB ? sB : sA;
    const long long needed = all_products ? (long long)sA * sB : (long long)sm * (2 * sM - sm + 1) / 2;
    long long best = -1;
    BlocksPlan bp{0, 0, 0, 0, 0};
    for (int G = 9; G >= 7; --G) {
        const int NGA = (sA + G - 1) / G, NGB = (sB + G - 1) / G, NG = NGA > NGB ? NGA : NGB;
        long long cost = 0;
        for (int I = 0; I < NGA; ++I)
            for (int J = 0; J < NGB; ++J) {
                if (all_products || I + J < NG - 1) cost += G * G;
                else if (I + J == NG - 1) cost += G * (G + 1) / 2;
            }
        if (best < 0 || cost <= best) {         // ties go to the smaller group (fewer accumulators per block)
            best = cost;
            bp = BlocksPlan{G, NGA * G, NGB * G, cost, needed};
        }
    }
    if (5 * best > 8 * needed) return false;
    if (plan) *plan = bp;
    return true;
}

// Split-k runs over column panels of C, one after the other, so that the totals of a panel (8 bytes per diagonal
// and entry) stay near kPanelBytes whatever the size of C: columns per panel, a multiple of the padding.
std::atomic<long long> g_panel_bytes{1LL << 30};
void fused_set_panel_bytes(long long bytes) { g_panel_bytes = bytes > 0 ? bytes : (1LL << 62); }

static int fused_panel_cols(int diagonals, int m, int n)
{
    const long long mp = round_up(m > 0 ? m : 1, kPad), np = round_up(n > 0 ? n : 1, kPad);
    long long w = g_panel_bytes.load() / (8LL * mp * diagonals) / kPad * kPad;
    if (w < kPad) w = kPad;
    return (int)(w < np ? w : np);
}

// int64 values the split-k buffer holds per entry of C: the diagonals, or -- where the 16x16x64 kernel gives every
// k-block an int32 slot -- half the int32 values of all slots (rounded up).  The slots are taken when all of C fits
// four times the panel budget in ONE panel (2048 x 2048 x 262144, 7 slices, 14 k-blocks: 1.6 GB; 18.9 -> 18.1 ms,
// while two panels of slots ran 19.4 ms); else int64 totals over column panels as before.
static int fused_values_per_entry(int sA, int sB, bool all_products, int kp, int m, int n, bool *kslots)
{
    const bool all = all_products && sA > 1;
    const int s = all ? 2 * sA - 1 : (sA > sB ? sA : sB);
    *kslots = false;
    if (sA == sB && !all && fused16_preferred(s, true))
        if (const int nb = fused16_split_k_slots(s, kp)) {
            const int values = (nb * s + 1) / 2;
            const long long mp = round_up(m > 0 ? m : 1, kPad), np = round_up(n > 0 ? n : 1, kPad);
            if (nb == 2 || 2LL * values * mp * np <= g_panel_bytes.load()) {
                *kslots = nb > 2;
                return values;
            }
        }
    return s;
}

size_t fused_totals_bytes(int sA, int sB, bool all_products, int m, int n, int k)
{
    if (!fused_capable(sA, sB, all_products) || fused_single_block(sA, sB, k) || m <= 0 || n <= 0) return 0;
    const bool all = all_products && sA > 1;
    const int s = all ? 2 * sA - 1 : (sA > sB ? sA : sB);        // diagonals; the tile shape is tabulated by them
    bool kslots = false;
    const int values = fused_values_per_entry(sA, sB, all_products, round_up(k > 0 ? k : 1, kPad), m, n, &kslots);
    if (!kslots) {
        const int w = fused_panel_cols(values, m, n);
        if (w < n) n = w;
    }
    int tm = 128, tn = 128;
    if (sA == sB && !all && fused16_preferred(s, true)) fused16_tile(s, tm, tn);
    else switch (s) {
#define OZ_CASE(S_) case S_: fused_tile<S_>(tm, tn); break;
        OZ_CASE(1) OZ_CASE(2) OZ_CASE(3) OZ_CASE(4) OZ_CASE(5) OZ_CASE(6) OZ_CASE(7) OZ_CASE(8) OZ_CASE(9) OZ_CASE(10) OZ_CASE(11) OZ_CASE(12) OZ_CASE(13) OZ_CASE(14) OZ_CASE(15) OZ_CASE(16) OZ_CASE(17) OZ_CASE(18) OZ_CASE(19) OZ_CASE(20)
#undef OZ_CASE
    }
    const size_t tiles = (size_t)((m + tm - 1) / tm) * ((n + tn - 1) / tn);
    return tiles * (size_t)values * tm * tn * sizeof(long long);
}

// Column panel of the block path: about g_panel_bytes of totals as for split-k, then narrowed (by up to a half) to
// the width whose tiles fill the 256 compute units in whole rounds best -- every block is a launch of its own, so a
// last round that is half empty is paid once per block (8192 rows, 24 diagonals: 640 columns are 2.5 rounds of
// 128 x 64 tiles, 512 columns are 2).
static int blocks_panel_cols(int diagonals, int m, int n, int tile_m, int tile_n)
{
    const int w0 = fused_panel_cols(diagonals, m, n);
    if (w0 >= n) return w0;
    const long long tm = (m + tile_m - 1) / tile_m;
    int best = w0;
    double best_eff = 0.0;
    for (int w = w0; w >= kPad && 2 * w >= w0; w -= kPad) {
        const long long tiles = tm * ((w + tile_n - 1) / tile_n), rounds = (tiles + 255) / 256;
        const double eff = (double)tiles / (double)(rounds * 256);
        if (eff > best_eff + 0.02) { best_eff = eff; best = w; }
    }
    return best;
}

static int blocks_total_diagonals(const BlocksPlan &p, bool all_products)
{
    return all_products ? p.spA + p.spB - 1 : (p.spA > p.spB ? p.spA : p.spB);
}

// int64 values the buffer holds per entry of C: the diagonals of the totals, or -- with a slot per window -- half the
// int32 values of all slots (rounded up); the column panels are sized by it.
static int blocks_values_per_entry(const BlocksPlan &p, bool all_products, int kp)
{
    if (!blocks_slots(p, all_products, kp)) return blocks_total_diagonals(p, all_products);
    int nf, nr;
    blocks_window_counts(p, all_products, nf, nr);
    return (nf * p.G + nr * (p.G - 1) + 1) / 2;
}

size_t blocks_totals_bytes(int sA, int sB, bool all_products, int m, int n, int k)
{
    BlocksPlan p;
    if (m <= 0 || n <= 0 || !blocks_plan(sA, sB, all_products, &p)) return 0;
    const int na_tot = blocks_values_per_entry(p, all_products, round_up(k > 0 ? k : 1, kPad));
    const int w = blocks_panel_cols(na_tot, m, n, 128, 64);          // tile 128 x 64
    const int wn = w < n ? w : n;
    return (size_t)((m + 127) / 128) * ((wn + 63) / 64) * (size_t)na_tot * 128 * 64 * sizeof(long long);
}

hipError_t launch_gemm_blocks(int m, int n, int kp, int sA, int sB, bool all_products, const int8_t *pA,
                              const int8_t *pB, const int32_t *eA, const int32_t *eB, double *C, int ldc,
                              long long *totals, int Q, hipStream_t st)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    BlocksPlan p;
    if (!blocks_plan(sA, sB, all_products, &p) || !totals) return hipErrorInvalidValue;
    const int na_tot = blocks_total_diagonals(p, all_products);
    const int diagonals = all_products ? sA + sB - 1 : (sA > sB ? sA : sB);
    note_gemm_kernel("blocks of slice groups: %d x %d groups of %d slices through gemm_fused16_kernel<%d> and <%d> "
                     "tile 128x64%s", p.spA / p.G, p.spB / p.G, p.G, p.G, p.G - 1,
                     blocks_slots(p, all_products, kp) ? ", a slot per block" : ", shared totals");
    // one column panel of C after the other through the same buffer
    const int w = blocks_panel_cols(blocks_values_per_entry(p, all_products, kp), m, n, 128, 64);
    const size_t frag_row_bytes = (size_t)(kp / kFrag) * (p.spA > p.spB ? p.spA : p.spB) * kFragBytes;      // one 32-column fragment row of B
    for (int c0 = 0; c0 < n; c0 += w) {
        const int nc = n - c0 < w ? n - c0 : w;
        const int8_t *pBc = pB + (size_t)(c0 / kFrag) * frag_row_bytes;
        double *Cc = C + (size_t)c0 * ldc;
        if (hipError_t e = launch_blocks16(m, nc, kp, p, all_products, diagonals, na_tot, pA, pBc, eA, eB + c0, Cc, ldc, totals, Q, st);
            e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

static hipError_t launch_gemm_fused_once(int m, int n, int kp, int sA, int sB, bool all_products, const int8_t *pA,
                                         const int8_t *pB, const int32_t *eA, const int32_t *eB, double *C, int ldc,
                                         int32_t *dump, long long *totals, int Q, bool kslots, hipStream_t st);

hipError_t launch_gemm_fused(int m, int n, int kp, int sA, int sB, bool all_products, const int8_t *pA,
                             const int8_t *pB, const int32_t *eA, const int32_t *eB, double *C, int ldc,
                             int32_t *dump, long long *totals, int Q, hipStream_t st)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    if (!fused_capable(sA, sB, all_products)) return hipErrorInvalidValue;
    if (!totals) return launch_gemm_fused_once(m, n, kp, sA, sB, all_products, pA, pB, eA, eB, C, ldc, dump, totals, Q, false, st);
    // split-k: one column panel of C after the other, all through the same totals buffer
    bool kslots = false;
    const int values = fused_values_per_entry(sA, sB, all_products, kp, m, n, &kslots);
    const int w = kslots ? round_up(n, kPad) : fused_panel_cols(values, m, n);
    const size_t frag_row_bytes = (size_t)(kp / kFrag) * sB * kFragBytes;      // one 32-column fragment row of B
    for (int c0 = 0; c0 < n; c0 += w) {
        const int nc = n - c0 < w ? n - c0 : w;
        hipError_t e = launch_gemm_fused_once(m, nc, kp, sA, sB, all_products, pA, pB + (size_t)(c0 / kFrag) * frag_row_bytes,
                                              eA, eB + c0, C + (size_t)c0 * ldc, ldc, dump, totals, Q, kslots, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

static hipError_t launch_gemm_fused_once(int m, int n, int kp, int sA, int sB, bool all_products, const int8_t *pA,
                                         const int8_t *pB, const int32_t *eA, const int32_t *eB, double *C, int ldc,
                                         int32_t *dump, long long *totals, int Q, bool kslots, hipStream_t st)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    if (all_products && sA > 1) {
        if (dump) return hipErrorInvalidValue;
        if (totals) return dispatch_fused_all<kBlocked>(sA, m, n, kp, pA, pB, eA, eB, C, ldc, totals, Q, st);
        return dispatch_fused_all<kPlain>(sA, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, Q, st);
    }
    if (sA == sB) {
        const int s = sA;
        if (!dump && !totals && s <= kSmallMaxS) {
            // The 64 x 64 tile where it finishes sooner.  A launch takes (rounds of the compute units) x (time of a
            // tile), a partly filled round nearly as long as a full one; the small tile runs its products at the fraction
            // kSmallSpeed of the tabulated tile's rate (8192^3, both kernels measured per slice count).  So few tiles
            // of the tabulated shape lose to many small ones (2048^2, s = 2: 128 tiles of 256 x 128 against 4 rounds of
            // 64 x 64: the small tile is 18 % faster), but not always (2560^2: 200 large tiles are 57 % faster than 7
            // rounds of small ones, which a plain "fewer tiles than compute units" rule gets wrong).
            int tm = 128, tn = 128;
            if (fused16_preferred(s, false)) fused16_tile(s, tm, tn);
            else if (s <= 4 || s == 6) { tm = 128; tn = 128; }
            else { tm = 128; tn = 64; }
            const long long tiles = (long long)((m + tm - 1) / tm) * ((n + tn - 1) / tn);
            const long long small_tiles = (long long)((m + 63) / 64) * ((n + 63) / 64);
            const long long limit = g_small_below_tiles.load();
            bool small;
            if (limit < 0) {
                static constexpr double kSmallSpeed[kSmallMaxS + 1] = {0, 0.7, 0.63, 0.69, 0.74, 0.70, 0.76, 0.87, 0.72, 0.80, 0.93, 0.9, 0.9};
                const int cus = device_cus();
                const double tabulated = fused16_preferred(s, false) ? fused16_launch_cost(s, m, n, cus) : launch_cost(m, n, tm, tn, cus);
                small = small_tiles > tiles && launch_cost(m, n, 64, 64, cus) / kSmallSpeed[s] < tabulated;
            } else
                small = tiles < limit && small_tiles > tiles;     // test knob: a plain threshold on the tile count
            if (small)
                return dispatch_fused_small(s, m, n, kp, pA, pB, eA, eB, C, ldc, Q, st);
        }
        // the 16x16x64 kernel where it is the faster one
        if (fused16_preferred(s, totals != nullptr))
            return launch_gemm_fused16(m, n, kp, s, pA, pB, eA, eB, C, ldc, dump, totals, Q, kslots, st);
        if (dump) return dispatch_fused<kDump, 0>(s, m, n, kp, pA, pB, eA, eB, C, ldc, dump, nullptr, Q, s, st);
        if (totals) return dispatch_fused<kBlocked, 0>(s, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, totals, Q, s, st);
        return dispatch_fused<kPlain, 0>(s, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, nullptr, Q, s, st);
    }
    if (dump) return hipErrorInvalidValue;
    // different slice counts: the kernel for the larger count, the short operand's count at run time
    const int s = sA > sB ? sA : sB, sm = sA > sB ? sB : sA;
    if (sA < sB) {
        if (totals) return dispatch_fused<kBlocked, 1>(s, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, totals, Q, sm, st);
        return dispatch_fused<kPlain, 1>(s, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, nullptr, Q, sm, st);
    }
    if (totals) return dispatch_fused<kBlocked, 2>(s, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, totals, Q, sm, st);
    return dispatch_fused<kPlain, 2>(s, m, n, kp, pA, pB, eA, eB, C, ldc, nullptr, nullptr, Q, sm, st);
}

hipError_t launch_gemm_generic(int m, int n, int kp, int s, const int8_t *pA, const int8_t *pB, const int32_t *eA,
                               const int32_t *eB, double *C, int ldc, int pair_l, int pair_h, int kb_begin,
                               int kb_end, int32_t *dump, hipStream_t st)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    const int tiles_m = (m + 127) / 128, tiles_n = (n + 63) / 64;
    note_gemm_kernel("gemm_generic_kernel tile 128x64");
    // int32-safe k-block for one pair: kblk * 127^2 < 2^31, rounded down to a whole number of stages
    const int kblk32 = (int)(kMaxInt32K / kFrag) / 4 * 4;
    gemm_generic_kernel<<<tiles_m * tiles_n, kThreads, 0, st>>>(pA, pB, eA, eB, C, ldc, m, n, s, kp / kFrag, tiles_m,
                                                                tiles_n, kblk32, pair_l, pair_h, kb_begin, kb_end,
                                                                dump);
    return hipGetLastError();
}

}  // namespace oz
