// Slice products for ANY pair of slice counts (sA for A, sB for B) and any k: the general
// form of the product step of Algorithm 1 (Sect. 3) with the product set
//     l <= sA,  h <= sB,  l + h <= dmax        (dmax = max(sA, sB) + 1 for the reduced variant of
// the subsection "Reduction in number of products", sA + sB for "Computation of all products"),
// accumulated by diagonals in ascending order as in gemm.hip.
//
// The pair set is a band of the (l, h) grid, too large to hold in registers at once for big
// slice counts, so it is cut two ways:
//   * diagonals are taken G at a time (G int32 accumulator sets per wavefront); binary64 S is
//     carried in registers from one group to the next, so the additions keep their order (a level of
//     the level-wise accumulation that straddles two groups parks its partial sum in C meanwhile);
//   * inside a group, the slices of A are taken LA at a time.  A chunk of LA slices of A meets,
//     on the G diagonals of the group, a window of LB = G + LA - 1 consecutive slices of B, and
//     the product A-slice `la` x window slot `hb` belongs to diagonal slot a = hb + la - (LA-1):
//     all register and LDS indices are compile-time, only validity (slice exists, diagonal
//     computed) is a wavefront-uniform runtime mask.
// Each (group, chunk) is one sweep over k with the LDS-DMA double buffer of the fused kernel;
// every staged slice fragment feeds up to G (A) or LA (B) MFMAs.
//
// int32 safety: a diagonal receives at most LA products per sweep.  If all sweeps of a group together
// stay below 133144 terms per accumulator, int32 suffices (TOTALS = false).  Otherwise (TOTALS) k is
// cut into blocks of at most 133144 / LA terms; the kernel keeps a bound on the terms an accumulator
// has received and, whenever one more block could pass 133144, adds the accumulators, exactly, into
// int64 totals and restarts them from zero (at k = 8192 that is after every fourth sweep, not after
// each one).  The totals live in a scratch slot per work-group (the grid is persistent, so the scratch
// does not grow with the matrix).
#include "gemm_dev.h"

namespace oz {

namespace {

constexpr int kG = 8, kLA = 4, kLB = kG + kLA - 1;
constexpr int kWVM = 4, kWVN = 2;                       // 8 wavefronts, 32 x 32 outputs each: tile 128 x 64
constexpr int kPersistentGroups = 256;                  // work-groups of the persistent grid (one per CU)

__device__ __forceinline__ void wait_all_vm() { wait_vmcnt<0>(); }

// Roles: X is the operand whose slices are taken LA at a time (the one with FEWER slices: every
// staged X slice then meets up to G diagonals), Y the one seen through the window of LB slices.
//   CHUNK_A   X = A (else X = B); the MFMA operand order (B fragment first) does not change, so the
//             lanes of the result always run along m
//   KB32      32-deep k-blocks per LDS stage (1 is used: 2 measured slower, the unrolled masked body grows too long)
template <bool CHUNK_A, int KB32>
struct BandGeom {
    static constexpr int FX = CHUNK_A ? kWVM : kWVN, FY = CHUNK_A ? kWVN : kWVM;   // fragment rows per tile
    static constexpr int UX = kLA * FX, UY = kLB * FY, UNITS1 = UX + UY;           // 1 KiB units per k-block
    static constexpr int UNITS = KB32 * UNITS1, STAGE = UNITS * kFragBytes;
};

template <bool TOTALS, bool CHUNK_A, int KB32>
__global__ __launch_bounds__(64 * kWVM * kWVN) void gemm_banded_kernel(
    const int8_t *__restrict__ pA, const int8_t *__restrict__ pB, const int32_t *__restrict__ eA,
    const int32_t *__restrict__ eB, double *__restrict__ C, int ldc, int m, int n, int sA, int sB, int dmax, int KB,
    int tiles_m, int tiles_n, long long *__restrict__ totals, int stages_per_block, int Q)
{
    using Geo = BandGeom<CHUNK_A, KB32>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % kWVM, wn = wave / kWVM;
    const int wx = CHUNK_A ? wm : wn, wy = CHUNK_A ? wn : wm;
    const int sX = CHUNK_A ? sA : sB, sY = CHUNK_A ? sB : sA;
    const int ntiles = tiles_m * tiles_n;
    const int nrounds = (ntiles + gridDim.x - 1) / gridDim.x;
    const int nst = KB / KB32;
    long long *tot = TOTALS ? totals + ((size_t)blockIdx.x * (kWVM * kWVN) + wave) * (size_t)(kG * 16 * 64) + lane
                            : nullptr;

    for (int round = 0; round < nrounds; ++round) {
        int tile_id = round * gridDim.x + blockIdx.x;
        if (tile_id >= ntiles) break;
        // one XCD-aware numbering over all tiles; the grid size is a multiple of 8 (or a single
        // round), so (tile_id % 8) names the XCD this work-group runs on
        int tm, tn;
        tile_of_block(tile_id, ntiles, tiles_m, tiles_n, tm, tn);

        const size_t rowX_bytes = (size_t)KB * sX * kFragBytes, rowY_bytes = (size_t)KB * sY * kFragBytes;
        const int8_t *rowX = CHUNK_A ? pA + (size_t)tm * kWVM * rowX_bytes : pB + (size_t)tn * kWVN * rowX_bytes;
        const int8_t *rowY = CHUNK_A ? pB + (size_t)tn * kWVN * rowY_bytes : pA + (size_t)tm * kWVM * rowY_bytes;

        double S[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) S[r] = 0.0;

        const int mi = (tm * kWVM + wm) * 32 + (lane & 31);
        const int n0 = (tn * kWVN + wn) * 32;

        // The short group comes FIRST: the early diagonals hold few products, the late ones many, and a late
        // group of only a few diagonals would sweep k once per chunk for little work.
        const int first = (dmax - 1) % kG ? (dmax - 1) % kG : kG;
        for (int d0 = 2, dlast = 1 + first; d0 <= dmax; d0 = dlast + 1, dlast += kG) {
            v16i acc[kG];
#pragma unroll
            for (int a = 0; a < kG; ++a)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][r] = 0;
            bool have_totals = false;
            int terms = 0;                      // products x k summed into an accumulator since the last flush (bound)

            const int x_lo = d0 - sY > 1 ? d0 - sY : 1;
            const int x_hi = dlast - 1 < sX ? dlast - 1 : sX;
            for (int x0 = x_lo; x0 <= x_hi; x0 += kLA) {
                const int ymin = d0 - (x0 + kLA - 1);          // slice of Y in window slot 0
                // validity of the (c, a) products of this sweep, bit c*G + a:  X slice x0+c times Y slice
                // d0+a-(x0+c) belongs to diagonal d0+a
                unsigned mask = 0;
#pragma unroll
                for (int c = 0; c < kLA; ++c)
#pragma unroll
                    for (int a = 0; a < kG; ++a) {
                        const int x = x0 + c, y = d0 + a - x;
                        if (x <= x_hi && y >= 1 && y <= sY && d0 + a <= dlast) mask |= 1u << (c * kG + a);
                    }
                if (mask == 0) continue;
                unsigned needX = 0, needY = 0;                  // which slices have to be staged
#pragma unroll
                for (int c = 0; c < kLA; ++c)
#pragma unroll
                    for (int a = 0; a < kG; ++a)
                        if (mask >> (c * kG + a) & 1u) { needX |= 1u << c; needY |= 1u << (a - c + kLA - 1); }

                auto issue_stage = [&](int st, int buf) {
#pragma unroll
                    for (int i = 0; i < (Geo::UNITS + 7) / 8; ++i) {
                        const int u = wave + i * 8;
                        if (u >= Geo::UNITS) break;
                        const int kbl = u / Geo::UNITS1, v = u % Geo::UNITS1;
                        const size_t kb = (size_t)st * KB32 + kbl;
                        const int8_t *src;
                        if (v < Geo::UX) {
                            const int c = v / Geo::FX, r = v % Geo::FX;
                            if (!(needX >> c & 1u)) continue;
                            src = rowX + (size_t)r * rowX_bytes + (kb * sX + (x0 + c - 1)) * kFragBytes;
                        } else {
                            const int yb = (v - Geo::UX) / Geo::FY, r = (v - Geo::UX) % Geo::FY;
                            if (!(needY >> yb & 1u)) continue;
                            src = rowY + (size_t)r * rowY_bytes + (kb * sY + (ymin + yb - 1)) * kFragBytes;
                        }
                        lds_dma16(src, lane * 16, lds0 + buf * Geo::STAGE + u * kFragBytes);
                    }
                };

                // the sweep over k, in blocks short enough for int32 (one block unless TOTALS)
                for (int b0 = 0; b0 < nst; b0 += stages_per_block) {
                    const int b1 = b0 + stages_per_block < nst ? b0 + stages_per_block : nst;
                    issue_stage(b0, 0);
                    wait_all_vm();
                    __syncthreads();
                    int buf = 0;
                    for (int st = b0; st < b1; ++st) {
                        if (st + 1 < b1) issue_stage(st + 1, buf ^ 1);
#pragma unroll
                        for (int kbl = 0; kbl < KB32; ++kbl) {
                            const unsigned char *cur = lds + buf * Geo::STAGE + kbl * Geo::UNITS1 * kFragBytes;
                            v4i yf[kLB];
#pragma unroll
                            for (int yb = 0; yb < kLB; ++yb)
                                if (needY >> yb & 1u)
                                    yf[yb] = *(const v4i *)(cur + (Geo::UX + yb * Geo::FY + wy) * kFragBytes + lane * 16);
#pragma unroll
                            for (int c = 0; c < kLA; ++c) {
                                if (!(needX >> c & 1u)) continue;
                                const v4i xf = *(const v4i *)(cur + (c * Geo::FX + wx) * kFragBytes + lane * 16);
#pragma unroll
                                for (int a = 0; a < kG; ++a)
                                    if (mask >> (c * kG + a) & 1u) {
                                        const v4i yv = yf[a - c + kLA - 1];
                                        acc[a] = CHUNK_A ? __builtin_amdgcn_mfma_i32_32x32x32_i8(yv, xf, acc[a], 0, 0, 0)
                                                         : __builtin_amdgcn_mfma_i32_32x32x32_i8(xf, yv, acc[a], 0, 0, 0);
                                    }
                            }
                        }
                        wait_all_vm();
                        __syncthreads();
                        buf ^= 1;
                    }
                    terms += kLA * (b1 - b0) * KB32 * kFrag;
                    if (TOTALS && terms + kLA * (stages_per_block < nst ? stages_per_block : nst) * KB32 * kFrag > (int)kMaxInt32K) {
                        terms = 0;
                        // the next k-block could overflow int32: int64 totals (+)= accumulators, accumulators restart from zero.
                        // (The base is laundered through an empty asm so that the 128 slot addresses are formed
                        // here, when needed, instead of being hoisted into registers for the whole kernel.)
                        long long *tb = tot;
                        asm volatile("" : "+v"(tb));
#pragma unroll
                        for (int a = 0; a < kG; ++a) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                long long *t = tb + ((size_t)a * 16 + r) * 64;
                                long long v = acc[a][r];
                                if (have_totals) v += *t;
                                *t = v;
                                acc[a][r] = 0;
                            }
                            asm volatile("" ::: "memory");   // one diagonal at a time
                        }
                        have_totals = true;
                    }
                }
            }
            // the group's diagonals are complete: S <- S + 2^{-7d} D_d, ascending d, in levels of Q diagonals.
            // A level may straddle two groups (Q does not divide G): its partial sum is then parked in this
            // lane's own element of C until the next group continues it.  (Read back with a device-scope
            // load so that it cannot be served from a stale L1 line.)
            const int open_in = (d0 - 2) % Q;                           // diagonals of the open level summed so far
            const bool open_out = dlast != dmax && (dlast - 1) % Q != 0;
            long long *te = tot;
            if (TOTALS) asm volatile("" : "+v"(te));
            int nlane = n0 + 4 * (lane >> 5);   // (laundered like `te`: the 16 element positions are formed here)
            asm volatile("" : "+v"(nlane));
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int nj = nlane + 8 * (r >> 2) + (r & 3);
                const bool inside = mi < m && nj < n;
                double *park = inside ? C + mi + (size_t)nj * ldc : nullptr;
                LevelSum sum;
                sum.S = S[r];
                sum.cnt = open_in;
                if (open_in && inside) sum.L = __hip_atomic_load(park, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int a = 0; a < kG; ++a) {
                    if (d0 + a > dlast) break;
                    long long v = acc[a][r];
                    if (TOTALS && have_totals) v += te[((size_t)a * 16 + r) * 64];
                    sum.add(ldexp((double)v, -kSliceBits * (d0 + a)), Q, d0 + a == dmax);
                }
                S[r] = sum.S;
                if (open_out && inside) __hip_atomic_store(park, sum.L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("" ::: "memory");   // one output element at a time
            }
        }

        if (mi < m) {
            const int ea = eA[mi];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int nj = n0 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (nj < n) C[mi + (size_t)nj * ldc] = ldexp(S[r], ea + eB[nj]);
            }
        }
    }
}

template <bool TOTALS, bool CHUNK_A, int KB32>
hipError_t launch_band(int m, int n, int kp, int sA, int sB, int dmax, const int8_t *pA, const int8_t *pB,
                       const int32_t *eA, const int32_t *eB, double *C, int ldc, long long *totals, int Q,
                       hipStream_t st)
{
    using Geo = BandGeom<CHUNK_A, KB32>;
    static_assert(2 * Geo::STAGE <= kLdsBytes, "LDS double buffer too large");
    auto kern = gemm_banded_kernel<TOTALS, CHUNK_A, KB32>;
    static std::atomic<unsigned long long> configured{0};
    if (hipError_t e = allow_dynamic_lds((const void *)kern, 2 * Geo::STAGE, configured); e != hipSuccess) return e;
    const int tiles_m = (m + 127) / 128, tiles_n = (n + 63) / 64;
    const int ntiles = tiles_m * tiles_n;
    const int grid = ntiles < kPersistentGroups ? ntiles : kPersistentGroups;
    const int KB = kp / kFrag, nst = KB / KB32;
    // a k-block adds at most LA products of (32 * KB32 * stages) terms to an accumulator
    const int stages_per_block = TOTALS ? (int)(kMaxInt32K / kLA / kFrag) / KB32 : nst;
    kern<<<grid, 64 * kWVM * kWVN, 2 * Geo::STAGE, st>>>(pA, pB, eA, eB, C, ldc, m, n, sA, sB, dmax, KB, tiles_m,
                                                         tiles_n, totals, stages_per_block, Q);
    return hipGetLastError();
}

}  // namespace

size_t banded_totals_bytes(int sA, int sB, int k)
{
    // without totals an accumulator of a group receives at most ceil(sX / LA) * LA products of kp terms
    // each (sX: slices of the chunked operand, the smaller count); that has to fit int32
    const long long kp = round_up(k > 0 ? k : 1, kPad);
    const long long sX = sA <= sB ? sA : sB;
    const long long chunks = (sX + kLA - 1) / kLA;
    if (chunks * kLA * kp <= kMaxInt32K) return 0;
    return (size_t)kPersistentGroups * (kWVM * kWVN) * kG * 16 * 64 * sizeof(long long);
}

hipError_t launch_gemm_banded(int m, int n, int kp, int sA, int sB, int dmax, const int8_t *pA, const int8_t *pB,
                              const int32_t *eA, const int32_t *eB, double *C, int ldc, long long *totals, int Q,
                              hipStream_t st)
{
    if (Q < 1 || Q > kG) return hipErrorInvalidValue;
    if (m <= 0 || n <= 0) return hipSuccess;
    note_gemm_kernel("gemm_banded_kernel (%d, %d) slices, tile 128x64", sA, sB);
    const bool chunk_a = sA <= sB;
    if (totals) {
        return chunk_a ? launch_band<true, true, 1>(m, n, kp, sA, sB, dmax, pA, pB, eA, eB, C, ldc, totals, Q, st)
                       : launch_band<true, false, 1>(m, n, kp, sA, sB, dmax, pA, pB, eA, eB, C, ldc, totals, Q, st);
    }
    return chunk_a ? launch_band<false, true, 1>(m, n, kp, sA, sB, dmax, pA, pB, eA, eB, C, ldc, nullptr, Q, st)
                   : launch_band<false, false, 1>(m, n, kp, sA, sB, dmax, pA, pB, eA, eB, C, ldc, nullptr, Q, st);
}

}  // namespace oz
