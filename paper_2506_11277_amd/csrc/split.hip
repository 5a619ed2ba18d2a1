// Bit-splitting of a binary64 matrix into s signed 7-bit slices (Sect. 3, eq.
// (bit-splitting-alg) in its bit-level reading: slice l holds bits (l-1)t+1 .. lt of
// |x| / 2^e after the binary point, and carries the sign of x).
//
// |x| = I * 2^q with I the integer significand, so  floor(|x| 2^{lt - e}) mod 2^t  is a
// shift of I by (e - q - lt) places and a mask: integer work only, exact.
//
// Round-to-nearest variant (second tweak of the "Enhanced algorithm" paragraph of Sect. 3): the block
// scale is 2^{e+1}, and with R_l = the integer nearest to |x| 2^{7l - e - 1} (ties to even) slice l is
// sign(x) (R_l - 128 R_{l-1}), a value in [-64, 64].  R_l = floor(.) + c_l with the round-up decision
//     c_l = guard & (sticky | lsb)
// read off the bits of I below the cut, so  slice l = field_l + c_l - 128 c_{l-1}:  still shifts and
// masks only; c_l is carried from one slice to the next.
//
// The MFMA layout written here is the one the GEMM kernel reads (see include/ozimmu.h):
// fragments of 32 (R) x 32 (K) bytes, 16 contiguous K-bytes per wavefront lane.
#include "oz_common.h"

namespace oz {

namespace {

struct Elem {
    unsigned long long I;   // integer significand
    int base;               // e - q : right shift that would bring bit position 0 (the binary point) to bit 0
    int neg;
};

__device__ __forceinline__ Elem decompose(unsigned long long bits, int e)
{
    Elem el;
    const int E = (int)((bits >> 52) & 0x7ff);
    const unsigned long long f = bits & 0xfffffffffffffULL;
    el.I = E ? (f | (1ULL << 52)) : f;
    el.base = e - ((E ? E : 1) - 1075);
    el.neg = (int)(bits >> 63);
    return el;
}

// slice l (1-based), as an unsigned byte holding the two's complement int8
__device__ __forceinline__ unsigned int slice_byte(const Elem &el, int l)
{
    const int sh = el.base - kSliceBits * l;
    unsigned long long v;
    if (sh >= 64) v = 0;
    else if (sh >= 0) v = el.I >> sh;
    else if (sh <= -kSliceBits) v = 0;
    else v = el.I << (-sh);
    int d = (int)(v & 127ULL);
    d = el.neg ? -d : d;
    return (unsigned int)d & 0xffu;
}

// slice l by round-to-nearest (el.base taken from the biased exponent e + 1).  `carry` is bit `bit` of a
// per-lane mask: on entry c_{l-1}, on exit c_l (the caller walks l = 1, 2, ... with the mask cleared first:
// c_0 = 0 because |x| 2^{-e-1} < 1/2).
template <bool NEAREST>
__device__ __forceinline__ unsigned int slice_of(const Elem &el, int l, unsigned int &carry, int bit)
{
    if (!NEAREST) return slice_byte(el, l);
    const int sh = el.base - kSliceBits * l;      // bits of I below the cut
    int field, c = 0;
    if (sh > 64) field = 0;                       // I < 2^53 lies below half a unit
    else if (sh >= 1) {
        const unsigned long long t = el.I >> (sh - 1);            // guard bit at bit 0, the slice above it
        const unsigned int lo = (unsigned int)t;
        const bool sticky = (t << (sh - 1)) != el.I;
        field = (int)((lo >> 1) & 127u);
        c = (int)(lo & 1u) & ((int)sticky | (int)((lo >> 1) & 1u));
    } else if (sh > -kSliceBits) field = (int)((el.I << (-sh)) & 127ULL);   // nothing below the cut
    else field = 0;
    int d = field + c - 128 * (int)((carry >> bit) & 1u);
    carry = (carry & ~(1u << bit)) | ((unsigned int)c << bit);
    d = el.neg ? -d : d;
    return (unsigned int)d & 0xffu;
}

// ---- side 'A': X is R x K column-major (R contiguous).  lane <-> row, each lane walks 16
//      consecutive k, so the 16 K-bytes of a lane come out of registers: the transposition to
//      K-contiguous fragments costs nothing, reads are 512 B per wavefront load, writes are
//      512 B contiguous per half wavefront.
template <bool NEAREST>
__device__ __forceinline__ void split_rows_block(int bx, int by, const unsigned long long *__restrict__ X, int ldx,
                                                 int R, int K, int s, int cs, const int32_t *__restrict__ exps,
                                                 int8_t *__restrict__ planes, int KB,
                                                 const unsigned long long *__restrict__ maxbits = nullptr,
                                                 int32_t *__restrict__ exps_out = nullptr)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = bx * 64 + lane;
    const int k0 = by * 64 + w * 16;
    // (maxbits given: the exponent comes from the row's maximum, biased by one for nearest slices, and the
    // work-groups of the first k-block store it, zero for the padding rows)
    const int e = r >= R ? 0 : maxbits ? exponent_above(maxbits[r]) + (NEAREST ? 1 : 0) : exps[r];
    if (exps_out && by == 0 && w == 0) exps_out[r] = e;
    Elem el[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int kk = k0 + i;
        unsigned long long bits = (r < R && kk < K) ? X[r + (size_t)kk * ldx] : 0ULL;
        el[i] = decompose(bits, e);
    }
    const int rb = r >> 5, kb = k0 >> 5, half = (k0 >> 4) & 1;
    // (the planes hold cs >= s slices per entry; those beyond s are zeros)
    uint4 *dst = (uint4 *)(planes + ((size_t)rb * KB + kb) * (size_t)cs * kFragBytes) + ((r & 31) + 32 * half);
    for (int l = s + 1; l <= cs; ++l) dst[(size_t)(l - 1) * (kFragBytes / 16)] = make_uint4(0, 0, 0, 0);
    unsigned int carry = 0;
    for (int l = 1; l <= s; ++l) {
        unsigned int wd[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            wd[q] = slice_of<NEAREST>(el[4 * q], l, carry, 4 * q) |
                    (slice_of<NEAREST>(el[4 * q + 1], l, carry, 4 * q + 1) << 8) |
                    (slice_of<NEAREST>(el[4 * q + 2], l, carry, 4 * q + 2) << 16) |
                    (slice_of<NEAREST>(el[4 * q + 3], l, carry, 4 * q + 3) << 24);
        dst[(size_t)(l - 1) * (kFragBytes / 16)] = make_uint4(wd[0], wd[1], wd[2], wd[3]);
    }
}

// ---- side 'B': X is K x R column-major (K contiguous).  A work-group takes 32 columns x 128 k;
//      lanes read along k (coalesced), slice bytes are packed four k at a time into LDS rows,
//      then re-read so that lane <-> column and a wavefront emits whole 1 KiB fragments.
constexpr int kColTileK = 128;
constexpr int kColLdsRow = kColTileK + 16;   // bytes per (slice, column) row in LDS
constexpr int kColGroup = 8;                 // slices per LDS pass

template <bool NEAREST>
__global__ __launch_bounds__(256) void split_rows_kernel(const unsigned long long *__restrict__ X, int ldx, int R,
                                                         int K, int s, const int32_t *__restrict__ exps,
                                                         int8_t *__restrict__ planes, int KB)
{
    split_rows_block<NEAREST>(blockIdx.x, blockIdx.y, X, ldx, R, K, s, s, exps, planes, KB);
}

template <bool NEAREST>
__device__ __forceinline__ void split_cols_block(int bx, int by, const unsigned long long *__restrict__ X, int ldx,
                                                 int R, int K, int s, int cs, const int32_t *__restrict__ exps,
                                                 int8_t *__restrict__ planes, int KB,
                                                 const unsigned long long *__restrict__ maxbits = nullptr,
                                                 int32_t *__restrict__ exps_out = nullptr)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[kColGroup * 32 * kColLdsRow];
    const int t = threadIdx.x;
    const int j0 = bx * 32, k0 = by * kColTileK;
    const int kq = (t & 31) * 4;
    Elem el[4][4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int jj = p * 8 + (t >> 5);
        const int j = j0 + jj;
        const int e = j >= R ? 0 : maxbits ? exponent_above(maxbits[j]) + (NEAREST ? 1 : 0) : exps[j];
        if (exps_out && by == 0 && (t & 31) == 0) exps_out[j] = e;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = k0 + kq + i;
            unsigned long long bits = (j < R && kk < K) ? X[kk + (size_t)j * ldx] : 0ULL;
            el[p][i] = decompose(bits, e);
        }
    }
    const int jj2 = t & 31, ch = t >> 5;                    // phase 2: column, 16-byte chunk along k
    const int rb = j0 >> 5;
    const int kb = (k0 + ch * 16) >> 5, half = ch & 1;
    uint4 *dst = (uint4 *)(planes + ((size_t)rb * KB + kb) * (size_t)cs * kFragBytes) + (jj2 + 32 * half);
    for (int l = s + 1; l <= cs; ++l) dst[(size_t)(l - 1) * (kFragBytes / 16)] = make_uint4(0, 0, 0, 0);
    unsigned int carry = 0;
    for (int l0 = 1; l0 <= s; l0 += kColGroup) {
        const int nl = (s - l0 + 1) < kColGroup ? (s - l0 + 1) : kColGroup;
        for (int dl = 0; dl < nl; ++dl) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int jj = p * 8 + (t >> 5);
                unsigned int wd = slice_of<NEAREST>(el[p][0], l0 + dl, carry, 4 * p) |
                                  (slice_of<NEAREST>(el[p][1], l0 + dl, carry, 4 * p + 1) << 8) |
                                  (slice_of<NEAREST>(el[p][2], l0 + dl, carry, 4 * p + 2) << 16) |
                                  (slice_of<NEAREST>(el[p][3], l0 + dl, carry, 4 * p + 3) << 24);
                *(unsigned int *)(lds + ((size_t)dl * 32 + jj) * kColLdsRow + kq) = wd;
            }
        }
        __syncthreads();
        for (int dl = 0; dl < nl; ++dl) {
            uint4 v = *(const uint4 *)(lds + ((size_t)dl * 32 + jj2) * kColLdsRow + ch * 16);
            dst[(size_t)(l0 + dl - 1) * (kFragBytes / 16)] = v;
        }
        __syncthreads();
    }
}

template <bool NEAREST>
__global__ __launch_bounds__(256) void split_cols_kernel(const unsigned long long *__restrict__ X, int ldx, int R,
                                                         int K, int s, const int32_t *__restrict__ exps,
                                                         int8_t *__restrict__ planes, int KB)
{
    split_cols_block<NEAREST>(blockIdx.x, blockIdx.y, X, ldx, R, K, s, s, exps, planes, KB);
}

// Both operands in one launch: the first nblkA work-groups slice A (numbered rows-block fastest), the others B.
template <bool NEAREST>
__global__ __launch_bounds__(256) void split_both_kernel(const unsigned long long *__restrict__ A, int lda, int m,
                                                         const unsigned long long *__restrict__ B, int ldb, int n, int K,
                                                         int sA, int sB, int cA, int cB,
                                                         const unsigned long long *__restrict__ maxA,
                                                         const unsigned long long *__restrict__ maxB,
                                                         int32_t *__restrict__ eA, int32_t *__restrict__ eB,
                                                         int8_t *__restrict__ pA, int8_t *__restrict__ pB, int KB,
                                                         int gxA, int nblkA, int gxB)
{
    const int b = blockIdx.x;
    if (b < nblkA) split_rows_block<NEAREST>(b % gxA, b / gxA, A, lda, m, K, sA, cA, nullptr, pA, KB, maxA, eA);
    else split_cols_block<NEAREST>((b - nblkA) % gxB, (b - nblkA) / gxB, B, ldb, n, K, sB, cB, nullptr, pB, KB, maxB, eB);
}

// ---- plain layout: plane l is a matrix shaped like X (utility / test path) ----
template <bool NEAREST>
__global__ __launch_bounds__(256) void split_plain_kernel(const unsigned long long *__restrict__ X, int ldx, int rows,
                                                          int cols, int s, const int32_t *__restrict__ exps,
                                                          int by_row, int8_t *__restrict__ planes)
{
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    const size_t plane = (size_t)rows * cols;
    for (int c = blockIdx.y; c < cols; c += gridDim.y) {
        const int e = by_row ? exps[r] : exps[c];
        const Elem el = decompose(X[r + (size_t)c * ldx], e);
        unsigned int carry = 0;
        for (int l = 1; l <= s; ++l)
            planes[(size_t)(l - 1) * plane + r + (size_t)c * rows] = (int8_t)slice_of<NEAREST>(el, l, carry, 0);
    }
}

}  // namespace

hipError_t launch_split(char side, int rows, int cols, const double *X, int ldx, int s, const int32_t *exps,
                        int8_t *planes, int layout, bool nearest, hipStream_t st)
{
    if (layout == OZIMMU_LAYOUT_PLAIN) {
        if (rows <= 0 || cols <= 0) return hipSuccess;
        dim3 grid((rows + 255) / 256, cols < 65535 ? cols : 65535);
        auto kern = nearest ? split_plain_kernel<true> : split_plain_kernel<false>;
        kern<<<grid, 256, 0, st>>>((const unsigned long long *)X, ldx, rows, cols, s, exps, side == 'A' ? 1 : 0, planes);
        return hipGetLastError();
    }
    const int R = side == 'A' ? rows : cols, K = side == 'A' ? cols : rows;
    const int Rp = round_up(R > 0 ? R : 1, kPad), Kp = round_up(K > 0 ? K : 1, kPad);
    const int KB = Kp / kFrag;
    if (side == 'A') {
        dim3 grid(Rp / 64, Kp / 64);
        if (grid.y > 65535) return hipErrorInvalidValue;
        auto kern = nearest ? split_rows_kernel<true> : split_rows_kernel<false>;
        kern<<<grid, 256, 0, st>>>((const unsigned long long *)X, ldx, R, K, s, exps, planes, KB);
    } else {
        dim3 grid(Rp / 32, Kp / kColTileK);
        if (grid.y > 65535) return hipErrorInvalidValue;
        auto kern = nearest ? split_cols_kernel<true> : split_cols_kernel<false>;
        kern<<<grid, 256, 0, st>>>((const unsigned long long *)X, ldx, R, K, s, exps, planes, KB);
    }
    return hipGetLastError();
}

hipError_t launch_split_both(int m, int n, int k, const double *A, int lda, const double *B, int ldb, int sA, int sB,
                             int cA, int cB, const unsigned long long *maxA, const unsigned long long *maxB, int32_t *eA,
                             int32_t *eB, int8_t *pA, int8_t *pB, bool nearest, hipStream_t st)
{
    if (cA < sA || cB < sB) return hipErrorInvalidValue;
    const int mp = round_up(m > 0 ? m : 1, kPad), np = round_up(n > 0 ? n : 1, kPad), kp = round_up(k > 0 ? k : 1, kPad);
    const int gxA = mp / 64, gxB = np / 32;
    const long long nblkA = (long long)gxA * (kp / 64), nblkB = (long long)gxB * (kp / kColTileK);
    if (nblkA + nblkB > 0x7fffffffLL) return hipErrorInvalidValue;
    auto kern = nearest ? split_both_kernel<true> : split_both_kernel<false>;
    kern<<<(unsigned)(nblkA + nblkB), 256, 0, st>>>((const unsigned long long *)A, lda, m,
                                                    (const unsigned long long *)B, ldb, n, k, sA, sB, cA, cB, maxA, maxB, eA, eB,
                                                    pA, pB, kp / kFrag, gxA, (int)nblkA, gxB);
    return hipGetLastError();
}

}  // namespace oz
