// Scale extraction: per-row (A) and per-column (B) reduction of |x| on the bit patterns.
//
// For finite non-negative binary64 values the order of the values is the order of their bit
// patterns read as unsigned integers, so max |x| and the smallest nonzero |x| are integer
// max/min reductions: exact and independent of the reduction order (Sect. 3, eq. (alpha-def),
// (beta-def); the minimum feeds kappa of eq. (a-bound-row-2), (b-bound) in Sect. 4).
#include "oz_common.h"

// The operands are streamed once here (and once more by the slicing kernel, which gains nothing from finding
// them in a cache): loads marked non-temporal run 10 % faster (8192^3: 0.184 -> 0.165 ms for both operands).
#define OZ_LD(p) __builtin_nontemporal_load(&(p))

namespace oz {

namespace {

constexpr unsigned long long kAbsMask = 0x7fffffffffffffffULL;
constexpr unsigned long long kExpMask = 0x7ff0000000000000ULL;
constexpr unsigned long long kNoMin = 0xffffffffffffffffULL;

struct Acc {
    unsigned long long mx, mn;
    unsigned int bad;
};

__device__ __forceinline__ void fold(Acc &a, unsigned long long bits)
{
    unsigned long long v = bits & kAbsMask;
    a.mx = v > a.mx ? v : a.mx;
    unsigned long long w = v ? v : kNoMin;
    a.mn = w < a.mn ? w : a.mn;
    a.bad |= (v & kExpMask) == kExpMask;
}

// ---- side 'B': one work-group per column, wavefront-shuffle tree, then 4 partials via LDS ----
__device__ __forceinline__ void colreduce_block(int j, const unsigned long long *__restrict__ X, int ldx, int rows,
                                                unsigned long long *__restrict__ maxbits,
                                                unsigned long long *__restrict__ minbits,
                                                unsigned int *__restrict__ flags)
{
    const unsigned long long *col = X + (size_t)j * ldx;
    Acc a{0ULL, kNoMin, 0u};
    int r = threadIdx.x;
    // 4 independent loads in flight per lane
    for (; r + 768 < rows; r += 1024) {
        unsigned long long v0 = OZ_LD(col[r]), v1 = OZ_LD(col[r + 256]), v2 = OZ_LD(col[r + 512]), v3 = OZ_LD(col[r + 768]);
        fold(a, v0); fold(a, v1); fold(a, v2); fold(a, v3);
    }
    for (; r < rows; r += 256) fold(a, OZ_LD(col[r]));

    for (int off = 32; off > 0; off >>= 1) {
        unsigned long long omx = __shfl_xor(a.mx, off);
        unsigned long long omn = __shfl_xor(a.mn, off);
        unsigned int ob = __shfl_xor(a.bad, off);
        a.mx = omx > a.mx ? omx : a.mx;
        a.mn = omn < a.mn ? omn : a.mn;
        a.bad |= ob;
    }
    __shared__ unsigned long long smx[4], smn[4];
    __shared__ unsigned int sbad[4];
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { smx[w] = a.mx; smn[w] = a.mn; sbad[w] = a.bad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long mx = smx[0], mn = smn[0];
        unsigned int bad = sbad[0];
        for (int i = 1; i < 4; ++i) {
            mx = smx[i] > mx ? smx[i] : mx;
            mn = smn[i] < mn ? smn[i] : mn;
            bad |= sbad[i];
        }
        maxbits[j] = mx;
        if (minbits) minbits[j] = mn;
        if (bad) atomicOr(flags, 1u);
    }
}

__global__ __launch_bounds__(256) void colreduce_kernel(const unsigned long long *__restrict__ X, int ldx, int rows,
                                                        unsigned long long *__restrict__ maxbits,
                                                        unsigned long long *__restrict__ minbits,
                                                        unsigned int *__restrict__ flags)
{
    colreduce_block(blockIdx.x, X, ldx, rows, maxbits, minbits, flags);
}

// ---- side 'A': lane <-> row (coalesced along the column-major rows), 4 wavefronts split a
//      chunk of columns, partials meet in LDS, one integer atomic per row and work-group ----
constexpr int kRowChunk = 256;   // columns per work-group

__device__ __forceinline__ void rowreduce_block(int bx, int by, const unsigned long long *__restrict__ X, int ldx,
                                                int rows, int cols, unsigned long long *__restrict__ maxbits,
                                                unsigned long long *__restrict__ minbits,
                                                unsigned int *__restrict__ flags)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = bx * 64 + lane;
    const int c0 = by * kRowChunk + w * (kRowChunk / 4);
    int c1 = c0 + kRowChunk / 4;
    c1 = c1 < cols ? c1 : cols;
    Acc a{0ULL, kNoMin, 0u};
    if (r < rows) {
        const unsigned long long *p = X + r;
        int c = c0;
        for (; c + 7 < c1; c += 8) {
            unsigned long long v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = OZ_LD(p[(size_t)(c + u) * ldx]);
#pragma unroll
            for (int u = 0; u < 8; ++u) fold(a, v[u]);
        }
        for (; c < c1; ++c) fold(a, p[(size_t)c * ldx]);
    }
    __shared__ unsigned long long smx[4][64], smn[4][64];
    __shared__ unsigned int sbad[4][64];
    smx[w][lane] = a.mx; smn[w][lane] = a.mn; sbad[w][lane] = a.bad;
    __syncthreads();
    if (w == 0 && r < rows) {
        unsigned long long mx = smx[0][lane], mn = smn[0][lane];
        unsigned int bad = sbad[0][lane];
        for (int i = 1; i < 4; ++i) {
            mx = smx[i][lane] > mx ? smx[i][lane] : mx;
            mn = smn[i][lane] < mn ? smn[i][lane] : mn;
            bad |= sbad[i][lane];
        }
        if (mx) atomicMax(&maxbits[r], mx);
        if (minbits && mn != kNoMin) atomicMin(&minbits[r], mn);
        if (bad) atomicOr(flags, 1u);
    }
}

__global__ __launch_bounds__(256) void rowreduce_kernel(const unsigned long long *__restrict__ X, int ldx, int rows,
                                                        int cols, unsigned long long *__restrict__ maxbits,
                                                        unsigned long long *__restrict__ minbits,
                                                        unsigned int *__restrict__ flags)
{
    rowreduce_block(blockIdx.x, blockIdx.y, X, ldx, rows, cols, maxbits, minbits, flags);
}

// Both operands in one launch (ozimmu_dgemm: fewer, larger launches matter for small problems): the first
// nblkA work-groups reduce A (numbered rows-block fastest), the others one column of B each.
__global__ __launch_bounds__(256) void reduce_both_kernel(const unsigned long long *__restrict__ A, int lda, int m, int k,
                                                          const unsigned long long *__restrict__ B, int ldb, int n,
                                                          unsigned long long *__restrict__ maxA,
                                                          unsigned long long *__restrict__ maxB,
                                                          unsigned int *__restrict__ flags, int gxA, int nblkA)
{
    const int b = blockIdx.x;
    if (b < nblkA) rowreduce_block(b % gxA, b / gxA, A, lda, m, k, maxA, nullptr, flags);
    else colreduce_block(b - nblkA, B, ldb, k, maxB, nullptr, flags);
}

// header cleared, row maxima of A set to 0 (they are formed with atomic max)
__global__ void init_scales_kernel(unsigned long long *hdr, unsigned long long *maxA, int m)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 32) hdr[i] = 0ULL;
    if (i < m) maxA[i] = 0ULL;
}

__global__ void fill_u64_kernel(unsigned long long *p, unsigned long long v, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void clear_header_kernel(unsigned long long *hdr)
{
    if (threadIdx.x < 32) hdr[threadIdx.x] = 0ULL;
}

__global__ void finalize_kernel(const unsigned long long *__restrict__ maxbits,
                                const unsigned long long *__restrict__ minbits, int32_t *__restrict__ exps,
                                int nblk, int nblk_padded, unsigned long long *kappa_bits, int bias)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= nblk_padded) return;
    if (b >= nblk) { exps[b] = 0; return; }
    unsigned long long mx = maxbits[b];
    exps[b] = exponent_above(mx) + bias;
    if (kappa_bits && mx) {
        double ratio = __longlong_as_double((long long)mx) / __longlong_as_double((long long)minbits[b]);
        atomicMax(kappa_bits, (unsigned long long)__double_as_longlong(ratio));
    }
}

// exponents of both operands in one launch (no kappa)
__global__ void finalize_both_kernel(const unsigned long long *__restrict__ maxA, int32_t *__restrict__ expA, int m,
                                     int mp, const unsigned long long *__restrict__ maxB, int32_t *__restrict__ expB,
                                     int n, int np, int bias)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < mp) { expA[b] = b < m ? exponent_above(maxA[b]) + bias : 0; return; }
    b -= mp;
    if (b < np) expB[b] = b < n ? exponent_above(maxB[b]) + bias : 0;
}

}  // namespace

hipError_t launch_scales_fused(int m, int n, int k, const double *A, int lda, const double *B, int ldb,
                               unsigned long long *hdr, unsigned long long *maxA, unsigned long long *maxB,
                               int32_t *expA, int mp, int32_t *expB, int np, int bias, bool finalize, hipStream_t st)
{
    const int mm = m > 0 ? m : 0;
    init_scales_kernel<<<(mm + 32 + 255) / 256, 256, 0, st>>>(hdr, maxA, mm);
    const int gxA = (mm + 63) / 64, gyA = k > 0 ? (k + kRowChunk - 1) / kRowChunk : 0;
    const long long nblkA = (long long)gxA * gyA, nblkB = n > 0 ? n : 0;
    if (nblkA + nblkB > 0x7fffffffLL) return hipErrorInvalidValue;
    if (nblkA + nblkB > 0)
        reduce_both_kernel<<<(unsigned)(nblkA + nblkB), 256, 0, st>>>((const unsigned long long *)A, lda, m, k,
                                                                      (const unsigned long long *)B, ldb, n, maxA, maxB,
                                                                      (unsigned int *)hdr, gxA > 0 ? gxA : 1, (int)nblkA);
    // (the slicing kernel that follows forms the exponents from the maxima itself and stores them; only a call that
    // ends here, an empty product, needs them from this launch)
    if (finalize) finalize_both_kernel<<<(mp + np + 255) / 256, 256, 0, st>>>(maxA, expA, m, mp, maxB, expB, n, np, bias);
    return hipGetLastError();
}

hipError_t launch_clear_header(void *header, hipStream_t st)
{
    clear_header_kernel<<<1, 64, 0, st>>>((unsigned long long *)header);
    return hipGetLastError();
}

hipError_t launch_reduce(char side, int rows, int cols, const double *X, int ldx, unsigned long long *maxbits,
                         unsigned long long *minbits, unsigned int *flags, hipStream_t st)
{
    const int nblk = side == 'A' ? rows : cols;
    if (nblk <= 0) return hipSuccess;
    if (side == 'A') {
        fill_u64_kernel<<<(nblk + 255) / 256, 256, 0, st>>>(maxbits, 0ULL, nblk);
        if (minbits) fill_u64_kernel<<<(nblk + 255) / 256, 256, 0, st>>>(minbits, kNoMin, nblk);
        if (cols > 0) {
            dim3 grid((rows + 63) / 64, (cols + kRowChunk - 1) / kRowChunk);
            if (grid.y > 65535) return hipErrorInvalidValue;
            rowreduce_kernel<<<grid, 256, 0, st>>>((const unsigned long long *)X, ldx, rows, cols, maxbits, minbits,
                                                   flags);
        }
    } else {
        colreduce_kernel<<<cols, 256, 0, st>>>((const unsigned long long *)X, ldx, rows, maxbits, minbits, flags);
    }
    return hipGetLastError();
}

hipError_t launch_finalize(const unsigned long long *maxbits, const unsigned long long *minbits, int32_t *exps,
                           int nblk, int nblk_padded, unsigned long long *kappa_bits, int bias, hipStream_t st)
{
    if (nblk_padded <= 0) return hipSuccess;
    finalize_kernel<<<(nblk_padded + 255) / 256, 256, 0, st>>>(maxbits, minbits, exps, nblk, nblk_padded, kappa_bits,
                                                               bias);
    return hipGetLastError();
}

}  // namespace oz
