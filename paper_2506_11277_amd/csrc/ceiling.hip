// Measurement aid for the benchmark: what int8 rate do the matrix cores of THIS chip sustain
// when nothing else happens?  A register-only loop of independent v_mfma_i32_32x32x32_i8 or
// v_mfma_i32_16x16x64_i8 (no LDS, no memory), two wavefronts per SIMD, with constant operands, one pseudo-random
// operand pair, or a register tile of pseudo-random operands.
// The two differ markedly on MI355X (the clock drops under the switching power of real data),
// which is the context the roofline fraction of the GEMM kernel has to be read in.
#include "gemm_dev.h"

namespace oz {
namespace {


// SHAPE16: v_mfma_i32_16x16x64_i8 (16 accumulator sets of 4 registers) instead of 32x32x32 (8 sets of 16): the
// same number of int8 operations per iteration.
template <bool SHAPE16>
__global__ __launch_bounds__(512) void mfma_loop_kernel(int iters, int random_operands, int *sink)
{
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 17u;
    auto next = [&]() { x = x * 1664525u + 1013904223u; return (int)x; };
    // random_operands 0: constants; 1: one pseudo-random A and B register set for every instruction; 2: a tile of
    // pseudo-random operands as a GEMM's register tile has it (4 A x 4 B fragments for 16x16x64, 2 x 4 for
    // 32x32x32), so that consecutive instructions see different operands.
    v4i a[4], b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (random_operands) {
            a[q] = v4i{next(), next(), next(), next()};
            b[q] = v4i{next(), next(), next(), next()};
        } else {
            a[q] = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
            b[q] = v4i{0x02020202, 0x02020202, 0x02020202, 0x02020202};
        }
    }
    if (random_operands != 2) {
#pragma unroll
        for (int q = 1; q < 4; ++q) { a[q] = a[0]; b[q] = b[0]; }
    }
    int s = 0;
    if (SHAPE16) {
        v4i acc[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = v4i{0, 0, 0, 0};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) s ^= acc[i][r];
    } else {
        v16i acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i & 1], b[i >> 1], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) s ^= acc[i][r];
    }
    if (s == 0x7fffffff) sink[0] = s;   // keeps the loop alive; practically never taken
}

// The same 16x16x64 loop with the data movement of the GEMM kernel added, and nothing else of it (no barriers, no
// dependence on the data that moves): LDSR operand registers are re-read from LDS per 16 matrix instructions
// (ds_read_b128, one iteration ahead of their use), and DMA copies of 1 KiB per wavefront go from an L2-resident
// window of `src` into LDS per 16 matrix instructions (global_load_lds_dwordx4).  The GEMM kernel at 7 slices does
// 4 reads and 1.5 copies per 16 instructions.  What this loop sustains under the board's power cap is what the
// cap leaves once the bytes move, however well a kernel hides their latency.
template <int LDSR, int DMA2, bool VIAREG = false>     // DMA2: copies per 32 matrix instructions
__global__ __launch_bounds__(512) void mfma_traffic_kernel(int iters, const int8_t *__restrict__ src, int windows,
                                                           int *sink)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // 128 KiB: [0, 64K) read, [64K, 128K) filled
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 17u;
    auto next = [&]() { x = x * 1664525u + 1013904223u; return (int)x; };
    // pseudo-random bytes in this wavefront's 8 KiB of the read region
    for (int i = 0; i < 8; ++i) *(v4i *)(lds + wave * 8192 + i * 1024 + lane * 16) = v4i{next(), next(), next(), next()};
    __syncthreads();
    v4i a[4], b[4], an[4], bn[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        a[q] = an[q] = v4i{next(), next(), next(), next()};
        b[q] = bn[q] = v4i{next(), next(), next(), next()};
    }
    v4i acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = v4i{0, 0, 0, 0};
    const int8_t *win = src + (size_t)(blockIdx.x % windows) * 65536 + wave * 8192;
    unsigned cnt = 0;
    v4i pend[4] = {a[0], a[1], a[2], a[3]};
    for (int it = 0; it < iters; it += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (LDSR > 0 && i < LDSR) {
                    // operand for the NEXT 16 instructions, from a rotating 1 KiB fragment of the wavefront's region
                    const v4i v = *(const v4i *)(lds + wave * 8192 + ((h * 4 + i) & 7) * 1024 + lane * 16);
                    if (i & 1) bn[(i >> 1) & 3] = v; else an[(i >> 1) & 3] = v;
                }
                acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
                if (DMA2 > 0 && (h * 16 + i) * DMA2 / 32 != (h * 16 + i + 1) * DMA2 / 32) {
                    const unsigned o = (cnt++ & 7u) * 1024;
                    if (VIAREG) {
                        // the same copy through registers: store what was loaded four copies ago, load the next
                        const int slot = ((h * 16 + i) * DMA2 / 32) & 3;
                        *(v4i *)(lds + 65536 + wave * 8192 + o + lane * 16) = pend[slot];
                        pend[slot] = *(const v4i *)(win + o + lane * 16);
                    } else
                        lds_dma16(win + o, lane * 16, lds0 + 65536 + wave * 8192 + o);
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) { a[q] = an[q]; b[q] = bn[q]; }
        }
        if (DMA2 > 0) wait_vmcnt<8>();
    }
    wait_vmcnt<0>();
    int s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) s ^= acc[i][r];
    if (s == 0x7fffffff) sink[0] = s;
}

// Plain copy of 16-byte words: a kernel whose HBM traffic is known exactly (n16 * 16 bytes read, the same
// written), against which the readings of the memory counters can be scaled.
__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                               size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

}  // namespace
}  // namespace oz

extern "C" int ozimmu_calibration_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return OZIMMU_BAD_ARG;
    if (bytes == 0) return OZIMMU_OK;
    oz::calibration_copy_kernel<<<8192, 256, 0, (hipStream_t)stream>>>((const uint4 *)src, (uint4 *)dst, bytes / 16);
    return hipGetLastError() == hipSuccess ? OZIMMU_OK : OZIMMU_HIP_ERROR;
}

static int measure_ceiling(int random_operands, bool shape16, int *sink, float *tops, void *stream);

extern "C" int ozimmu_measure_int8_with_traffic(int lds_reads, int dma_copies_per_32, const void *src, size_t src_bytes,
                                                int *sink, float *tops, void *stream)
{
    if (!sink || !tops || !src || src_bytes < 65536 || ((uintptr_t)src & 15)) return OZIMMU_BAD_ARG;
    void (*kern)(int, const int8_t *, int, int *) = nullptr;
    if (lds_reads == 0 && dma_copies_per_32 == 0) kern = oz::mfma_traffic_kernel<0, 0>;
    else if (lds_reads == 4 && dma_copies_per_32 == 0) kern = oz::mfma_traffic_kernel<4, 0>;
    else if (lds_reads == 0 && dma_copies_per_32 == 3) kern = oz::mfma_traffic_kernel<0, 3>;
    else if (lds_reads == 4 && dma_copies_per_32 == 3) kern = oz::mfma_traffic_kernel<4, 3>;
    else if (lds_reads == 2 && dma_copies_per_32 == 3) kern = oz::mfma_traffic_kernel<2, 3>;
    else if (lds_reads == 4 && dma_copies_per_32 == 2) kern = oz::mfma_traffic_kernel<4, 2>;
    else if (lds_reads == 3 && dma_copies_per_32 == 2) kern = oz::mfma_traffic_kernel<3, 2>;
    else if (lds_reads == 5 && dma_copies_per_32 == 4) kern = oz::mfma_traffic_kernel<5, 4>;
    else if (lds_reads == 6 && dma_copies_per_32 == 4) kern = oz::mfma_traffic_kernel<6, 4>;
    else if (lds_reads == 5 && dma_copies_per_32 == 3) kern = oz::mfma_traffic_kernel<5, 3>;
    else if (lds_reads == 4 && dma_copies_per_32 == -3) kern = oz::mfma_traffic_kernel<4, 3, true>;
    else if (lds_reads == 0 && dma_copies_per_32 == -3) kern = oz::mfma_traffic_kernel<0, 3, true>;
    else return OZIMMU_BAD_ARG;
    hipStream_t st = (hipStream_t)stream;
    int cus = 0, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return OZIMMU_HIP_ERROR;
    constexpr int kLds = 128 * 1024;
    if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLds) != hipSuccess)
        return OZIMMU_HIP_ERROR;
    const size_t w = src_bytes / 65536;
    const int windows = w > 64 ? 64 : (int)w;         // a few MiB at most: resident in the L2s
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return OZIMMU_HIP_ERROR;
    const int iters = 12000, wgs = cus * 4;
    int rc = OZIMMU_OK;
    float ms = 0.f;
    kern<<<wgs, 512, kLds, st>>>(iters / 8, (const int8_t *)src, windows, sink);   // warm-up
    if (hipEventRecord(e0, st) != hipSuccess) rc = OZIMMU_HIP_ERROR;
    kern<<<wgs, 512, kLds, st>>>(iters, (const int8_t *)src, windows, sink);
    if (hipGetLastError() != hipSuccess) rc = OZIMMU_HIP_ERROR;
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
        rc = OZIMMU_HIP_ERROR;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc == OZIMMU_OK) *tops = (float)(2.0 * 16 * 16 * 64 * 16.0 * iters * 8.0 * wgs / (ms * 1e-3) / 1e12);
    return rc;
}

extern "C" int ozimmu_measure_int8_ceiling(int random_operands, int *sink, float *tops, void *stream)
{
    return measure_ceiling(random_operands, false, sink, tops, stream);
}

extern "C" int ozimmu_measure_int8_ceiling2(int random_operands, int shape, int *sink, float *tops, void *stream)
{
    if ((shape != 0 && shape != 1) || random_operands < 0 || random_operands > 2) return OZIMMU_BAD_ARG;
    return measure_ceiling(random_operands, shape == 1, sink, tops, stream);
}

static int measure_ceiling(int random_operands, bool shape16, int *sink, float *tops, void *stream)
{
    if (!sink || !tops) return OZIMMU_BAD_ARG;
    hipStream_t st = (hipStream_t)stream;
    int cus = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return OZIMMU_HIP_ERROR;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return OZIMMU_HIP_ERROR;
    const int iters = 12000, wgs = cus * 4;     // about 50-70 ms: long enough for the clock to settle
    int rc = OZIMMU_OK;
    float ms = 0.f;
    auto kern = shape16 ? oz::mfma_loop_kernel<true> : oz::mfma_loop_kernel<false>;
    kern<<<wgs, 512, 0, st>>>(iters / 8, random_operands, sink);   // warm-up
    if (hipEventRecord(e0, st) != hipSuccess) rc = OZIMMU_HIP_ERROR;
    kern<<<wgs, 512, 0, st>>>(iters, random_operands, sink);
    if (hipGetLastError() != hipSuccess) rc = OZIMMU_HIP_ERROR;
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
        rc = OZIMMU_HIP_ERROR;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc == OZIMMU_OK) *tops = (float)(2.0 * 32 * 32 * 32 * 8.0 * iters * 8.0 * wgs / (ms * 1e-3) / 1e12);
    return rc;
}
