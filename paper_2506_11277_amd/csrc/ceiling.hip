// Measurement aid for the benchmark: what int8 rate do the matrix cores of THIS chip sustain
// when nothing else happens?  A register-only loop of independent v_mfma_i32_32x32x32_i8 or
// v_mfma_i32_16x16x64_i8 (no LDS, no memory), two wavefronts per SIMD, with constant operands, one pseudo-random
// operand pair, or a register tile of pseudo-random operands.
// The two differ markedly on MI355X (the clock drops under the switching power of real data),
// which is the context the roofline fraction of the GEMM kernel has to be read in.
#include "oz_common.h"

namespace oz {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

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
