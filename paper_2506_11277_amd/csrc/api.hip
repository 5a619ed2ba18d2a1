// extern "C" boundary of libozimmu: argument checks, workspace carve-up, kernel sequencing.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "oz_common.h"

using namespace oz;

namespace oz {
static thread_local char t_last_kernel[160] = "";
void note_gemm_kernel(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(t_last_kernel, sizeof(t_last_kernel), fmt, ap);
    va_end(ap);
}
const char *last_gemm_kernel() { return t_last_kernel; }
}  // namespace oz

namespace {

inline bool bad_matrix(int rows, int cols, const void *p, int ld)
{
    if (rows < 0 || cols < 0) return true;
    if (ld < (rows > 1 ? rows : 1)) return true;
    return rows > 0 && cols > 0 && p == nullptr;
}


#define OZ_TRY(expr)                                        \
    do {                                                    \
        hipError_t e__ = (expr);                            \
        if (e__ != hipSuccess) return OZIMMU_HIP_ERROR;     \
    } while (0)

// Optional per-phase timing of ozimmu_dgemm with HIP events recorded on the caller's stream.  One timer per
// process, guarded by a mutex; a call claims its slot of four events when it starts, so calls from several threads
// never share events (their phases then interleave on the device, which is why the header asks for one thread).
struct Profile {
    std::mutex mutex;
    bool on = false;
    int capacity = 0, calls = 0;
    hipEvent_t *ev = nullptr;   // 4 events per call: start, after scales, after split, after gemm
} g_prof;

// slot of this call's events, or null when the timer is off or full
inline hipEvent_t *prof_claim()
{
    std::lock_guard<std::mutex> lock(g_prof.mutex);
    if (!g_prof.on || g_prof.calls >= g_prof.capacity) return nullptr;
    return g_prof.ev + 4 * (size_t)g_prof.calls++;
}

inline void prof_mark(hipEvent_t *slot, int phase, hipStream_t st)
{
    if (slot) (void)hipEventRecord(slot[phase], st);
}

// scales of both operands into the workspace (optionally with the minima for kappa)
int scales_into_workspace(const Workspace &w, char *ws, int m, int n, int k, const double *A, int lda,
                          const double *B, int ldb, bool with_min, int bias, hipStream_t st)
{
    auto *hdr = (unsigned long long *)(ws + w.off_header);
    auto *flags = (unsigned int *)(ws + w.off_header);
    auto *maxA = (unsigned long long *)(ws + w.off_maxA), *minA = (unsigned long long *)(ws + w.off_minA);
    auto *maxB = (unsigned long long *)(ws + w.off_maxB), *minB = (unsigned long long *)(ws + w.off_minB);
    OZ_TRY(launch_clear_header(hdr, st));
    OZ_TRY(launch_reduce('A', m, k, A, lda, maxA, with_min ? minA : nullptr, flags, st));
    OZ_TRY(launch_reduce('B', k, n, B, ldb, maxB, with_min ? minB : nullptr, flags, st));
    OZ_TRY(launch_finalize(maxA, minA, (int32_t *)(ws + w.off_expA), m, w.mp, with_min ? hdr + 1 : nullptr, bias, st));
    OZ_TRY(launch_finalize(maxB, minB, (int32_t *)(ws + w.off_expB), n, w.np, with_min ? hdr + 2 : nullptr, bias, st));
    return OZIMMU_OK;
}

}  // namespace

extern "C" {

const char *ozimmu_status_string(int status)
{
    switch (status) {
        case OZIMMU_OK: return "ok";
        case OZIMMU_BAD_ARG: return "bad argument";
        case OZIMMU_NONFINITE: return "non-finite input";
        case OZIMMU_HIP_ERROR: return "HIP runtime error";
        case OZIMMU_UNREACHABLE: return "tolerance unreachable";
        case OZIMMU_TOO_LARGE: return "problem too large for the static workspace";
    }
    return "unknown status";
}

size_t ozimmu_workspace_bytes(int m, int n, int k, int s)
{
    if (m < 0 || n < 0 || k < 0 || s < 1 || s > OZIMMU_MAX_SLICES) return 0;
    return carve(m, n, k, s, s).total;
}

size_t ozimmu_workspace_bytes2(int m, int n, int k, int sA, int sB, int all_products)
{
    if (m < 0 || n < 0 || k < 0 || sA < 1 || sA > OZIMMU_MAX_SLICES || sB < 1 || sB > OZIMMU_MAX_SLICES) return 0;
    return carve(m, n, k, sA, sB, all_products != 0).total;
}

size_t ozimmu_planes_bytes(char side, int rows, int cols, int s, int layout)
{
    if ((side != 'A' && side != 'B') || rows < 0 || cols < 0 || s < 1 || s > OZIMMU_MAX_SLICES) return 0;
    if (layout == OZIMMU_LAYOUT_PLAIN) return (size_t)s * rows * cols;
    if (layout != OZIMMU_LAYOUT_MFMA) return 0;
    const int R = side == 'A' ? rows : cols, K = side == 'A' ? cols : rows;
    return (size_t)s * round_up(R > 0 ? R : 1, kPad) * round_up(K > 0 ? K : 1, kPad);
}

size_t ozimmu_split_scratch_bytes(char side, int rows, int cols)
{
    if ((side != 'A' && side != 'B') || rows < 0 || cols < 0) return 0;
    const int nblk = side == 'A' ? rows : cols;
    return 256 + 8 * (size_t)(nblk > 0 ? nblk : 1);
}

static int kappas(int m, int n, int k, const double *A, int lda, const double *B, int ldb, double *kA, double *kB,
                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (bad_matrix(m, k, A, lda) || bad_matrix(k, n, B, ldb)) return OZIMMU_BAD_ARG;
    const Workspace w = carve(m, n, k, 1, 1);
    if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255)) return OZIMMU_BAD_ARG;
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    int rc = scales_into_workspace(w, ws, m, n, k, A, lda, B, ldb, true, 0, st);
    if (rc) return rc;
    unsigned long long host[3];
    OZ_TRY(hipMemcpyAsync(host, ws + w.off_header, sizeof(host), hipMemcpyDeviceToHost, st));
    OZ_TRY(hipStreamSynchronize(st));
    if (host[0] & 1ULL) return OZIMMU_NONFINITE;
    double ratioA, ratioB;
    std::memcpy(&ratioA, &host[1], 8);
    std::memcpy(&ratioB, &host[2], 8);
    *kA = 2.0 * ratioA;
    *kB = 2.0 * ratioB;
    return OZIMMU_OK;
}

int ozimmu_estimate_slices(int m, int n, int k, const double *A, int lda, const double *B, int ldb, double tol,
                           int *s_out, double *kappa, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!s_out || !(tol > 0.0)) return OZIMMU_BAD_ARG;
    double kA, kB;
    int rc = kappas(m, n, k, A, lda, B, ldb, &kA, &kB, workspace, workspace_bytes, stream);
    if (rc) return rc;
    if (kappa) { kappa[0] = kA; kappa[1] = kB; }
    // left-hand side of eq. (err-bound) with s_A = s_B = s, tried for s = 1, 2, ...
    for (int s = 1; s <= OZIMMU_MAX_SLICES; ++s) {
        const double lhs = std::ldexp(kA, -s * kSliceBits) + std::ldexp(kB, -s * kSliceBits);
        if (lhs <= tol) { *s_out = s; return OZIMMU_OK; }
    }
    *s_out = OZIMMU_MAX_SLICES;
    return OZIMMU_UNREACHABLE;
}

static int chi(int sA, int sB)
{
    const int sM = sA > sB ? sA : sB, sm = sA > sB ? sB : sA;
    return sm * (2 * sM - sm + 1) / 2;
}

int ozimmu_estimate_slices2(int m, int n, int k, const double *A, int lda, const double *B, int ldb, double tol,
                            int *sA_out, int *sB_out, double *kappa, void *workspace, size_t workspace_bytes,
                            void *stream)
{
    if (!sA_out || !sB_out || !(tol > 0.0)) return OZIMMU_BAD_ARG;
    double kA, kB;
    int rc = kappas(m, n, k, A, lda, B, ldb, &kA, &kB, workspace, workspace_bytes, stream);
    if (rc) return rc;
    if (kappa) { kappa[0] = kA; kappa[1] = kB; }
    // every (sA, sB) that meets eq. (err-bound); keep the one with the fewest products chi(sA, sB),
    // then the smaller sA + sB, then the smaller sA
    bool found = false;
    int bA = OZIMMU_MAX_SLICES, bB = OZIMMU_MAX_SLICES;
    for (int sA = 1; sA <= OZIMMU_MAX_SLICES; ++sA)
        for (int sB = 1; sB <= OZIMMU_MAX_SLICES; ++sB) {
            const double lhs = std::ldexp(kA, -sA * kSliceBits) + std::ldexp(kB, -sB * kSliceBits);
            if (!(lhs <= tol)) continue;
            const int c = chi(sA, sB), cb = chi(bA, bB);
            if (!found || c < cb || (c == cb && (sA + sB < bA + bB || (sA + sB == bA + bB && sA < bA)))) {
                found = true;
                bA = sA;
                bB = sB;
            }
        }
    *sA_out = bA;
    *sB_out = bB;
    return found ? OZIMMU_OK : OZIMMU_UNREACHABLE;
}

int ozimmu_split2(char side, int rows, int cols, const double *X, int ldx, int s, int splitting, int8_t *planes,
                  int32_t *exps, int layout, void *scratch, void *stream)
{
    if ((side != 'A' && side != 'B') || bad_matrix(rows, cols, X, ldx) || s < 1 || s > OZIMMU_MAX_SLICES ||
        (splitting != OZIMMU_SPLIT_TRUNCATE && splitting != OZIMMU_SPLIT_NEAREST) ||
        (layout != OZIMMU_LAYOUT_PLAIN && layout != OZIMMU_LAYOUT_MFMA) || !scratch || ((uintptr_t)scratch & 255))
        return OZIMMU_BAD_ARG;
    const int nblk = side == 'A' ? rows : cols;
    if (nblk > 0 && !exps) return OZIMMU_BAD_ARG;
    if (ozimmu_planes_bytes(side, rows, cols, s, layout) > 0 && !planes) return OZIMMU_BAD_ARG;
    hipStream_t st = (hipStream_t)stream;
    auto *hdr = (unsigned long long *)scratch;
    auto *maxbits = hdr + 32;
    OZ_TRY(launch_clear_header(hdr, st));
    OZ_TRY(launch_reduce(side, rows, cols, X, ldx, maxbits, nullptr, (unsigned int *)hdr, st));
    const bool nearest = splitting == OZIMMU_SPLIT_NEAREST;
    OZ_TRY(launch_finalize(maxbits, nullptr, exps, nblk, nblk, nullptr, nearest ? 1 : 0, st));
    OZ_TRY(launch_split(side, rows, cols, X, ldx, s, exps, planes, layout, nearest, st));
    return OZIMMU_OK;
}

int ozimmu_split(char side, int rows, int cols, const double *X, int ldx, int s, int8_t *planes, int32_t *exps,
                 int layout, void *scratch, void *stream)
{
    return ozimmu_split2(side, rows, cols, X, ldx, s, OZIMMU_SPLIT_TRUNCATE, planes, exps, layout, scratch, stream);
}

int ozimmu_max_level_diagonals(int k, int sA, int sB)
{
    if (k < 0 || sA < 1 || sA > OZIMMU_MAX_SLICES || sB < 1 || sB > OZIMMU_MAX_SLICES) return 0;
    // A diagonal holds at most min(sA, sB) products of k terms of magnitude at most 127^2.  In units of the
    // last diagonal of a level of Q diagonals, the level and each of its partial sums are integers below
    //     min(sA, sB) k 127^2 (1 + 2^7 + ... + 2^{7(Q-1)});
    // they are binary64 numbers while that stays below 2^53.
    const long long per_diag = (long long)(sA < sB ? sA : sB) * (k > 0 ? k : 1) * 127 * 127;   // < 2^51
    int Q = 0;
    long long geo = 0;                         // 1 + 2^7 + ... + 2^{7(Q-1)}
    while (Q < 8) {
        const long long next = geo * 128 + 1;
        if ((__int128)per_diag * next >= ((__int128)1 << 53)) break;
        geo = next;
        ++Q;
    }
    return Q;
}

static int dgemm_impl(int m, int n, int k, const double *A, int lda, const double *B, int ldb, double *C, int ldc,
                      int sA, int sB, bool all_products, int splitting, int Q, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    if (bad_matrix(m, k, A, lda) || bad_matrix(k, n, B, ldb) || bad_matrix(m, n, C, ldc) || sA < 1 ||
        sA > OZIMMU_MAX_SLICES || sB < 1 || sB > OZIMMU_MAX_SLICES ||
        (splitting != OZIMMU_SPLIT_TRUNCATE && splitting != OZIMMU_SPLIT_NEAREST) || Q < 1 ||
        Q > ozimmu_max_level_diagonals(k, sA, sB))
        return OZIMMU_BAD_ARG;
    const bool nearest = splitting == OZIMMU_SPLIT_NEAREST;
    const Workspace w = carve(m, n, k, sA, sB, all_products);
    if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255)) return OZIMMU_BAD_ARG;
    // exact conversion of a diagonal sum to binary64 needs s * k * 127^2 < 2^53: true for every int k
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    hipEvent_t *prof = (m > 0 && n > 0) ? prof_claim() : nullptr;
    prof_mark(prof, 0, st);
    auto *eA = (int32_t *)(ws + w.off_expA), *eB = (int32_t *)(ws + w.off_expB);
    auto *pA = (int8_t *)(ws + w.off_planesA), *pB = (int8_t *)(ws + w.off_planesB);
    // two launches for the maxima of both operands, one for their exponents and slices
    auto *maxA = (unsigned long long *)(ws + w.off_maxA), *maxB = (unsigned long long *)(ws + w.off_maxB);
    OZ_TRY(launch_scales_fused(m, n, k, A, lda, B, ldb, (unsigned long long *)(ws + w.off_header), maxA, maxB, eA, w.mp,
                               eB, w.np, nearest ? 1 : 0, m == 0 || n == 0, st));
    if (m == 0 || n == 0) return OZIMMU_OK;
    prof_mark(prof, 1, st);
    // (w.cA, w.cB: the counts the GEMM runs with -- counts that differ little run as equal ones, zero slices appended)
    OZ_TRY(launch_split_both(m, n, k, A, lda, B, ldb, sA, sB, w.cA, w.cB, maxA, maxB, eA, eB, pA, pB, nearest, st));
    prof_mark(prof, 2, st);
    const int cA = w.cA, cB = w.cB;
    if (w.path == kPathBlocks) {
        OZ_TRY(launch_gemm_blocks(m, n, w.kp, sA, sB, all_products, pA, pB, eA, eB, C, ldc,
                                  (long long *)(ws + w.off_totals), Q, st));
    } else if (w.path == kPathFused) {
        long long *totals = fused_single_block(cA, cB, k) ? nullptr : (long long *)(ws + w.off_totals);
        OZ_TRY(launch_gemm_fused(m, n, w.kp, cA, cB, all_products, pA, pB, eA, eB, C, ldc, nullptr, totals, Q, st));
    } else {
        const int dmax = all_products ? cA + cB : (cA > cB ? cA : cB) + 1;
        long long *totals = banded_totals_bytes(cA, cB, k) ? (long long *)(ws + w.off_totals) : nullptr;
        OZ_TRY(launch_gemm_banded(m, n, w.kp, cA, cB, dmax, pA, pB, eA, eB, C, ldc, totals, Q, st));
    }
    prof_mark(prof, 3, st);
    return OZIMMU_OK;
}

int ozimmu_dgemm(int m, int n, int k, const double *A, int lda, const double *B, int ldb, double *C, int ldc, int s,
                 void *workspace, size_t workspace_bytes, void *stream)
{
    return dgemm_impl(m, n, k, A, lda, B, ldb, C, ldc, s, s, false, OZIMMU_SPLIT_TRUNCATE, 1, workspace,
                      workspace_bytes, stream);
}

int ozimmu_dgemm2(int m, int n, int k, const double *A, int lda, const double *B, int ldb, double *C, int ldc,
                  int sA, int sB, int all_products, void *workspace, size_t workspace_bytes, void *stream)
{
    return dgemm_impl(m, n, k, A, lda, B, ldb, C, ldc, sA, sB, all_products != 0, OZIMMU_SPLIT_TRUNCATE, 1, workspace,
                      workspace_bytes, stream);
}

int ozimmu_dgemm3(int m, int n, int k, const double *A, int lda, const double *B, int ldb, double *C, int ldc,
                  int sA, int sB, int all_products, int splitting, int level_diagonals, void *workspace,
                  size_t workspace_bytes, void *stream)
{
    return dgemm_impl(m, n, k, A, lda, B, ldb, C, ldc, sA, sB, all_products != 0, splitting, level_diagonals,
                      workspace, workspace_bytes, stream);
}

// ---- the entry point that allocates nothing ----------------------------------------------------------------
// Its workspace is this file-scope device array: every GPU the library runs on holds one copy of it, at an address
// of its own, until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// address that kernels and copies take is looked up once per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[OZIMMU_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (null on failure)
void *static_workspace()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int ozimmu_dgemm_static(int m, int n, int k, const double *A, int lda, const double *B, int ldb, double *C, int ldc,
                        int s, void *stream)
{
    if (m < 0 || n < 0 || k < 0 || s < 1 || s > OZIMMU_MAX_SLICES) return OZIMMU_BAD_ARG;
    if (carve(m, n, k, s, s).total > (size_t)OZIMMU_STATIC_WORKSPACE_BYTES) return OZIMMU_TOO_LARGE;
    void *ws = static_workspace();
    if (!ws) return OZIMMU_HIP_ERROR;
    // every kernel of the path clears what it needs to find cleared (header, maxima, split-k totals) with fill
    // kernels of its own, so the contents the last call left behind do not matter
    return dgemm_impl(m, n, k, A, lda, B, ldb, C, ldc, s, s, false, OZIMMU_SPLIT_TRUNCATE, 1, ws,
                      (size_t)OZIMMU_STATIC_WORKSPACE_BYTES, stream);
}

int ozimmu_profile_start(int max_calls)
{
    std::lock_guard<std::mutex> lock(g_prof.mutex);
    if (max_calls < 1 || max_calls > 4096 || g_prof.on) return OZIMMU_BAD_ARG;
    g_prof.ev = new hipEvent_t[4 * (size_t)max_calls];
    for (int i = 0; i < 4 * max_calls; ++i)
        if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
            // give back what was created: the timer stays off and empty
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);
            delete[] g_prof.ev;
            g_prof.ev = nullptr;
            g_prof.capacity = g_prof.calls = 0;
            return OZIMMU_HIP_ERROR;
        }
    g_prof.capacity = max_calls;
    g_prof.calls = 0;
    g_prof.on = true;
    return OZIMMU_OK;
}

int ozimmu_profile_stop(int *calls, float *phase_ms)
{
    std::lock_guard<std::mutex> lock(g_prof.mutex);
    if (!g_prof.on || !calls || !phase_ms) return OZIMMU_BAD_ARG;
    g_prof.on = false;
    int rc = OZIMMU_OK;
    double sum[3] = {0, 0, 0};
    for (int c = 0; c < g_prof.calls; ++c) {
        hipEvent_t *e = g_prof.ev + 4 * c;
        if (hipEventSynchronize(e[3]) != hipSuccess) rc = OZIMMU_HIP_ERROR;
        for (int p = 0; p < 3 && rc == OZIMMU_OK; ++p) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, e[p], e[p + 1]) != hipSuccess) rc = OZIMMU_HIP_ERROR;
            sum[p] += ms;
        }
    }
    for (int i = 0; i < 4 * g_prof.capacity; ++i) (void)hipEventDestroy(g_prof.ev[i]);
    delete[] g_prof.ev;
    g_prof.ev = nullptr;
    *calls = g_prof.calls;
    for (int p = 0; p < 3; ++p) phase_ms[p] = g_prof.calls ? (float)(sum[p] / g_prof.calls) : 0.f;
    g_prof.capacity = g_prof.calls = 0;
    return rc;
}

int ozimmu_check(void *workspace, void *stream)
{
    if (!workspace) return OZIMMU_BAD_ARG;
    unsigned int flag = 0;
    hipStream_t st = (hipStream_t)stream;
    OZ_TRY(hipMemcpyAsync(&flag, workspace, sizeof(flag), hipMemcpyDeviceToHost, st));
    OZ_TRY(hipStreamSynchronize(st));
    return (flag & 1u) ? OZIMMU_NONFINITE : OZIMMU_OK;
}

int ozimmu_get_exponents(int m, int n, int k, int s, const void *workspace, int32_t *eA, int32_t *eB, void *stream)
{
    if (m < 0 || n < 0 || k < 0 || s < 1 || s > OZIMMU_MAX_SLICES || !workspace) return OZIMMU_BAD_ARG;
    const Workspace w = carve(m, n, k, s, s);
    hipStream_t st = (hipStream_t)stream;
    const char *ws = (const char *)workspace;
    if (eA && m) OZ_TRY(hipMemcpyAsync(eA, ws + w.off_expA, 4 * (size_t)m, hipMemcpyDeviceToDevice, st));
    if (eB && n) OZ_TRY(hipMemcpyAsync(eB, ws + w.off_expB, 4 * (size_t)n, hipMemcpyDeviceToDevice, st));
    return OZIMMU_OK;
}

const char *ozimmu_last_gemm_kernel(void) { return last_gemm_kernel(); }

int ozimmu_debug_panel_bytes(long long bytes)
{
    fused_set_panel_bytes(bytes);
    return OZIMMU_OK;
}

int ozimmu_debug_small_tile_limit(long long tiles)
{
    if (tiles < -1) return OZIMMU_BAD_ARG;
    fused_set_small_tile_limit(tiles);
    return OZIMMU_OK;
}

int ozimmu_debug_tile_choice(int choice)
{
    if (choice < 0 || choice > 2) return OZIMMU_BAD_ARG;
    fused16_set_tile_choice(choice);
    return OZIMMU_OK;
}

int ozimmu_debug_diagonals(int m, int n, int k, int s, const void *workspace, int32_t *D, void *stream)
{
    if (m <= 0 || n <= 0 || k < 0 || !workspace || !D || !fused_single_block(s, s, k)) return OZIMMU_BAD_ARG;
    const Workspace w = carve(m, n, k, s, s);
    const char *ws = (const char *)workspace;
    OZ_TRY(launch_gemm_fused(m, n, w.kp, s, s, false, (const int8_t *)(ws + w.off_planesA),
                             (const int8_t *)(ws + w.off_planesB),
                             nullptr, nullptr, nullptr, m, D, nullptr, 1, (hipStream_t)stream));
    return OZIMMU_OK;
}

int ozimmu_debug_slice_product(int m, int n, int k, int s, const void *workspace, int l, int h, int k0, int k1,
                               int32_t *P, void *stream)
{
    if (m <= 0 || n <= 0 || k < 0 || s < 1 || s > OZIMMU_MAX_SLICES || !workspace || !P || l < 1 || l > s || h < 1 ||
        h > s || k0 < 0 || k1 < k0 || k1 > k || (k0 % kFrag) != 0 || (long long)(k1 - k0) > kMaxInt32K)
        return OZIMMU_BAD_ARG;
    const Workspace w = carve(m, n, k, s, s);
    const char *ws = (const char *)workspace;
    // the planes are zero beyond k, so the last (partial) fragment may be read whole
    const int kb_begin = k0 / kFrag, kb_end = (k1 + kFrag - 1) / kFrag;
    if (k1 != k && (k1 % kFrag) != 0) return OZIMMU_BAD_ARG;
    OZ_TRY(launch_gemm_generic(m, n, w.kp, s, (const int8_t *)(ws + w.off_planesA),
                               (const int8_t *)(ws + w.off_planesB), nullptr, nullptr, nullptr, m, l, h, kb_begin,
                               kb_end, P, (hipStream_t)stream));
    return OZIMMU_OK;
}

}  // extern "C"
