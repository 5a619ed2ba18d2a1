"""Thin Python binding of libozimmu (C ABI declared in include/ozimmu.h).

Argument marshalling only: every step of the method runs in the HIP kernels of the shared
library.  PyTorch provides device memory and the current stream, nothing else.  There is no
CPU fallback: if the library is missing, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libozimmu.so")

OK, BAD_ARG, NONFINITE, HIP_ERROR, UNREACHABLE, TOO_LARGE = 0, 1, 2, 3, 4, 5
STATIC_WORKSPACE_BYTES = 64 << 20
MAX_SLICES = 32
LAYOUT_PLAIN, LAYOUT_MFMA = 0, 1
SPLIT_TRUNCATE, SPLIT_NEAREST = 0, 1

_c = ctypes
_SIGNATURES = {
    "ozimmu_status_string": (_c.c_char_p, [_c.c_int]),
    "ozimmu_workspace_bytes": (_c.c_size_t, [_c.c_int] * 4),
    "ozimmu_planes_bytes": (_c.c_size_t, [_c.c_char, _c.c_int, _c.c_int, _c.c_int, _c.c_int]),
    "ozimmu_split_scratch_bytes": (_c.c_size_t, [_c.c_char, _c.c_int, _c.c_int]),
    "ozimmu_estimate_slices": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_int,
                                          _c.c_double, _c.POINTER(_c.c_int), _c.POINTER(_c.c_double), _c.c_void_p,
                                          _c.c_size_t, _c.c_void_p]),
    "ozimmu_split": (_c.c_int, [_c.c_char, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int, _c.c_int, _c.c_void_p,
                                _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "ozimmu_dgemm": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_int,
                                _c.c_void_p, _c.c_int, _c.c_int, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "ozimmu_dgemm_static": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_int,
                                       _c.c_void_p, _c.c_int, _c.c_int, _c.c_void_p]),
    "ozimmu_workspace_bytes2": (_c.c_size_t, [_c.c_int] * 6),
    "ozimmu_dgemm2": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_int,
                                 _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_size_t,
                                 _c.c_void_p]),
    "ozimmu_split2": (_c.c_int, [_c.c_char, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p,
                                 _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "ozimmu_max_level_diagonals": (_c.c_int, [_c.c_int] * 3),
    "ozimmu_dgemm3": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_int,
                                 _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                 _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "ozimmu_estimate_slices2": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_int,
                                           _c.c_double, _c.POINTER(_c.c_int), _c.POINTER(_c.c_int),
                                           _c.POINTER(_c.c_double), _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "ozimmu_check": (_c.c_int, [_c.c_void_p, _c.c_void_p]),
    "ozimmu_get_exponents": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p,
                                        _c.c_void_p, _c.c_void_p]),
    "ozimmu_last_gemm_kernel": (_c.c_char_p, []),
    "ozimmu_profile_start": (_c.c_int, [_c.c_int]),
    "ozimmu_profile_stop": (_c.c_int, [_c.POINTER(_c.c_int), _c.POINTER(_c.c_float)]),
    "ozimmu_calibration_copy": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "ozimmu_measure_int8_ceiling2": (_c.c_int, [_c.c_int, _c.c_int, _c.c_void_p, _c.POINTER(_c.c_float), _c.c_void_p]),
    "ozimmu_measure_int8_with_traffic": (_c.c_int, [_c.c_int, _c.c_int, _c.c_void_p, _c.c_size_t, _c.c_void_p,
                                                    _c.POINTER(_c.c_float), _c.c_void_p]),
    "ozimmu_measure_int8_ceiling": (_c.c_int, [_c.c_int, _c.c_void_p, _c.POINTER(_c.c_float), _c.c_void_p]),
    "ozimmu_debug_small_tile_limit": (_c.c_int, [_c.c_longlong]),
    "ozimmu_debug_tile_choice": (_c.c_int, [_c.c_int]),
    "ozimmu_debug_panel_bytes": (_c.c_int, [_c.c_longlong]),
    "ozimmu_debug_diagonals": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p,
                                          _c.c_void_p]),
    "ozimmu_debug_slice_product": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_int,
                                              _c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p]),
}

_lib = None


class OzimmuError(RuntimeError):
    def __init__(self, code, what=""):
        name = lib().ozimmu_status_string(code).decode() if _lib is not None else str(code)
        super().__init__(f"{what}: ozimmu status {code} ({name})")
        self.code = code


def lib():
    """The loaded shared library.  Raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with paper_2506_11277_amd/build.py "
                              f"(or __graft_entry__.build()); there is no CPU fallback")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _colmajor_ld(X, what):
    """Leading dimension of a column-major 2-D float64 device tensor (stride(0) == 1)."""
    if X.dim() != 2 or X.dtype != torch.float64 or not X.is_cuda:
        raise ValueError(f"{what}: 2-D float64 CUDA tensor expected")
    rows, cols = X.shape
    if rows <= 1 and cols <= 1:
        return max(1, rows)
    if rows > 1 and X.stride(0) != 1:
        raise ValueError(f"{what}: column-major tensor expected (stride(0) == 1); use ozimmu.colmajor_empty / "
                         f"x.t().contiguous().t()")
    ld = X.stride(1) if cols > 1 else max(1, rows)
    if ld < max(1, rows):
        raise ValueError(f"{what}: leading dimension {ld} smaller than {rows}")
    return ld


def colmajor_empty(rows, cols, device="cuda", dtype=torch.float64):
    """An uninitialised rows-by-cols tensor stored column-major."""
    return torch.empty((cols, rows), device=device, dtype=dtype).t()


def to_colmajor(x_host, device="cuda"):
    """Upload a numpy / CPU array as a column-major device tensor (layout change on the host side only)."""
    t = torch.as_tensor(x_host, dtype=torch.float64)
    out = colmajor_empty(t.shape[0], t.shape[1], device=device)
    out.copy_(t)
    return out


def workspace_bytes(m, n, k, s):
    b = lib().ozimmu_workspace_bytes(m, n, k, s)
    if b == 0:
        raise OzimmuError(BAD_ARG, "workspace_bytes")
    return b


def alloc_workspace(m, n, k, s, device="cuda"):
    return torch.empty(workspace_bytes(m, n, k, s), dtype=torch.uint8, device=device)


def check(workspace):
    """Synchronises; raises OzimmuError(NONFINITE) if the last call on this workspace met NaN/Inf."""
    rc = lib().ozimmu_check(workspace.data_ptr(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "check")


def dgemm(A, B, s, C=None, workspace=None, check_finite=False):
    """C = A @ B through s int8 slices.  A (m x k), B (k x n): column-major float64 CUDA tensors.

    The call is asynchronous and does not look at the non-finite flag: if A or B hold a NaN or an Inf, C is
    unspecified until check(workspace) has been called (it raises OzimmuError(NONFINITE)); check_finite=True
    does that here, at the price of a synchronisation.  Pass your own workspace to be able to call check()."""
    lda = _colmajor_ld(A, "A")
    ldb = _colmajor_ld(B, "B")
    m, k = A.shape
    k2, n = B.shape
    if k != k2:
        raise ValueError("inner dimensions differ")
    if C is None:
        C = colmajor_empty(m, n, device=A.device)
    ldc = _colmajor_ld(C, "C")
    if tuple(C.shape) != (m, n):
        raise ValueError("C has the wrong shape")
    if workspace is None:
        workspace = alloc_workspace(m, n, k, s, device=A.device)
    rc = lib().ozimmu_dgemm(m, n, k, A.data_ptr(), lda, B.data_ptr(), ldb, C.data_ptr(), ldc, s,
                            workspace.data_ptr(), workspace.numel(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "dgemm")
    if check_finite:
        check(workspace)
    return C


def dgemm_static(A, B, s, C):
    """dgemm through the library's static workspace: the call allocates nothing, so C must be given.
    Raises OzimmuError(TOO_LARGE) beyond STATIC_WORKSPACE_BYTES of workspace."""
    lda = _colmajor_ld(A, "A")
    ldb = _colmajor_ld(B, "B")
    ldc = _colmajor_ld(C, "C")
    m, k = A.shape
    k2, n = B.shape
    if k != k2 or tuple(C.shape) != (m, n):
        raise ValueError("shapes do not match")
    rc = lib().ozimmu_dgemm_static(m, n, k, A.data_ptr(), lda, B.data_ptr(), ldb, C.data_ptr(), ldc, s, _stream())
    if rc != OK:
        raise OzimmuError(rc, "dgemm_static")
    return C


def dgemm2(A, B, sA, sB, all_products=False, C=None, workspace=None, check_finite=False):
    """C = A @ B with sA slices of A and sB slices of B.  As for dgemm, C is unspecified for non-finite input
    until check(workspace) has passed (check_finite=True calls it)."""
    lda = _colmajor_ld(A, "A")
    ldb = _colmajor_ld(B, "B")
    m, k = A.shape
    k2, n = B.shape
    if k != k2:
        raise ValueError("inner dimensions differ")
    if C is None:
        C = colmajor_empty(m, n, device=A.device)
    ldc = _colmajor_ld(C, "C")
    if tuple(C.shape) != (m, n):
        raise ValueError("C has the wrong shape")
    if workspace is None:
        nbytes = lib().ozimmu_workspace_bytes2(m, n, k, sA, sB, int(all_products))
        if nbytes == 0:
            raise OzimmuError(BAD_ARG, "workspace_bytes2")
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=A.device)
    rc = lib().ozimmu_dgemm2(m, n, k, A.data_ptr(), lda, B.data_ptr(), ldb, C.data_ptr(), ldc, sA, sB,
                             int(all_products), workspace.data_ptr(), workspace.numel(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "dgemm2")
    if check_finite:
        check(workspace)
    return C


def max_level_diagonals(k, sA, sB):
    return lib().ozimmu_max_level_diagonals(k, sA, sB)


def dgemm3(A, B, sA, sB, all_products=False, splitting=SPLIT_TRUNCATE, level_diagonals=1, C=None, workspace=None,
           check_finite=False):
    """dgemm2 with the slicing (truncation / round-to-nearest) and the level size of the accumulation chosen.
    As for dgemm, C is unspecified for non-finite input until check(workspace) has passed."""
    lda = _colmajor_ld(A, "A")
    ldb = _colmajor_ld(B, "B")
    m, k = A.shape
    k2, n = B.shape
    if k != k2:
        raise ValueError("inner dimensions differ")
    if C is None:
        C = colmajor_empty(m, n, device=A.device)
    ldc = _colmajor_ld(C, "C")
    if tuple(C.shape) != (m, n):
        raise ValueError("C has the wrong shape")
    if workspace is None:
        nbytes = lib().ozimmu_workspace_bytes2(m, n, k, sA, sB, int(all_products))
        if nbytes == 0:
            raise OzimmuError(BAD_ARG, "workspace_bytes2")
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=A.device)
    rc = lib().ozimmu_dgemm3(m, n, k, A.data_ptr(), lda, B.data_ptr(), ldb, C.data_ptr(), ldc, sA, sB,
                             int(all_products), int(splitting), int(level_diagonals), workspace.data_ptr(),
                             workspace.numel(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "dgemm3")
    if check_finite:
        check(workspace)
    return C


def estimate_slices2(A, B, tol, workspace=None):
    """Returns (sA, sB, status, kappa_A, kappa_B): the cheapest pair of slice counts meeting tol."""
    lda = _colmajor_ld(A, "A")
    ldb = _colmajor_ld(B, "B")
    m, k = A.shape
    k2, n = B.shape
    if k != k2:
        raise ValueError("inner dimensions differ")
    if workspace is None:
        workspace = alloc_workspace(m, n, k, 1, device=A.device)
    sA = ctypes.c_int(0)
    sB = ctypes.c_int(0)
    kap = (ctypes.c_double * 2)()
    rc = lib().ozimmu_estimate_slices2(m, n, k, A.data_ptr(), lda, B.data_ptr(), ldb, float(tol), ctypes.byref(sA),
                                       ctypes.byref(sB), kap, workspace.data_ptr(), workspace.numel(), _stream())
    if rc not in (OK, UNREACHABLE):
        raise OzimmuError(rc, "estimate_slices2")
    return sA.value, sB.value, rc, kap[0], kap[1]


def estimate_slices(A, B, tol, workspace=None):
    """Returns (s, status, kappa_A, kappa_B); status is OK or UNREACHABLE.  Synchronises."""
    lda = _colmajor_ld(A, "A")
    ldb = _colmajor_ld(B, "B")
    m, k = A.shape
    k2, n = B.shape
    if k != k2:
        raise ValueError("inner dimensions differ")
    if workspace is None:
        workspace = alloc_workspace(m, n, k, 1, device=A.device)
    s = ctypes.c_int(0)
    kap = (ctypes.c_double * 2)()
    rc = lib().ozimmu_estimate_slices(m, n, k, A.data_ptr(), lda, B.data_ptr(), ldb, float(tol), ctypes.byref(s), kap,
                                      workspace.data_ptr(), workspace.numel(), _stream())
    if rc not in (OK, UNREACHABLE):
        raise OzimmuError(rc, "estimate_slices")
    return s.value, rc, kap[0], kap[1]


def split(side, X, s, layout=LAYOUT_PLAIN, splitting=SPLIT_TRUNCATE):
    """Returns (planes, exps): int8 byte buffer in the requested layout and int32 scale exponents."""
    ldx = _colmajor_ld(X, "X")
    rows, cols = X.shape
    nblk = rows if side == "A" else cols
    side_c = side.encode()
    nbytes = lib().ozimmu_planes_bytes(side_c, rows, cols, s, layout)
    planes = torch.empty(max(nbytes, 1), dtype=torch.int8, device=X.device)
    exps = torch.empty(max(nblk, 1), dtype=torch.int32, device=X.device)
    scratch = torch.empty(lib().ozimmu_split_scratch_bytes(side_c, rows, cols), dtype=torch.uint8, device=X.device)
    if splitting == SPLIT_TRUNCATE:
        rc = lib().ozimmu_split(side_c, rows, cols, X.data_ptr(), ldx, s, planes.data_ptr(), exps.data_ptr(), layout,
                                scratch.data_ptr(), _stream())
    else:
        rc = lib().ozimmu_split2(side_c, rows, cols, X.data_ptr(), ldx, s, int(splitting), planes.data_ptr(),
                                 exps.data_ptr(), layout, scratch.data_ptr(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "split")
    rc = lib().ozimmu_check(scratch.data_ptr(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "split")
    return planes[:nbytes], exps[:nblk]


def get_exponents(m, n, k, s, workspace):
    eA = torch.empty(max(m, 1), dtype=torch.int32, device=workspace.device)
    eB = torch.empty(max(n, 1), dtype=torch.int32, device=workspace.device)
    rc = lib().ozimmu_get_exponents(m, n, k, s, workspace.data_ptr(), eA.data_ptr(), eB.data_ptr(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "get_exponents")
    return eA[:m], eB[:n]


def profile_start(max_calls):
    rc = lib().ozimmu_profile_start(max_calls)
    if rc != OK:
        raise OzimmuError(rc, "profile_start")


def profile_stop():
    """Returns (calls, {"scales": ms, "split": ms, "gemm": ms}) averaged over the profiled dgemm calls."""
    calls = ctypes.c_int(0)
    ms = (ctypes.c_float * 3)()
    rc = lib().ozimmu_profile_stop(ctypes.byref(calls), ms)
    if rc != OK:
        raise OzimmuError(rc, "profile_stop")
    return calls.value, {"scales": ms[0], "split": ms[1], "gemm": ms[2]}


def last_gemm_kernel():
    """Name and tile of the GEMM kernel this thread's last dgemm* call launched."""
    return lib().ozimmu_last_gemm_kernel().decode()


def calibration_copy(dst, src):
    """Plain copy kernel of known traffic (src.nbytes read, the same written) for scaling memory counters."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("calibration_copy: sizes differ")
    rc = lib().ozimmu_calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream())
    if rc != OK:
        raise OzimmuError(rc, "calibration_copy")


def measure_int8_ceiling(random_operands, shape16=False):
    """Sustained int8 MFMA rate (TOP/s) of a register-only loop on the current device (32x32x32 or 16x16x64);
    random_operands: 0 constants, 1 one random operand pair, 2 a register tile of random operands."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    tops = ctypes.c_float(0.0)
    rc = lib().ozimmu_measure_int8_ceiling2(int(random_operands), int(bool(shape16)), sink.data_ptr(),
                                            ctypes.byref(tops), _stream())
    if rc != OK:
        raise OzimmuError(rc, "measure_int8_ceiling")
    return tops.value


def measure_int8_with_traffic(lds_reads, dma_copies_per_32):
    """Sustained rate (TOP/s) of the 16x16x64 loop on random operands with LDS re-reads and LDS-DMA copies from an
    L2-resident buffer going on beside it (the GEMM kernel for 7 slices: 4 reads per 16, 3 copies per 32)."""
    src = torch.randint(-127, 128, (4 << 20,), dtype=torch.int8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    tops = ctypes.c_float(0.0)
    rc = lib().ozimmu_measure_int8_with_traffic(int(lds_reads), int(dma_copies_per_32), src.data_ptr(), src.numel(),
                                                sink.data_ptr(), ctypes.byref(tops), _stream())
    if rc != OK:
        raise OzimmuError(rc, "measure_int8_with_traffic")
    return tops.value


def debug_small_tile_limit(tiles):
    """Test hook: tile-count threshold below which equal slice counts up to 12 use the 64 x 64 tile (0: never;
    -1, the default: wherever the small tile finishes sooner by the library's cost rule)."""
    rc = lib().ozimmu_debug_small_tile_limit(int(tiles))
    if rc != OK:
        raise OzimmuError(rc, "debug_small_tile_limit")


def debug_tile_choice(choice):
    """Test hook: 2 ... 6 slices on the tabulated tile (1), on the alternative tile (2), or chosen by size (0)."""
    rc = lib().ozimmu_debug_tile_choice(int(choice))
    if rc != OK:
        raise OzimmuError(rc, "debug_tile_choice")


def debug_panel_bytes(nbytes):
    """Test hook: bytes of split-k totals per column panel of C (<= 0: no panels); set before sizing workspaces."""
    lib().ozimmu_debug_panel_bytes(int(nbytes))


def debug_diagonals(m, n, k, s, workspace):
    """int32 tensor [s, n, m]: entry [d-2, j, i] = sum over l+h=d of (A_(l) B^(h))[i, j]."""
    D = torch.empty((s, n, m), dtype=torch.int32, device=workspace.device)
    rc = lib().ozimmu_debug_diagonals(m, n, k, s, workspace.data_ptr(), D.data_ptr(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "debug_diagonals")
    return D


def debug_slice_product(m, n, k, s, workspace, l, h, k0=0, k1=None):
    """int32 tensor [n, m]: entry [j, i] = sum_{k0 <= kk < k1} A_(l)[i,kk] B^(h)[kk,j]."""
    if k1 is None:
        k1 = k
    P = torch.empty((n, m), dtype=torch.int32, device=workspace.device)
    rc = lib().ozimmu_debug_slice_product(m, n, k, s, workspace.data_ptr(), l, h, k0, k1, P.data_ptr(), _stream())
    if rc != OK:
        raise OzimmuError(rc, "debug_slice_product")
    return P
