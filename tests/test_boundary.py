"""CPU-side checks of the C-ABI boundary: the library builds/loads and exports every symbol the
public header declares; argument validation that needs no GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ozimmu.h")              # the method's calls
BENCH_HEADER = os.path.join(ROOT, "include", "ozimmu_bench.h")  # benchmark aids and test hooks


@pytest.fixture(scope="module")
def handle():
    from paper_2506_11277_amd import ozimmu
    if not os.path.exists(ozimmu.LIB_PATH):
        from paper_2506_11277_amd import build
        build.build_lib()
    return ozimmu.lib()


def declared_functions(headers=(HEADER, BENCH_HEADER)):
    names = set()
    for header in headers:
        text = open(header).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ozimmu_\w+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_three_named_entry_points():
    names = declared_functions()
    for required in ("ozimmu_estimate_slices", "ozimmu_split", "ozimmu_dgemm"):
        assert required in names


def test_the_method_header_holds_no_benchmark_aid_or_test_hook():
    for name in declared_functions((HEADER,)):
        assert not re.search(r"debug|profile|measure|calibration", name), name
    assert "ozimmu_dgemm_static" in declared_functions((HEADER,))
    aids = declared_functions((BENCH_HEADER,))
    assert "ozimmu_profile_start" in aids and "ozimmu_debug_diagonals" in aids and "ozimmu_calibration_copy" in aids


def test_library_exports_every_declared_symbol(handle):
    raw = ctypes.CDLL(handle._name)
    for name in declared_functions():
        assert hasattr(raw, name), name


def test_binding_covers_every_declared_symbol():
    from paper_2506_11277_amd import ozimmu
    assert sorted(ozimmu._SIGNATURES) == declared_functions()


def test_status_strings(handle):
    assert handle.ozimmu_status_string(0) == b"ok"
    assert handle.ozimmu_status_string(2) == b"non-finite input"
    assert handle.ozimmu_status_string(99) == b"unknown status"


def test_size_queries_and_argument_validation_without_gpu(handle):
    # workspace grows with s and covers the padded planes
    w3 = handle.ozimmu_workspace_bytes(128, 128, 128, 3)
    w4 = handle.ozimmu_workspace_bytes(128, 128, 128, 4)
    assert w4 - w3 == 2 * 128 * 128
    assert handle.ozimmu_workspace_bytes(100, 90, 70, 2) == handle.ozimmu_workspace_bytes(128, 128, 128, 2)
    assert handle.ozimmu_workspace_bytes(8192, 8192, 8192, 7) >= 2 * 7 * 8192 * 8192
    assert handle.ozimmu_workspace_bytes(-1, 1, 1, 1) == 0
    assert handle.ozimmu_workspace_bytes(1, 1, 1, 0) == 0
    assert handle.ozimmu_workspace_bytes(1, 1, 1, 33) == 0
    assert handle.ozimmu_planes_bytes(b"A", 100, 200, 3, 0) == 3 * 100 * 200
    assert handle.ozimmu_planes_bytes(b"A", 100, 200, 3, 1) == 3 * 128 * 256
    assert handle.ozimmu_planes_bytes(b"B", 100, 200, 3, 1) == 3 * 256 * 128
    assert handle.ozimmu_planes_bytes(b"C", 100, 200, 3, 1) == 0
    # invalid arguments are rejected before any HIP call is made
    ws = ctypes.c_void_p(256)
    fake = ctypes.c_void_p(4096)
    assert handle.ozimmu_dgemm(4, 4, 4, fake, 3, fake, 4, fake, 4, 2, ws, 1 << 30, None) == 1      # lda < m
    assert handle.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 0, ws, 1 << 30, None) == 1      # s < 1
    assert handle.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 33, ws, 1 << 30, None) == 1     # s > max
    assert handle.ozimmu_dgemm(4, 4, 4, None, 4, fake, 4, fake, 4, 2, ws, 1 << 30, None) == 1      # null A
    assert handle.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 2, ws, 16, None) == 1           # workspace too small
    assert handle.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 2, ctypes.c_void_p(264), 1 << 30, None) == 1
    assert handle.ozimmu_dgemm(-1, 4, 4, fake, 4, fake, 4, fake, 4, 2, ws, 1 << 30, None) == 1
    s = ctypes.c_int(0)
    assert handle.ozimmu_estimate_slices(4, 4, 4, fake, 4, fake, 4, 0.0, ctypes.byref(s), None, ws, 1 << 30, None) == 1
    assert handle.ozimmu_estimate_slices(4, 4, 4, fake, 4, fake, 4, float("nan"), ctypes.byref(s), None, ws, 1 << 30,
                                         None) == 1
    assert handle.ozimmu_split(b"X", 4, 4, fake, 4, 2, fake, fake, 0, ws, None) == 1
    assert handle.ozimmu_split(b"A", 4, 4, fake, 4, 2, fake, fake, 7, ws, None) == 1


def test_workspace_accounts_for_nearly_equal_slice_counts_run_as_equal(handle):
    # counts that differ little run as equal counts with zero slices appended to the short operand: the workspace
    # is then that of the equal counts; counts that differ much keep planes of their own sizes
    w = lambda sA, sB, allp=0: handle.ozimmu_workspace_bytes2(256, 256, 256, sA, sB, allp)
    assert w(7, 8) == w(8, 8) == w(8, 7)
    assert w(17, 18) == w(18, 18) and w(19, 20) == w(20, 20)
    assert w(5, 8) == w(8, 8)
    assert w(8, 8) - w(4, 8) == 4 * 256 * 256           # (4, 8) is not padded: four slices less of A
    assert w(12, 12) - w(9, 12) == 3 * 256 * 256
    assert w(5, 4, 1) == w(5, 5, 1)                     # all products of nearly equal counts
    assert w(5, 2, 1) < w(5, 5, 1)
    # beyond the fused kernels the products are formed group of slices by group of slices: the planes hold whole
    # groups (here of 8 and of 7 slices), the same for every count that rounds up to them
    assert w(25, 31) == w(31, 31) == w(32, 32)
    assert w(21, 21) - w(20, 20) >= 2 * 256 * 256       # one more slice per operand, plus the totals of the blocks
    assert w(20, 7) == w(21, 7)                         # (20, 7): three groups of 7 times one group of 7


def test_level_size_limit_and_variant_argument_validation_without_gpu(handle):
    # largest Q with  min(sA, sB) k 127^2 (1 + 2^7 + ... + 2^{7(Q-1)}) < 2^53, recomputed with Python integers
    for k in (0, 1, 64, 128, 1000, 8192, 2 ** 17, 2 ** 18, 2 ** 31 - 1):
        for sA, sB in ((1, 1), (7, 7), (4, 12), (12, 4), (32, 32), (32, 1)):
            per = min(sA, sB) * max(k, 1) * 127 * 127
            want = max(q for q in range(0, 9) if q == 0 or per * sum(128 ** i for i in range(q)) < 2 ** 53)
            assert handle.ozimmu_max_level_diagonals(k, sA, sB) == want, (k, sA, sB)
            assert want >= 1
    assert handle.ozimmu_max_level_diagonals(8192, 7, 7) == 4
    assert handle.ozimmu_max_level_diagonals(2 ** 17, 7, 7) == 3      # the paper's value for a full int32 accumulator
    assert handle.ozimmu_max_level_diagonals(-1, 7, 7) == 0
    assert handle.ozimmu_max_level_diagonals(8, 0, 7) == 0 and handle.ozimmu_max_level_diagonals(8, 7, 33) == 0
    ws = ctypes.c_void_p(256)
    fake = ctypes.c_void_p(4096)
    args = (4, 4, 4, fake, 4, fake, 4, fake, 4)
    assert handle.ozimmu_dgemm3(*args, 2, 2, 0, 0, 0, ws, 1 << 30, None) == 1      # Q < 1
    assert handle.ozimmu_dgemm3(*args, 2, 2, 0, 0, 7, ws, 1 << 30, None) == 1      # Q beyond the exact range
    assert handle.ozimmu_dgemm3(*args, 2, 2, 0, 2, 1, ws, 1 << 30, None) == 1      # unknown splitting
    assert handle.ozimmu_dgemm3(*args, 2, 2, 0, 1, 1, ws, 16, None) == 1           # workspace too small
    assert handle.ozimmu_split2(b"A", 4, 4, fake, 4, 2, 5, fake, fake, 0, ws, None) == 1
