"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on
the same seeded inputs.  Integer stages (exponents, slices, slice products, diagonal sums) must
agree bit for bit; C must agree to 1e-15 relative (the stated bar) and is also required to be
bit-identical (the goal: the only roundings are the ordered binary64 additions, replicated)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import oracle
from paper_2506_11277_amd import ozimmu, workloads

REL_BAR = 1e-15


@pytest.fixture(params=["tabulated tile", "small tile"])
def tile_choice(request):
    """Small problems would all run the 64 x 64 tile; tests that take this fixture run once with that choice
    switched off (the kernels tabulated per slice count) and once with it on."""
    ozimmu.debug_small_tile_limit(0 if request.param == "tabulated tile" else 256)
    ozimmu.debug_tile_choice(1)
    yield request.param
    ozimmu.debug_small_tile_limit(-1)
    ozimmu.debug_tile_choice(0)


@pytest.fixture(autouse=True)
def tabulated_tile_by_default(request):
    """Every other test runs the kernels tabulated per slice count (neither the 64 x 64 tile nor the alternative
    tiles of 2, 3 and 4 slices, which the library would take at these sizes)."""
    if "tile_choice" not in request.fixturenames:
        ozimmu.debug_small_tile_limit(0)
        ozimmu.debug_tile_choice(1)
        yield
        ozimmu.debug_small_tile_limit(-1)
        ozimmu.debug_tile_choice(0)
    else:
        yield


def dev(X):
    return ozimmu.to_colmajor(np.asarray(X, dtype=np.float64))


def host(T):
    return T.cpu().numpy()


def untile(buf, R, K, s):
    """MFMA layout (include/ozimmu.h) -> [s, R, K]; also returns the padded array for zero checks."""
    Rp, Kp = -(-max(R, 1) // 128) * 128, -(-max(K, 1) // 128) * 128
    a = np.asarray(buf, dtype=np.int8).reshape(Rp // 32, Kp // 32, s, 2, 32, 16)   # rb, kb, l, khalf, r, kbyte
    full = a.transpose(2, 0, 4, 1, 3, 5).reshape(s, Rp, Kp)
    return full[:, :R, :K], full


def rel_err(C, Cref):
    denom = np.abs(Cref)
    diff = np.abs(C - Cref)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.where(diff == 0, 0.0, diff / denom)
    return float(np.max(r)) if r.size else 0.0


def assert_c_matches(C, Cref, what=""):
    r = rel_err(C, Cref)
    assert r <= REL_BAR, f"{what}: max relative difference {r:.3e} above the 1e-15 bar"
    assert np.array_equal(C, Cref), f"{what}: within the bar (rel {r:.3e}) but not bit-identical"


def inputs(kind, m, n, k, seed):
    if kind == "uniform":
        return workloads.uniform(m, n, k, seed)
    if kind == "lognormal":
        return workloads.lognormal(m, n, k, 2.0, seed)
    if kind == "pow2":
        return workloads.pow2_scaled(m, n, k, 30, seed)
    if kind == "special":
        A, B = workloads.lognormal(m, n, k, 4.0, seed)
        rng = np.random.default_rng(seed)
        if m > 2:
            A[1, :] = 0.0                       # zero row
        if n > 2:
            B[:, 2] = 0.0                       # zero column
        A[rng.random(A.shape) < 0.1] = 0.0
        B[rng.random(B.shape) < 0.1] = -0.0     # negative zeros
        if m > 3:
            A[3, :] *= 2.0 ** -1040             # subnormal row
        if m > 4 and k > 1:
            A[4, :] = 0.0
            A[4, k // 2] = 2.0 ** -3            # single power of two
        if n > 5:
            B[:, 5] *= 2.0 ** 900               # huge column
        return A, B
    raise ValueError(kind)


SHAPES = [(1, 1, 1), (5, 3, 2), (33, 70, 17), (128, 128, 128), (100, 90, 70), (129, 65, 33), (257, 130, 300)]


# ----------------------------------------------------------------------------- scales + slices

@pytest.mark.parametrize("kind", ["uniform", "lognormal", "pow2", "special"])
@pytest.mark.parametrize("m,n,k", SHAPES)
@pytest.mark.parametrize("s", [1, 3, 7, 12, 32])
def test_split_plain_layout_bit_exact(kind, m, n, k, s):
    A, B = inputs(kind, m, n, k, 11)
    for side, X in (("A", A), ("B", B)):
        want_planes, want_e = oracle.split(side, X, s)
        planes, e = ozimmu.split(side, dev(X), s, ozimmu.LAYOUT_PLAIN)
        rows, cols = X.shape
        got = host(planes).reshape(s, cols, rows).transpose(0, 2, 1)
        assert np.array_equal(host(e), want_e), (side, "exponents")
        assert np.array_equal(got, want_planes), (side, "slices")


@pytest.mark.parametrize("kind", ["uniform", "special"])
@pytest.mark.parametrize("m,n,k", SHAPES)
@pytest.mark.parametrize("s", [1, 7, 9, 17, 32])
def test_split_mfma_layout_bit_exact_and_zero_padded(kind, m, n, k, s):
    A, B = inputs(kind, m, n, k, 12)
    for side, X in (("A", A), ("B", B)):
        want_planes, want_e = oracle.split(side, X, s)
        planes, e = ozimmu.split(side, dev(X), s, ozimmu.LAYOUT_MFMA)
        R, K = (X.shape[0], X.shape[1]) if side == "A" else (X.shape[1], X.shape[0])
        got, full = untile(host(planes), R, K, s)
        want = want_planes if side == "A" else want_planes.transpose(0, 2, 1)
        assert np.array_equal(host(e), want_e)
        assert np.array_equal(got, want), side
        assert not full[:, R:, :].any() and not full[:, :, K:].any(), "padding must be zero"


def test_split_with_leading_dimension_larger_than_rows():
    A, B = workloads.lognormal(70, 50, 90, 1.0, 3)
    big = ozimmu.colmajor_empty(100, 90)
    big.fill_(7.0)
    big[:70, :] = torch.as_tensor(A)
    view = big[:70, :]
    assert view.stride(1) == 100
    planes, e = ozimmu.split("A", view, 5, ozimmu.LAYOUT_PLAIN)
    want_planes, want_e = oracle.split("A", A, 5)
    assert np.array_equal(host(e), want_e)
    assert np.array_equal(host(planes).reshape(5, 90, 70).transpose(0, 2, 1), want_planes)


# ----------------------------------------------------------------------------- integer products

@pytest.mark.parametrize("m,n,k", [(33, 70, 17), (100, 90, 70), (200, 130, 1000)])
def test_int32_slice_products_bit_exact(m, n, k):
    s = 5
    A, B = workloads.lognormal(m, n, k, 1.0, 21)
    pa, _ = oracle.split("A", A, s)
    pb, _ = oracle.split("B", B, s)
    ws = ozimmu.alloc_workspace(m, n, k, s)
    ozimmu.dgemm(dev(A), dev(B), s, workspace=ws)
    for (l, h) in [(1, 1), (1, 5), (3, 2), (5, 1), (5, 5), (2, 4)]:
        got = host(ozimmu.debug_slice_product(m, n, k, s, ws, l, h)).T
        want = oracle.slice_product(pa[l - 1], pb[h - 1])
        assert np.array_equal(got.astype(np.int64), want), (l, h)
    if k > 64:
        k0, k1 = 32, 32 * (k // 32)
        got = host(ozimmu.debug_slice_product(m, n, k, s, ws, 2, 3, k0, k1)).T
        want = oracle.slice_product(pa[1][:, k0:k1], pb[2][k0:k1, :])
        assert np.array_equal(got.astype(np.int64), want)


@pytest.mark.parametrize("m,n,k,s", [(33, 70, 17, 3), (128, 128, 128, 3), (100, 90, 70, 7), (257, 130, 300, 9),
                                     (130, 257, 513, 1), (64, 64, 2048, 6), (100, 300, 70, 12), (129, 129, 200, 4), (200, 100, 64, 2),
                                     (100, 90, 70, 13), (130, 70, 300, 16), (65, 129, 200, 17), (257, 130, 100, 18),
                                     (70, 130, 150, 19), (130, 130, 96, 20), (130, 70, 200, 10), (70, 200, 130, 11),
                                     (300, 200, 260, 5), (200, 300, 520, 8)])
def test_int32_diagonal_sums_of_fused_kernel_bit_exact(m, n, k, s):
    A, B = workloads.uniform(m, n, k, 22)
    pa, _ = oracle.split("A", A, s)
    pb, _ = oracle.split("B", B, s)
    ws = ozimmu.alloc_workspace(m, n, k, s)
    ozimmu.dgemm(dev(A), dev(B), s, workspace=ws)
    D = host(ozimmu.debug_diagonals(m, n, k, s, ws))          # [s, n, m]
    for d in range(2, s + 2):
        want = sum(oracle.slice_product(pa[l - 1], pb[d - l - 1]) for l in range(1, d) if l <= s and d - l <= s)
        assert np.array_equal(D[d - 2].T.astype(np.int64), want), d


@pytest.fixture
def alternative_tile():
    ozimmu.debug_tile_choice(2)
    yield
    ozimmu.debug_tile_choice(0)


@pytest.mark.parametrize("kind", ["uniform", "lognormal", "pow2", "special"])
@pytest.mark.parametrize("m,n,k", SHAPES + [(192, 128, 64), (193, 129, 65), (400, 300, 200), (577, 257, 130), (96, 500, 1000)])
@pytest.mark.parametrize("s,tile", [(2, "128x128 ring of 3"), (3, "128x128 ring of 3"), (4, "192x128"), (5, "128x64"), (6, "128x64")])
def test_alternative_tiles_of_few_slices(kind, m, n, k, s, tile, alternative_tile):
    # at these sizes the launcher would not take them by itself; the knob forces the alternative: for 4 slices the
    # 192 x 128 tile, whose wavefronts hold three fragment rows (tiles that end inside the first, second and third
    # of them, one and several tiles each way); for 2 and 3 slices the 128 x 128 tile with its ring of three stages;
    # for 5 and 6 slices the 128 x 64 tile
    A, B = inputs(kind, m, n, k, 37)
    ws = ozimmu.alloc_workspace(m, n, k, s)
    C = ozimmu.dgemm(dev(A), dev(B), s, workspace=ws, check_finite=True)
    name = f"gemm_fused16_kernel<{s}> tile {tile}"
    assert ozimmu.last_gemm_kernel().startswith(name), ozimmu.last_gemm_kernel()
    assert_c_matches(host(C), oracle.dgemm(A, B, s), f"{tile} tile {kind} {m}x{n}x{k}")
    pa, _ = oracle.split("A", A, s)
    pb, _ = oracle.split("B", B, s)
    D = host(ozimmu.debug_diagonals(m, n, k, s, ws))
    for d in range(2, s + 2):
        want = sum(oracle.slice_product(pa[l - 1], pb[d - l - 1]) for l in range(1, d) if l <= s and d - l <= s)
        assert np.array_equal(D[d - 2].T.astype(np.int64), want), d
    # nearest slices and levels of two diagonals run the same kernel
    C3 = ozimmu.dgemm3(dev(A), dev(B), s, s, False, ozimmu.SPLIT_NEAREST, 2)
    assert ozimmu.last_gemm_kernel().startswith(name)
    assert_c_matches(host(C3), oracle.dgemm3(A, B, s, s, nearest=True, Q=2), f"{tile} tile, nearest, Q = 2")


def test_extreme_slices_do_not_overflow_int32_in_fused_kernel():
    # 1 - 2^-53 has 53 one-bits: slices 1..7 all equal 127, the largest magnitude there is.  With
    # s = 7 and k = 19008 (s * k just under the fused kernel's limit of 133144) the last diagonal
    # reaches 7 * 19008 * 127^2 = 2 146 060 224, just below 2^31.
    s, k = 7, 19008
    x = 1.0 - 2.0 ** -53
    A = np.full((40, k), x)
    A[1::2, :] = -x
    B = np.full((k, 40), x)
    ws = ozimmu.alloc_workspace(40, 40, k, s)
    C = host(ozimmu.dgemm(dev(A), dev(B), s, workspace=ws))
    D = host(ozimmu.debug_diagonals(40, 40, k, s, ws))
    assert int(D[s - 1].max()) == s * k * 127 * 127 and int(D[s - 1].min()) == -s * k * 127 * 127
    assert_c_matches(C, oracle.dgemm(A, B, s), "extreme")


# ----------------------------------------------------------------------------- C, small and ragged

@pytest.mark.parametrize("kind", ["uniform", "lognormal", "pow2", "special"])
@pytest.mark.parametrize("m,n,k", SHAPES)
@pytest.mark.parametrize("s", list(range(1, 33)))
def test_dgemm_matches_oracle(kind, m, n, k, s, tile_choice):
    A, B = inputs(kind, m, n, k, 31)
    ws = ozimmu.alloc_workspace(m, n, k, s)
    C = ozimmu.dgemm(dev(A), dev(B), s, workspace=ws, check_finite=True)
    Cref, eA, eB = oracle.dgemm(A, B, s, return_exponents=True)
    gA, gB = ozimmu.get_exponents(m, n, k, s, ws)
    assert np.array_equal(host(gA), eA) and np.array_equal(host(gB), eB)
    assert_c_matches(host(C), Cref, f"{kind} {m}x{n}x{k} s={s}")


def test_dgemm_config_uniform_128():
    cfg = workloads.CONFIGS["uniform_128"]
    A, B = cfg["gen"]()
    for s in cfg["s"]:
        assert_c_matches(host(ozimmu.dgemm(dev(A), dev(B), s)), oracle.dgemm(A, B, s), f"uniform_128 s={s}")


def test_dgemm_config_lognormal_1024_all_slice_counts(tile_choice):
    cfg = workloads.CONFIGS["lognormal_1024"]
    A, B = cfg["gen"]()
    dA, dB = dev(A), dev(B)
    for s in cfg["s"]:
        print(f"lognormal_1024 s={s}", flush=True)
        assert_c_matches(host(ozimmu.dgemm(dA, dB, s)), oracle.dgemm(A, B, s), f"lognormal_1024 s={s}")


def test_dgemm_with_leading_dimensions_and_c_view(tile_choice):
    m, n, k, s = 70, 50, 90, 6
    A, B = workloads.lognormal(m, n, k, 1.0, 4)
    bigA = ozimmu.colmajor_empty(100, k); bigA.fill_(1e300); bigA[:m, :] = torch.as_tensor(A)
    bigB = ozimmu.colmajor_empty(130, n); bigB.fill_(1e300); bigB[:k, :] = torch.as_tensor(B)
    bigC = ozimmu.colmajor_empty(77, n); bigC.fill_(-1.0)
    ozimmu.dgemm(bigA[:m, :], bigB[:k, :], s, C=bigC[:m, :])
    assert_c_matches(host(bigC[:m, :]), oracle.dgemm(A, B, s), "ld")
    assert bool((bigC[m:, :] == -1.0).all()), "rows of the C buffer outside the view must stay untouched"


def test_k_blocked_accumulation_beyond_the_int32_range():
    # k * 127^2 > 2^31 with all slices at +-127: a single int32 sum would overflow
    k, s = 140000, 2
    x = 1.0 - 2.0 ** -53
    A = np.full((20, k), x); A[::3, :] = -x
    B = np.full((k, 24), x); B[:, 1::2] *= 0.5
    assert_c_matches(host(ozimmu.dgemm(dev(A), dev(B), s)), oracle.dgemm(A, B, s), "k-blocked extreme")
    A, B = workloads.lognormal(40, 30, 150000, 2.0, 8)
    assert_c_matches(host(ozimmu.dgemm(dev(A), dev(B), 7)), oracle.dgemm(A, B, 7), "k-blocked lognormal")


@pytest.mark.parametrize("s", [4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 16, 17, 18, 19, 20])
def test_k_blocked_on_every_fused_kernel(s):
    # the fused kernels (16x16x64 for s = 4 ... 9; 32x32x32 otherwise, with four 512-register wavefronts beyond
    # s = 12) in split-k mode, several tiles and k-blocks
    m, n = 130, 70
    k = 3 * (133144 // s) + 200
    k = min(k, 70000)
    print(f"k-blocked s={s} k={k}", flush=True)
    A, B = workloads.lognormal(m, n, k, 2.0, 80 + s)
    assert_c_matches(host(ozimmu.dgemm(dev(A), dev(B), s)), oracle.dgemm(A, B, s), f"k-blocked s={s}")
    x = 1.0 - 2.0 ** -53
    A = np.full((m, k), x); A[::3, :] = -x
    B = np.full((k, n), x); B[:, 1::2] *= 0.5
    assert_c_matches(host(ozimmu.dgemm(dev(A), dev(B), s)), oracle.dgemm(A, B, s), f"k-blocked extreme s={s}")


def test_contraction_longer_than_32_bit_plane_offsets():
    # k * s * 32 >= 2^31 bytes in a fragment row of the planes: the copies carry 32-bit offsets, which must be
    # relative to the k-block of the work-group and not to the row
    s = 9
    k = (1 << 31) // (32 * s) + 1000
    A, B = workloads.uniform(3, 2, k, 77)
    print(f"long contraction k={k}", flush=True)
    assert_c_matches(host(ozimmu.dgemm(dev(A), dev(B), s)), oracle.dgemm(A, B, s), "very long k")


def test_runs_are_bit_identical():
    A, B = workloads.lognormal(300, 200, 500, 1.0, 5)
    dA, dB = dev(A), dev(B)
    for s in (7, 12):
        C1 = host(ozimmu.dgemm(dA, dB, s))
        C2 = host(ozimmu.dgemm(dA, dB, s))
        assert np.array_equal(C1, C2)


def test_degenerate_sizes(tile_choice):
    A, B = workloads.uniform(8, 6, 0, 1)
    C = ozimmu.dgemm(dev(A), dev(B), 3)
    assert tuple(C.shape) == (8, 6) and bool((C == 0).all())
    A, B = workloads.uniform(0, 6, 5, 1)
    assert tuple(ozimmu.dgemm(dev(A), dev(B), 3).shape) == (0, 6)
    A, B = workloads.uniform(4, 0, 5, 1)
    assert tuple(ozimmu.dgemm(dev(A), dev(B), 3).shape) == (4, 0)
    Z = np.zeros((5, 7))
    A, B = workloads.uniform(5, 4, 7, 1)
    assert bool((ozimmu.dgemm(dev(Z), dev(B), 4) == 0).all())


def test_nonfinite_input_is_reported_not_fatal():
    A, B = workloads.uniform(40, 30, 50, 2)
    for bad in (np.nan, np.inf, -np.inf):
        for which in (0, 1):
            A2, B2 = A.copy(), B.copy()
            (A2 if which == 0 else B2)[7, 9] = bad
            ws = ozimmu.alloc_workspace(40, 30, 50, 4)
            ozimmu.dgemm(dev(A2), dev(B2), 4, workspace=ws)
            with pytest.raises(ozimmu.OzimmuError) as ei:
                ozimmu.check(ws)
            assert ei.value.code == ozimmu.NONFINITE
            with pytest.raises(ozimmu.OzimmuError) as ei:
                ozimmu.estimate_slices(dev(A2), dev(B2), 1e-9)
            assert ei.value.code == ozimmu.NONFINITE
    ws = ozimmu.alloc_workspace(40, 30, 50, 4)
    ozimmu.dgemm(dev(A), dev(B), 4, workspace=ws)
    ozimmu.check(ws)     # clean input: no error


# ----------------------------------------------------------------------------- estimator

@pytest.mark.parametrize("kind", ["uniform", "lognormal", "pow2", "special"])
@pytest.mark.parametrize("m,n,k", [(5, 3, 2), (100, 90, 70), (257, 130, 300)])
def test_estimator_matches_oracle(kind, m, n, k):
    A, B = inputs(kind, m, n, k, 41)
    dA, dB = dev(A), dev(B)
    for tol in (1e-2, 1e-8, 1e-15, 2.0 ** -53, 1e-300):
        assert ozimmu.estimate_slices(dA, dB, tol) == oracle.estimate_slices(A, B, tol, s_max=ozimmu.MAX_SLICES), tol


def test_estimator_on_config_lognormal_1024():
    A, B = workloads.CONFIGS["lognormal_1024"]["gen"]()
    dA, dB = dev(A), dev(B)
    for tol in (1e-8, 1e-15):
        got = ozimmu.estimate_slices(dA, dB, tol)
        assert got == oracle.estimate_slices(A, B, tol, s_max=ozimmu.MAX_SLICES)
        print("lognormal_1024 tol", tol, "->", got, flush=True)


# ----------------------------------------------------------------------------- different slice counts

PAIRS = [(1, 8), (8, 1), (3, 9), (9, 3), (2, 2), (7, 7), (13, 13), (16, 16), (18, 18), (20, 7), (7, 20), (32, 32),
         (1, 1), (12, 5), (25, 31),
         # counts that differ little: run as equal counts with zero slices appended to the short operand
         (7, 8), (8, 7), (5, 8), (4, 8), (6, 9), (8, 10), (12, 13), (12, 16), (17, 18), (20, 19), (11, 20), (3, 4), (1, 2)]


@pytest.mark.parametrize("kind", ["uniform", "lognormal", "special"])
@pytest.mark.parametrize("m,n,k", [(5, 3, 2), (100, 90, 70), (257, 130, 300)])
@pytest.mark.parametrize("sA,sB", PAIRS)
def test_dgemm2_matches_oracle(kind, m, n, k, sA, sB):
    A, B = inputs(kind, m, n, k, 51)
    C = ozimmu.dgemm2(dev(A), dev(B), sA, sB, check_finite=True)
    assert_c_matches(host(C), oracle.dgemm2(A, B, sA, sB), f"{kind} {m}x{n}x{k} sA={sA} sB={sB}")


@pytest.mark.parametrize("sA,sB", [(1, 1), (2, 5), (5, 2), (2, 2), (3, 3), (4, 4), (5, 5), (6, 6), (7, 7), (8, 8), (9, 9),
                                   (10, 10), (12, 12), (9, 17), (20, 20),
                                   (5, 4), (7, 9), (9, 6), (3, 2)])      # run as equal counts, zero slices appended
def test_dgemm2_all_products_matches_oracle(sA, sB):
    A, B = workloads.lognormal(130, 70, 200, 2.0, 52)
    C = ozimmu.dgemm2(dev(A), dev(B), sA, sB, all_products=True)
    assert_c_matches(host(C), oracle.dgemm2(A, B, sA, sB, full=True), f"all products sA={sA} sB={sB}")


def test_dgemm_equals_dgemm2_with_equal_counts():
    A, B = workloads.lognormal(200, 150, 400, 1.0, 53)
    dA, dB = dev(A), dev(B)
    for s in (1, 5, 7, 12, 13, 20):
        assert bool(torch.equal(ozimmu.dgemm(dA, dB, s), ozimmu.dgemm2(dA, dB, s, s)))


def test_band_kernel_with_int64_totals():
    # 20 slices of A, k = 7000: more than 133144 terms can meet in one diagonal accumulator, so the
    # band kernel has to spill to its int64 totals; entries chosen so that every slice is +-127 or 120
    k = 7000
    x = 1.0 - 2.0 ** -53
    A = np.full((70, k), x); A[::3, :] = -x
    B = np.full((k, 40), x); B[:, 1::2] *= 0.5
    for sA, sB in ((20, 20), (20, 9), (9, 20)):
        assert_c_matches(host(ozimmu.dgemm2(dev(A), dev(B), sA, sB)), oracle.dgemm2(A, B, sA, sB), f"totals {sA},{sB}")
    A, B = workloads.lognormal(70, 40, 40000, 2.0, 54)
    assert_c_matches(host(ozimmu.dgemm2(dev(A), dev(B), 14, 10)), oracle.dgemm2(A, B, 14, 10), "totals long k")


def test_well_scaled_operand_single_slice_on_gpu():
    rng = np.random.default_rng(8)
    A = rng.integers(-127, 128, size=(150, 300)) * np.ldexp(1.0, rng.integers(-20, 20, size=150))[:, None]
    _, B = workloads.lognormal(150, 90, 300, 2.0, 9)
    dA, dB = dev(A), dev(B)
    for s in (8, 12):
        assert bool(torch.equal(ozimmu.dgemm2(dA, dB, 1, s), ozimmu.dgemm(dA, dB, s)))


@pytest.mark.parametrize("kind", ["uniform", "lognormal", "special"])
def test_estimator2_matches_oracle(kind):
    A, B = inputs(kind, 100, 90, 70, 61)
    dA, dB = dev(A), dev(B)
    for tol in (1e-2, 1e-8, 1e-15, 1e-300):
        assert ozimmu.estimate_slices2(dA, dB, tol) == oracle.estimate_slices2(A, B, tol, s_max=ozimmu.MAX_SLICES), tol
    rng = np.random.default_rng(3)
    A2 = np.sign(A + 0.5) * np.ldexp(1.0, rng.integers(-5, 6, size=100))[:, None]      # kappa_A = 2
    got = ozimmu.estimate_slices2(dev(A2), dB, 1e-12)
    assert got == oracle.estimate_slices2(A2, B, 1e-12, s_max=ozimmu.MAX_SLICES)
    assert got[0] <= got[1]


@pytest.mark.parametrize("kappa_d", [1e10, 1e20, 1e30, 1e40])
def test_badly_scaled_workload_matches_oracle(kappa_d):
    # the diagonal-scaling test of the GPU benchmark section, slice counts as used there
    A, B = workloads.diag_scaled(200, kappa_d, 7)
    dA, dB = dev(A), dev(B)
    est = ozimmu.estimate_slices(dA, dB, 2.0 ** -53)
    assert est == oracle.estimate_slices(A, B, 2.0 ** -53, s_max=ozimmu.MAX_SLICES)
    for s in sorted({8, 12, 16, 18, est[0]}):
        assert_c_matches(host(ozimmu.dgemm(dA, dB, s)), oracle.dgemm(A, B, s), f"kappa_D={kappa_d:g} s={s}")


# ----------------------------------------------------------------------------- round-to-nearest slices, levels

def tie_heavy(rows, cols, seed):
    """Entries with few significant bits at many binary positions: rounding ties and carries at every cut."""
    rng = np.random.default_rng(seed)
    mant = rng.integers(1, 512, size=(rows, cols)).astype(np.float64)
    X = np.ldexp(mant, rng.integers(-40, 3, size=(rows, cols))) * rng.choice([-1.0, 1.0], size=(rows, cols))
    X[rng.random((rows, cols)) < 0.05] = 0.0
    return X


@pytest.mark.parametrize("kind", ["uniform", "lognormal", "special", "ties"])
@pytest.mark.parametrize("m,n,k", SHAPES)
@pytest.mark.parametrize("s", [1, 3, 8, 32])
def test_split_nearest_bit_exact_in_both_layouts(kind, m, n, k, s):
    A, B = (tie_heavy(m, k, 5), tie_heavy(k, n, 6)) if kind == "ties" else inputs(kind, m, n, k, 13)
    for side, X in (("A", A), ("B", B)):
        want_planes, want_e = oracle.split_nearest(side, X, s)
        rows, cols = X.shape
        planes, e = ozimmu.split(side, dev(X), s, ozimmu.LAYOUT_PLAIN, splitting=ozimmu.SPLIT_NEAREST)
        assert np.array_equal(host(e), want_e + 1), (side, "exponents of the doubled scales")
        assert np.array_equal(host(planes).reshape(s, cols, rows).transpose(0, 2, 1), want_planes), (side, "plain")
        planes, e = ozimmu.split(side, dev(X), s, ozimmu.LAYOUT_MFMA, splitting=ozimmu.SPLIT_NEAREST)
        R, K = (rows, cols) if side == "A" else (cols, rows)
        got, full = untile(host(planes), R, K, s)
        assert np.array_equal(host(e), want_e + 1)
        assert np.array_equal(got, want_planes if side == "A" else want_planes.transpose(0, 2, 1)), (side, "mfma")
        assert not full[:, R:, :].any() and not full[:, :, K:].any(), "padding must be zero"


VARIANT_CASES = [
    # sA, sB, all_products, nearest, Q        kernel that runs
    (7, 7, False, True, 1),                 # fused 16x16x64, split stage
    (8, 8, False, True, 1),
    (7, 7, False, False, 3),
    (6, 6, False, True, 3),                 # fused 32x32x32
    (9, 9, False, False, 2),                # fused 16x16x64 with part of B read on demand
    (10, 10, False, True, 2),               # fused 32x32x32
    (4, 4, False, False, 2),                # fused 16x16x64, wide tile
    (8, 8, False, False, 3),
    (12, 12, False, True, 4),
    (13, 13, False, False, 3),              # band kernel: groups of 6 diagonals
    (16, 16, False, True, 2),
    (5, 11, False, False, 3),
    (11, 5, False, True, 4),
    (7, 8, False, True, 3),                 # runs as (8, 8) with a zero slice appended to A
    (9, 7, False, False, 2),
    (6, 4, True, False, 3),
    (9, 9, True, True, 2),
    (18, 18, False, False, 4),
    (32, 32, False, False, 3),
]


@pytest.mark.parametrize("sA,sB,allp,nearest,Q", VARIANT_CASES)
@pytest.mark.parametrize("m,n,k,kind", [(100, 90, 70, "lognormal"), (257, 130, 300, "special"), (150, 200, 1000, "ties")])
def test_dgemm3_variants_bit_exact(sA, sB, allp, nearest, Q, m, n, k, kind, tile_choice):
    A, B = (tie_heavy(m, k, 7), tie_heavy(k, n, 8)) if kind == "ties" else inputs(kind, m, n, k, 14)
    assert Q <= ozimmu.max_level_diagonals(k, sA, sB)
    print(f"dgemm3 sA={sA} sB={sB} all={allp} nearest={nearest} Q={Q} {m}x{n}x{k} {kind}", flush=True)
    ws = torch.empty(ozimmu.lib().ozimmu_workspace_bytes2(m, n, k, sA, sB, int(allp)), dtype=torch.uint8, device="cuda")
    C = ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, ozimmu.SPLIT_NEAREST if nearest else ozimmu.SPLIT_TRUNCATE, Q,
                      workspace=ws)
    want, eA, eB = oracle.dgemm3(A, B, sA, sB, full=allp, nearest=nearest, Q=Q, return_exponents=True)
    assert_c_matches(host(C), want, "dgemm3")
    if sA == sB and not allp:
        gA, gB = ozimmu.get_exponents(m, n, k, sA, ws)
        assert np.array_equal(host(gA), eA) and np.array_equal(host(gB), eB)


@pytest.mark.parametrize("s,Q,nearest", [(4, 3, True), (7, 3, False), (8, 2, True), (12, 3, False), (14, 3, True)])
def test_dgemm3_variants_in_k_blocked_mode(s, Q, nearest):
    m, n = 130, 70
    k = min(2 * (133144 // s) + 200, 70000)
    assert Q <= ozimmu.max_level_diagonals(k, s, s)
    print(f"dgemm3 k-blocked s={s} Q={Q} nearest={nearest} k={k}", flush=True)
    A, B = workloads.lognormal(m, n, k, 2.0, 90 + s)
    C = ozimmu.dgemm3(dev(A), dev(B), s, s, False, ozimmu.SPLIT_NEAREST if nearest else ozimmu.SPLIT_TRUNCATE, Q)
    assert_c_matches(host(C), oracle.dgemm3(A, B, s, s, nearest=nearest, Q=Q), "dgemm3 k-blocked")


@pytest.mark.parametrize("sA,sB", [(2, 9), (9, 2), (5, 11), (14, 6), (3, 18), (17, 12), (8, 9), (7, 6), (18, 17), (19, 20)])
def test_different_slice_counts_in_k_blocked_mode(sA, sB):
    # fused kernel with the short operand's count at run time, split-k: k beyond 133144 / min(sA, sB)
    m, n = 130, 70
    k = min(2 * (133144 // min(sA, sB)) + 200, 150000)
    print(f"k-blocked sA={sA} sB={sB} k={k}", flush=True)
    A, B = workloads.lognormal(m, n, k, 2.0, 60 + sA)
    assert_c_matches(host(ozimmu.dgemm2(dev(A), dev(B), sA, sB)), oracle.dgemm2(A, B, sA, sB), "k-blocked unequal")


@pytest.mark.parametrize("s", [3, 6, 7, 9])
def test_all_products_in_k_blocked_mode(s):
    # the fused kernel's all-products set (2 s - 1 diagonals) in split-k mode
    m, n = 130, 70
    k = min(2 * (133144 // s) + 200, 100000)
    print(f"k-blocked all products s={s} k={k}", flush=True)
    A, B = workloads.lognormal(m, n, k, 2.0, 70 + s)
    got = host(ozimmu.dgemm3(dev(A), dev(B), s, s, True, ozimmu.SPLIT_TRUNCATE, 2))
    assert_c_matches(got, oracle.dgemm3(A, B, s, s, full=True, Q=2), "k-blocked all products")


def test_dgemm3_defaults_equal_dgemm2_and_bad_level_size_is_refused():
    A, B = workloads.lognormal(90, 80, 200, 1.0, 15)
    dA, dB = dev(A), dev(B)
    for sA, sB, allp in [(7, 7, False), (5, 9, False), (4, 6, True)]:
        assert torch.equal(ozimmu.dgemm3(dA, dB, sA, sB, allp), ozimmu.dgemm2(dA, dB, sA, sB, allp))
    qmax = ozimmu.max_level_diagonals(200, 7, 7)
    ozimmu.dgemm3(dA, dB, 7, 7, level_diagonals=qmax)
    for bad in (0, qmax + 1, 9):
        with pytest.raises(ozimmu.OzimmuError) as ei:
            ozimmu.dgemm3(dA, dB, 7, 7, level_diagonals=bad)
        assert ei.value.code == ozimmu.BAD_ARG
    with pytest.raises(ozimmu.OzimmuError):
        ozimmu.dgemm3(dA, dB, 7, 7, splitting=2)


def test_largest_admitted_level_is_exact_on_the_worst_case_input():
    # all slices at +-127 and every product of a diagonal of the same sign: the level sums reach the bound
    # ozimmu_max_level_diagonals is derived from; the oracle refuses a level that is not a binary64 number
    x = 1.0 - 2.0 ** -53
    for k, s in [(64, 7), (1000, 7), (8192, 5)]:
        A, B = np.full((40, k), x), np.full((k, 33), x)
        Q = ozimmu.max_level_diagonals(k, s, s)
        want = oracle.dgemm3(A, B, s, s, Q=Q)
        assert_c_matches(host(ozimmu.dgemm3(dev(A), dev(B), s, s, level_diagonals=Q)), want, f"worst case k={k}")


def test_variants_on_degenerate_and_strided_inputs():
    # empty dimensions, k = 0, a single entry, and leading dimensions larger than the row count, through dgemm2 / dgemm3
    for sA, sB, allp, nearest, Q in [(3, 9, False, False, 1), (14, 14, False, True, 2), (5, 5, True, False, 2), (20, 6, False, True, 3)]:
        sp = ozimmu.SPLIT_NEAREST if nearest else ozimmu.SPLIT_TRUNCATE
        A, B = workloads.uniform(8, 6, 0, 1)
        C = ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, sp, Q)
        assert tuple(C.shape) == (8, 6) and bool((C == 0).all())
        A, B = workloads.uniform(0, 6, 5, 1)
        assert tuple(ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, sp, Q).shape) == (0, 6)
        A, B = workloads.uniform(4, 0, 5, 1)
        assert tuple(ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, sp, Q).shape) == (4, 0)
        A, B = workloads.lognormal(1, 1, 1, 1.0, 2)
        assert_c_matches(host(ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, sp, Q)),
                         oracle.dgemm3(A, B, sA, sB, full=allp, nearest=nearest, Q=Q), "1x1x1")
        m, n, k = 70, 50, 90
        A, B = workloads.lognormal(m, n, k, 1.0, 4)
        bigA = ozimmu.colmajor_empty(100, k); bigA.fill_(1e300); bigA[:m, :] = torch.as_tensor(A)
        bigB = ozimmu.colmajor_empty(130, n); bigB.fill_(1e300); bigB[:k, :] = torch.as_tensor(B)
        bigC = ozimmu.colmajor_empty(77, n); bigC.fill_(-1.0)
        ozimmu.dgemm3(bigA[:m, :], bigB[:k, :], sA, sB, allp, sp, Q, C=bigC[:m, :])
        assert_c_matches(host(bigC[:m, :]), oracle.dgemm3(A, B, sA, sB, full=allp, nearest=nearest, Q=Q), "ld")
        assert bool((bigC[m:, :] == -1.0).all())


def test_nonfinite_input_is_reported_in_every_variant():
    A, B = workloads.uniform(40, 30, 50, 2)
    A[3, 4] = np.inf
    for sA, sB, nearest in [(4, 9, False), (15, 15, True), (22, 3, True)]:
        ws = torch.empty(ozimmu.lib().ozimmu_workspace_bytes2(40, 30, 50, sA, sB, 0), dtype=torch.uint8, device="cuda")
        ozimmu.dgemm3(dev(A), dev(B), sA, sB, False, ozimmu.SPLIT_NEAREST if nearest else ozimmu.SPLIT_TRUNCATE, 1,
                      workspace=ws)
        with pytest.raises(ozimmu.OzimmuError) as ei:
            ozimmu.check(ws)
        assert ei.value.code == ozimmu.NONFINITE


def test_seeded_random_configurations(tile_choice):
    # 60 configurations drawn from a fixed seed: shapes, slice counts, product set, slicing rule and level size
    rng = np.random.default_rng(20250611)
    for case in range(60):
        m, n = int(rng.integers(1, 300)), int(rng.integers(1, 300))
        k = int(rng.integers(1, 700))
        sA, sB = int(rng.integers(1, 33)), int(rng.integers(1, 33))
        if rng.random() < 0.4:
            sB = sA
        allp = bool(rng.random() < 0.25)
        nearest = bool(rng.random() < 0.5)
        Q = int(rng.integers(1, ozimmu.max_level_diagonals(k, sA, sB) + 1))
        phi = float(rng.choice([0.5, 2.0, 6.0]))
        print(f"case {case}: {m}x{n}x{k} sA={sA} sB={sB} all={allp} nearest={nearest} Q={Q} phi={phi}", flush=True)
        A, B = workloads.lognormal(m, n, k, phi, 5000 + case)
        got = host(ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, ozimmu.SPLIT_NEAREST if nearest else ozimmu.SPLIT_TRUNCATE, Q))
        assert_c_matches(got, oracle.dgemm3(A, B, sA, sB, full=allp, nearest=nearest, Q=Q), f"case {case}")


def test_seeded_random_configurations_with_special_values_and_every_tile_rule():
    # 150 more from a fixed seed, larger shapes and contraction lengths up to 30000 (k-blocks), with every setting
    # of the two tile knobs (automatic, forced either way), and in 40 % of the cases a zero row and column, a
    # subnormal, a huge, a negative-zero entry, a column scaled by a power of two and a row of powers of two
    rng = np.random.default_rng(2506112771)
    try:
        done = 0
        while done < 150:
            big = rng.random() < 0.25
            m, n = int(rng.integers(1, 1400 if big else 400)), int(rng.integers(1, 1400 if big else 400))
            k = int(rng.choice([rng.integers(1, 300), rng.integers(300, 3000), rng.integers(3000, 30000)], p=[.4, .35, .25]))
            if big:
                k = min(k, 600)
            sA = int(rng.integers(1, 33))
            sB = sA if rng.random() < 0.5 else int(rng.integers(1, 33))
            allp, nearest = bool(rng.random() < 0.15), bool(rng.random() < 0.3)
            Q = int(rng.integers(1, min(ozimmu.max_level_diagonals(k, sA, sB), 4) + 1))
            small, tile = int(rng.choice([-1, 0, 256])), int(rng.choice([0, 1, 2]))
            phi = float(rng.choice([0.5, 2.0, 6.0]))
            special = rng.random() < 0.4
            if m * n * k * (sA * sB if allp else max(sA, sB) ** 2 / 2) > 2e10:
                continue
            A, B = workloads.lognormal(m, n, k, phi, 7000 + done)
            if special:
                if m > 2:
                    A[int(rng.integers(0, m)), :] = 0.0
                if n > 2:
                    B[:, int(rng.integers(0, n))] = 0.0
                A[int(rng.integers(0, m)), int(rng.integers(0, k))] = 5e-324 * float(rng.integers(1, 1000))
                B[int(rng.integers(0, k)), int(rng.integers(0, n))] = -1.0e300
                B[int(rng.integers(0, k)), int(rng.integers(0, n))] = -0.0
                A[:, int(rng.integers(0, k))] *= 2.0 ** int(rng.integers(-300, 300))
                A[int(rng.integers(0, m)), :] = np.ldexp(1.0, int(rng.integers(-1000, -300)))
                A *= 1e-100                               # keeps the exact product finite
            print(f"case {done}: {m}x{n}x{k} sA={sA} sB={sB} all={allp} nearest={nearest} Q={Q} small={small} tile={tile} "
                  f"phi={phi} special={special}", flush=True)
            ozimmu.debug_small_tile_limit(small)
            ozimmu.debug_tile_choice(tile)
            got = host(ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, ozimmu.SPLIT_NEAREST if nearest else ozimmu.SPLIT_TRUNCATE, Q))
            want = oracle.dgemm3(A, B, sA, sB, full=allp, nearest=nearest, Q=Q)
            assert np.isfinite(want).all()
            assert_c_matches(got, want, f"case {done} ({ozimmu.last_gemm_kernel()})")
            done += 1
    finally:
        ozimmu.debug_small_tile_limit(-1)
        ozimmu.debug_tile_choice(0)


@pytest.mark.parametrize("sA,sB,allp", [(4, 4, False), (5, 5, False), (6, 6, False), (7, 7, False), (8, 8, False), (9, 9, False), (12, 12, False),
                                        (16, 16, False), (18, 18, False), (20, 20, False), (5, 11, False),
                                        (13, 4, False), (6, 6, True)])
def test_exactly_two_k_blocks(sA, sB, allp):
    # two k-blocks take the path without atomics: an int32 slot per block, added by the finish kernel
    m, n = 130, 70
    k = (133144 // min(sA, sB)) * 3 // 2
    print(f"two k-blocks sA={sA} sB={sB} all={allp} k={k}", flush=True)
    x = 1.0 - 2.0 ** -53
    A, B = workloads.lognormal(m, n, k, 2.0, 40 + sA)
    A[:7, :] = x                      # rows and columns whose slices are all +-127: the largest sums there are
    B[:, :5] = -x
    got = host(ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, ozimmu.SPLIT_TRUNCATE, 1))
    assert_c_matches(got, oracle.dgemm3(A, B, sA, sB, full=allp), "two k-blocks")


@pytest.mark.parametrize("sA,sB,allp,nearest,Q", [(7, 7, False, False, 1), (4, 12, False, False, 1), (12, 4, False, True, 2),
                                                  (3, 18, False, False, 3), (16, 16, False, True, 1), (6, 6, True, False, 2),
                                                  (25, 9, False, False, 1)])
def test_transposed_problem_gives_the_transposed_result(sA, sB, allp, nearest, Q):
    # (A B)^T = B^T A^T: rows of A become columns, slice counts swap sides, every diagonal sum and the order of
    # the additions stay the same -> bit-identical.  Exercises the row / column split kernels and the two
    # short-operand variants of the GEMM against each other.
    A, B = workloads.lognormal(150, 90, 260, 2.0, 77)
    sp = ozimmu.SPLIT_NEAREST if nearest else ozimmu.SPLIT_TRUNCATE
    C = host(ozimmu.dgemm3(dev(A), dev(B), sA, sB, allp, sp, Q))
    Ct = host(ozimmu.dgemm3(dev(B.T.copy()), dev(A.T.copy()), sB, sA, allp, sp, Q))
    assert np.array_equal(C, Ct.T)
    assert_c_matches(C, oracle.dgemm3(A, B, sA, sB, full=allp, nearest=nearest, Q=Q), "transposition")


def test_small_tile_is_taken_where_it_finishes_sooner():
    # the default rule: (rounds of the compute units) x (tile area) / (relative speed), over the tabulated tile, the
    # alternative tile of 2 ... 6 slices and the 64 x 64 tile.  2048^2 with 2 slices: 128 tiles of 256 x 128 (half a
    # round) lose to one round of 128 x 128; 2560^2: 200 such tiles win against two rounds; every kernel gives the
    # same bits
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("the expectations are worked out for 256 compute units")
    for n, s, want in [(1024, 3, "gemm_fused_kernel<3> equal counts tile 64x64"), (2048, 2, "gemm_fused16_kernel<2> tile 128x128 ring of 3"),
                       (2560, 2, "gemm_fused16_kernel<2> tile 256x128"), (3000, 3, "gemm_fused16_kernel<3> tile 128x128 ring of 3"),
                       (2304, 4, "gemm_fused16_kernel<4> tile 192x128"), (2560, 4, "gemm_fused16_kernel<4> tile 128x128"),
                       (2304, 6, "gemm_fused16_kernel<6> tile 128x64"), (2560, 6, "gemm_fused16_kernel<6> tile 128x128"),
                       (3000, 7, "gemm_fused16_kernel<7> tile 128x64"), (100, 7, "gemm_fused_kernel<7> equal counts tile 64x64")]:
        dA, dB = workloads.lognormal_device(n, n, 96, 1.0, 91)
        ozimmu.debug_small_tile_limit(-1)
        ozimmu.debug_tile_choice(0)
        C = ozimmu.dgemm(dA, dB, s)
        assert ozimmu.last_gemm_kernel().startswith(want), (n, s, ozimmu.last_gemm_kernel())
        ozimmu.debug_small_tile_limit(0 if "64x64" in want else 1 << 40)
        C2 = ozimmu.dgemm(dA, dB, s)
        assert not ozimmu.last_gemm_kernel().startswith(want)
        assert bool(torch.equal(C, C2)), (n, s)
        rows = np.array([0, 1, 63, 64, n // 2, n - 65, n - 1])
        tr = torch.as_tensor(rows, device="cuda")
        assert_c_matches(host(C[tr][:, tr]), oracle.dgemm(host(dA[tr, :]), host(dB[:, tr]), s), f"tile rule {n} s={s}")


def test_which_kernel_takes_which_product_set():
    # the launchers report what they ran; one case per path of the routing
    A, B = workloads.uniform(70, 60, 50, 5)
    dA, dB = dev(A), dev(B)
    expect = [((2, 2, False), "gemm_fused16_kernel<2> tile 256x128 ring of 3"),
              ((3, 3, False), "gemm_fused16_kernel<3> tile 256x128"),
              ((4, 4, False), "gemm_fused16_kernel<4> tile 128x128"),       # (192 x 128 where the tile grid favours it)
              ((6, 6, False), "gemm_fused16_kernel<6> tile 128x128"),
              ((7, 7, False), "gemm_fused16_kernel<7> tile 128x64"),
              ((12, 12, False), "gemm_fused_kernel<12> equal counts tile 128x64, 8 wavefronts"),
              ((16, 16, False), "gemm_fused_kernel<16> equal counts tile 64x64, 4 wavefronts"),
              ((7, 8, False), "gemm_fused16_kernel<8> tile 128x64"),                 # run as (8, 8), zero slice appended
              ((4, 12, False), "gemm_fused_kernel<12> different counts tile 128x64, 8 wavefronts"),
              ((7, 12, False), "gemm_fused_kernel<12> different counts tile 128x64, 8 wavefronts"),
              ((5, 14, False), "gemm_fused_kernel<14> different counts tile 64x64, 4 wavefronts"),     # 28 % surplus as blocks
              ((8, 16, False), "blocks of slice groups: 1 x 2 groups of 8 slices through gemm_fused16_kernel<8> and <7>"),
              ((14, 6, False), "blocks of slice groups: 2 x 1 groups of 7 slices through gemm_fused16_kernel<7> and <6>"),
              ((6, 6, True), "gemm_fused_kernel<6> all products tile 128x64, 8 wavefronts"),
              ((18, 18, False), "gemm_fused_kernel<18> equal counts tile 64x64, 4 wavefronts"),   # one k-block
              ((17, 18, False), "gemm_fused_kernel<18> equal counts tile 64x64, 4 wavefronts"),
              ((24, 24, False), "blocks of slice groups: 3 x 3 groups of 8 slices through gemm_fused16_kernel<8> and <7>"),
              ((26, 26, False), "blocks of slice groups: 3 x 3 groups of 9 slices"),
              ((25, 31, False), "blocks of slice groups: 4 x 4 groups of 8 slices"),
              ((20, 7, False), "blocks of slice groups: 3 x 1 groups of 7 slices"),
              ((13, 13, True), "blocks of slice groups: 2 x 2 groups of 7 slices through gemm_fused16_kernel<7> and <6>"),
              ((21, 21, False), "blocks of slice groups: 3 x 3 groups of 7 slices through gemm_fused16_kernel<7> and <6> tile 128x64, a slot per block"),
              ((16, 16, True), "blocks of slice groups: 2 x 2 groups of 8 slices through gemm_fused16_kernel<8> and <7>"),
              ((12, 5, True), "gemm_banded_kernel (12, 5) slices")]
    for (sA, sB, allp), name in expect:
        C = ozimmu.dgemm2(dA, dB, sA, sB, allp)
        assert ozimmu.last_gemm_kernel().startswith(name), (sA, sB, allp, ozimmu.last_gemm_kernel())
        assert_c_matches(host(C), oracle.dgemm3(A, B, sA, sB, full=allp), f"routing ({sA},{sB},{allp})")
    # 18 slices whose contraction needs two k-blocks (18 k > 133144) run as two groups of 9 instead
    A, B = workloads.uniform(70, 60, 7424, 6)
    for sA in (18, 17):
        C = ozimmu.dgemm2(dev(A), dev(B), sA, 18)
        assert ozimmu.last_gemm_kernel().startswith("blocks of slice groups: 2 x 2 groups of 9 slices through gemm_fused16_kernel<9> and <8> tile 128x64, a slot per block")
        assert_c_matches(host(C), oracle.dgemm2(A, B, sA, 18), f"routing ({sA},18) long k")


@pytest.mark.parametrize("s,k", [(21, 300), (21, 19200), (24, 300), (24, 17000), (26, 16000), (27, 2000), (28, 257), (32, 17000), (32, 1000)])
def test_blocks_of_slice_groups_over_column_panels_and_k_blocks(s, k):
    # 21 ... 32 slices run as blocks of the (l, h) grid, each block storing its int32 diagonal sums into a slot of
    # its own (k within 133144 / G) or adding them to shared int64 totals (k beyond: several k-blocks per block
    # launch; G = 7, 8 or 9 slices per group): column panels of 128 (buffer budget of one byte: two or three
    # panels, the last one ragged), zero slices appended (26 -> 27)
    m, n = (130, 300) if k < 1000 else (40, 200)
    A, B = workloads.lognormal(m, n, k, 2.0, 60 + s)
    want = oracle.dgemm(A, B, s)
    got_whole = host(ozimmu.dgemm(dev(A), dev(B), s))
    try:
        ozimmu.debug_panel_bytes(1)
        small_ws = ozimmu.workspace_bytes(m, n, k, s)
        got = host(ozimmu.dgemm(dev(A), dev(B), s))
    finally:
        ozimmu.debug_panel_bytes(1 << 30)
    assert small_ws < ozimmu.workspace_bytes(m, n, k, s)
    assert_c_matches(got_whole, want, "blocks")
    assert_c_matches(got, want, "blocks, column panels")


@pytest.mark.parametrize("sA,sB,allp", [(7, 7, False), (4, 4, False), (16, 16, False), (5, 11, False), (6, 6, True)])
def test_split_k_over_column_panels(sA, sB, allp):
    # totals budget of one byte: panels of 128 columns, so n = 300 takes three panels (the last one ragged)
    m, n = 130, 300
    k = (133144 // min(sA, sB)) * 5 // 2
    A, B = workloads.lognormal(m, n, k, 2.0, 30 + sA)
    want = oracle.dgemm3(A, B, sA, sB, full=allp)
    try:
        ozimmu.debug_panel_bytes(1)
        small_ws = ozimmu.lib().ozimmu_workspace_bytes2(m, n, k, sA, sB, int(allp))
        got = host(ozimmu.dgemm2(dev(A), dev(B), sA, sB, allp))
    finally:
        ozimmu.debug_panel_bytes(1 << 30)
    assert small_ws < ozimmu.lib().ozimmu_workspace_bytes2(m, n, k, sA, sB, int(allp))
    assert_c_matches(got, want, "column panels")
