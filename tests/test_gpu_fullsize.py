"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (same entry point, same workspace sizing).  The oracle cannot form a whole
8192^3 product, but every row of A and column of B carries its own scale, so any sub-block
C[rows, cols] is exactly the product of A[rows, :] and B[:, cols]: the oracle computes sampled
sub-blocks one by one and the GPU's entries must match them bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import oracle
from paper_2506_11277_amd import ozimmu, workloads


def sample_indices(n, seed, count=20):
    rng = np.random.default_rng(seed)
    # first and last tiles, and both sides of the boundaries of the 4 x 2 grid of tile regions (n/4, n/2, 3n/4)
    fixed = [0, 1, 31, 32, 33, 63, 64, 127, 128, 129, 255, 256, n // 4 - 1, n // 4, n // 2 - 1, n // 2, 3 * n // 4 - 1,
             3 * n // 4, n - 129, n - 128, n - 65, n - 33, n - 2, n - 1]
    idx = sorted(set(i for i in fixed if 0 <= i < n) | set(rng.integers(0, n, size=count).tolist()))
    return np.array(idx, dtype=np.int64)


def check_sampled(dA, dB, s, tag):
    m, k = dA.shape
    n = dB.shape[1]
    ws = ozimmu.alloc_workspace(m, n, k, s)
    C = ozimmu.dgemm(dA, dB, s, workspace=ws, check_finite=True)
    rows, cols = sample_indices(m, 1), sample_indices(n, 2)
    tr, tc = torch.as_tensor(rows, device="cuda"), torch.as_tensor(cols, device="cuda")
    As = dA[tr, :].cpu().numpy()
    Bs = dB[:, tc].cpu().numpy()
    want, eA, eB = oracle.dgemm(As, Bs, s, return_exponents=True)
    got = C[tr][:, tc].cpu().numpy()
    gA, gB = ozimmu.get_exponents(m, n, k, s, ws)
    assert np.array_equal(gA[tr].cpu().numpy(), eA) and np.array_equal(gB[tc].cpu().numpy(), eB), tag
    diff = np.abs(got - want)
    rel = float(np.max(np.where(diff == 0, 0.0, diff / np.abs(want))))
    assert rel <= 1e-15, f"{tag}: relative difference {rel:.3e}"
    assert np.array_equal(got, want), f"{tag}: not bit-identical (rel {rel:.3e})"
    # a second run is bit-identical everywhere (fixed summation order, no atomics on C)
    C2 = ozimmu.dgemm(dA, dB, s, workspace=ws)
    assert bool(torch.equal(C, C2)), f"{tag}: run-to-run difference"
    return C


def check_block(dA, dB, C, s, r0, c0, size, tag):
    """One contiguous size x size block of C (every entry of the tiles it covers) against the oracle."""
    want = oracle.dgemm(dA[r0:r0 + size, :].cpu().numpy(), dB[:, c0:c0 + size].cpu().numpy(), s)
    got = C[r0:r0 + size, c0:c0 + size].cpu().numpy()
    assert np.array_equal(got, want), f"{tag}: block at ({r0}, {c0}) not bit-identical"


def check_whole_matrix_against_other_tile_shape(dA, dB, C, s, tag):
    """Every entry of C: the kernel with the 64 x 64 tile (another tile grid, another order of work-groups) must
    give the same matrix bit for bit, nothing may be left unwritten, and the result must be a product of A and B."""
    assert bool(torch.isfinite(C).all()), f"{tag}: non-finite entries"
    ref = torch.matmul(dA, dB)
    err = (torch.linalg.norm(C - ref) / torch.linalg.norm(ref)).item()
    assert err <= max(2.0 ** (-7 * s + 12), 1e-13), f"{tag}: normwise distance to the binary64 product {err:.3e}"
    del ref
    try:
        ozimmu.debug_small_tile_limit(1 << 40)
        C2 = ozimmu.dgemm(dA, dB, s)
    finally:
        ozimmu.debug_small_tile_limit(-1)
    assert bool(torch.equal(C, C2)), f"{tag}: the two tile shapes differ"


def test_full_size_pow2_scaled_8192():
    cfg = workloads.CONFIGS["pow2_scaled_8192"]
    A, B = cfg["gen"]()
    dA, dB = ozimmu.to_colmajor(A), ozimmu.to_colmajor(B)
    m, n = dA.shape[0], dB.shape[1]
    for s in cfg["s"]:                       # 2 ... 9: every slice count of the benchmark's sweep
        print("pow2_scaled_8192 s =", s, flush=True)
        C = check_sampled(dA, dB, s, f"pow2_scaled_8192 s={s}")
        # a tile-aligned 256 x 256 block across the corner where four tile regions meet
        check_block(dA, dB, C, s, 3 * m // 4 - 128, n // 2 - 128, 256, f"pow2_scaled_8192 s={s}")
        check_whole_matrix_against_other_tile_shape(dA, dB, C, s, f"pow2_scaled_8192 s={s}")


def test_power_of_two_scaling_is_removed_exactly_at_full_size():
    # the row / column scalings of this workload only shift exponents: C must equal the product of
    # the unscaled base matrices times the same powers of two, bit for bit
    m = n = k = 2048
    A, B = workloads.pow2_scaled(m, n, k, 30, 77)
    ea = np.floor(np.log2(np.abs(A).max(axis=1))).astype(np.int64)
    eb = np.floor(np.log2(np.abs(B).max(axis=0))).astype(np.int64)
    A0 = A * np.ldexp(1.0, -ea)[:, None]
    B0 = B * np.ldexp(1.0, -eb)[None, :]
    C = ozimmu.dgemm(ozimmu.to_colmajor(A), ozimmu.to_colmajor(B), 7).cpu().numpy()
    C0 = ozimmu.dgemm(ozimmu.to_colmajor(A0), ozimmu.to_colmajor(B0), 7).cpu().numpy()
    assert np.array_equal(C, C0 * np.ldexp(1.0, ea)[:, None] * np.ldexp(1.0, eb)[None, :])


def test_full_size_lognormal_4096():
    cfg = workloads.CONFIGS["lognormal_4096"]
    A, B = cfg["gen"]()
    dA, dB = ozimmu.to_colmajor(A), ozimmu.to_colmajor(B)
    s_est, status, kA, kB = ozimmu.estimate_slices(dA, dB, 2.0 ** -53)
    assert (s_est, status, kA, kB) == oracle.estimate_slices(A, B, 2.0 ** -53, s_max=ozimmu.MAX_SLICES)
    for s in sorted(set(cfg["s"] + [s_est])):
        print("lognormal_4096 s =", s, flush=True)
        check_sampled(dA, dB, s, f"lognormal_4096 s={s}")


def test_full_size_long_k_forces_k_blocking():
    # k = 262144: a single int32 sum would overflow (k * 127^2 > 2^31); inputs drawn on the device
    dA, dB = workloads.lognormal_device(2048, 2048, 262144, 2.0, 1004)
    print("long-k inputs ready", flush=True)
    check_sampled(dA, dB, 7, "lognormal_longk s=7")


def check_sampled_variant(dA, dB, sA, sB, allp, nearest, Q, tag):
    m, k = dA.shape
    n = dB.shape[1]
    C = ozimmu.dgemm3(dA, dB, sA, sB, allp, ozimmu.SPLIT_NEAREST if nearest else ozimmu.SPLIT_TRUNCATE, Q,
                      check_finite=True)
    rows, cols = sample_indices(m, 3, 12), sample_indices(n, 4, 12)
    tr, tc = torch.as_tensor(rows, device="cuda"), torch.as_tensor(cols, device="cuda")
    want = oracle.dgemm3(dA[tr, :].cpu().numpy(), dB[:, tc].cpu().numpy(), sA, sB, full=allp, nearest=nearest, Q=Q)
    got = C[tr][:, tc].cpu().numpy()
    assert np.array_equal(got, want), f"{tag}: not bit-identical"


def test_full_size_variants_8192():
    # the 16x16x64 kernel (s = 4, 7, 8), nearest slices, levels, different slice counts, the four-wavefront shape (13),
    # all products, and the blocks of slice groups over their 13 ... 16 column panels at the benchmark size: groups of
    # 9 (18), 7 (21, through the 32x32x32 kernel), 8 (24, 32, (25, 31)), different group counts ((20, 7)), all
    # products of (16, 16)
    cfg = workloads.CONFIGS["pow2_scaled_8192"]
    A, B = cfg["gen"]()
    dA, dB = ozimmu.to_colmajor(A), ozimmu.to_colmajor(B)
    qmax = ozimmu.max_level_diagonals(8192, 7, 7)
    assert qmax == 4
    for sA, sB, allp, nearest, Q in [(4, 4, False, False, 1), (8, 8, False, True, 3), (7, 7, False, True, qmax),
                                     (5, 10, False, False, 3), (13, 13, False, True, 3), (3, 4, True, False, 2),
                                     (18, 18, False, False, 2), (6, 6, True, False, 1), (21, 21, False, False, 1),
                                     (24, 24, False, False, 1), (32, 32, False, True, 3), (25, 31, False, False, 1),
                                     (20, 7, False, False, 1), (16, 16, True, False, 1)]:
        print(f"variant sA={sA} sB={sB} all={allp} nearest={nearest} Q={Q}", flush=True)
        check_sampled_variant(dA, dB, sA, sB, allp, nearest, Q, f"8192 ({sA},{sB}) all={allp} nearest={nearest} Q={Q}")


def test_large_ragged_shapes():
    # no dimension a multiple of any tile or stage size; several kernels of the family
    m, n, k = 5003, 7001, 3001
    dA, dB = workloads.lognormal_device(m, n, k, 1.0, 2024)
    for sA, sB, allp, nearest, Q in [(7, 7, False, False, 1), (14, 14, False, False, 3), (5, 10, False, True, 2),
                                     (6, 6, True, False, 1), (22, 22, False, False, 1), (4, 4, False, False, 1),
                                     (7, 8, False, False, 1)]:
        print(f"ragged sA={sA} sB={sB} all={allp} nearest={nearest} Q={Q}", flush=True)
        check_sampled_variant(dA, dB, sA, sB, allp, nearest, Q, f"ragged ({sA},{sB}) all={allp}")


def test_more_than_two_to_the_31_entries_of_C():
    # 46400 x 46400 (2.15e9 entries, 17 GB): element offsets of C, and of the int64 totals of the block path,
    # pass 2^31; short k keeps the products cheap.  The sampled rows and columns include the last ones.
    m = n = 46400
    k = 192
    dA, dB = workloads.lognormal_device(m, n, k, 1.0, 2026)
    for s in (2, 7, 12, 24):
        print(f"2^31 entries s={s}", flush=True)
        C = check_sampled(dA, dB, s, f"46400x46400x192 s={s}")
        assert bool(torch.isfinite(C[:, -1]).all()) and bool(torch.isfinite(C[-1, :]).all())
        del C
        torch.cuda.empty_cache()


def test_more_than_two_to_the_31_entries_of_A():
    # 16421 x 140001 (2.3e9 entries, 18 GB; its slice planes up to 16 GB): element offsets of an operand and byte
    # offsets of its planes pass 2^31 and 2^32, and k is long enough to need k-blocks; nothing a multiple of a tile
    m, n, k = 16421, 200, 140001
    dA, dB = workloads.lognormal_device(m, n, k, 1.0, 2027)
    for s in (3, 7):
        print(f"2^31 entries of A s={s}", flush=True)
        C = check_sampled(dA, dB, s, f"16421x200x140001 s={s}")
        del C
        torch.cuda.empty_cache()


def test_uneven_regions_of_the_two_dimensional_tile_order():
    # 63 tile rows of 128: the four row bands of the XCD grid hold 15, 16, 16, 16 tile rows, the launch is padded
    # to 8 x the largest region and the surplus work-groups must leave without touching anything
    m, n, k = 8057, 1000, 700
    dA, dB = workloads.lognormal_device(m, n, k, 1.0, 2025)
    for s in (7, 4, 10, 13):
        print(f"uneven regions s={s}", flush=True)
        check_sampled_variant(dA, dB, s, s, False, False, 1, f"uneven regions s={s}")
    # every entry, not only the sampled ones: the kernel with the 64 x 64 tile (another tile grid, other regions)
    # must give the same matrix bit for bit, and the sampled entries of one of them are the oracle's
    for s in (7, 4, 10):
        C1 = ozimmu.dgemm(dA, dB, s)
        try:
            ozimmu.debug_small_tile_limit(1 << 40)
            C2 = ozimmu.dgemm(dA, dB, s)
        finally:
            ozimmu.debug_small_tile_limit(-1)
        assert not bool(torch.isnan(C1).any()) and bool(torch.equal(C1, C2)), f"uneven regions s={s}: tile shapes differ"

