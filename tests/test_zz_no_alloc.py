"""ozimmu_dgemm_static (the entry point that allocates nothing, its workspace a static device array inside the
library) against ozimmu_dgemm with a caller-owned workspace, through the C ABI: bit-identical C on two calls in a
row, the second with a smaller input, then a k-blocked call; sizes beyond the static array are refused; the call
recorded into a HIP graph and replayed."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2506_11277_amd import ozimmu, workloads


def both_ways(m, n, k, s, seed):
    A, B = workloads.lognormal(m, n, k, 1.0, seed)
    dA, dB = ozimmu.to_colmajor(A), ozimmu.to_colmajor(B)
    handle = ozimmu.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # existing entry point, workspace from torch
    ws = ozimmu.alloc_workspace(m, n, k, s)
    C0 = ozimmu.colmajor_empty(m, n)
    C0.fill_(float("nan"))
    rc = handle.ozimmu_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, C0.data_ptr(), m, s, ws.data_ptr(),
                             ws.numel(), stream)
    assert rc == ozimmu.OK
    # the new one: inputs and outputs only
    C1 = ozimmu.colmajor_empty(m, n)
    C1.fill_(float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = handle.ozimmu_dgemm_static(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, C1.data_ptr(), m, s, stream)
    assert rc == ozimmu.OK
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    c0, c1 = C0.cpu().numpy(), C1.cpu().numpy()
    assert np.isfinite(c0).all()
    diff = np.abs(c1 - c0)
    rel = float(np.max(np.where(diff == 0, 0.0, diff / np.abs(c0)))) if c0.size else 0.0
    assert rel <= 1e-15, f"relative difference {rel:.3e}"
    assert np.array_equal(c0, c1), "within 1e-15 but not bit-identical"


def test_static_workspace_entry_point_matches_dgemm_on_consecutive_calls():
    both_ways(300, 200, 500, 7, 4101)        # several tiles, ragged edges
    both_ways(100, 70, 130, 5, 4102)         # smaller: the array still holds the planes of the call before
    both_ways(64, 96, 20000, 9, 4103)        # 9 * 20000 > 133144: k cut into blocks, int64 totals in the array
    both_ways(130, 129, 257, 24, 4104)       # 24 slices: blocks of slice groups, int64 totals
    both_ways(300, 200, 500, 7, 4101)        # the first case once more


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    handle = ozimmu.lib()
    fake = ctypes.c_void_p(4096)
    assert handle.ozimmu_workspace_bytes(4096, 4096, 4096, 7) > ozimmu.STATIC_WORKSPACE_BYTES
    assert handle.ozimmu_dgemm_static(4096, 4096, 4096, fake, 4096, fake, 4096, fake, 4096, 7, None) == ozimmu.TOO_LARGE
    assert handle.ozimmu_status_string(ozimmu.TOO_LARGE) == b"problem too large for the static workspace"
    assert handle.ozimmu_dgemm_static(4, 4, 4, fake, 4, fake, 4, fake, 4, 0, None) == ozimmu.BAD_ARG
    assert handle.ozimmu_dgemm_static(4, 4, 4, fake, 3, fake, 4, fake, 4, 2, None) == ozimmu.BAD_ARG


@pytest.mark.parametrize("shape,s", [((128, 128, 128), 3), ((300, 200, 500), 7), ((64, 96, 20000), 9),
                                     ((130, 129, 257), 24)])
def test_static_entry_point_replays_from_a_captured_graph(shape, s):
    # One of the callers the entry point is for: the whole call (scales, slices, products, accumulation; for long k
    # and for 24 slices also the clearing of the int64 totals) recorded into a graph, replayed several times with
    # eager calls of other sizes -- which overwrite the shared static array -- in between; every replay must give
    # the eager result bit for bit.
    m, n, k = shape
    A, B = workloads.lognormal(m, n, k, 1.0, 4200 + s)
    dA, dB = ozimmu.to_colmajor(A), ozimmu.to_colmajor(B)
    want = ozimmu.dgemm(dA, dB, s)
    C = ozimmu.colmajor_empty(m, n)
    ozimmu.dgemm_static(dA, dB, s, C)         # outside capture: symbol address and kernel attributes are set up
    torch.cuda.synchronize()
    assert bool(torch.equal(C, want))
    A2, B2 = workloads.lognormal(90, 110, 70, 1.0, 4300 + s)
    dA2, dB2 = ozimmu.to_colmajor(A2), ozimmu.to_colmajor(B2)
    C2 = ozimmu.colmajor_empty(90, 110)
    graph = torch.cuda.CUDAGraph()
    print(f"capture {shape} s={s}", flush=True)
    with torch.cuda.graph(graph):
        ozimmu.dgemm_static(dA, dB, s, C)
    for rep in range(4):
        C.fill_(float("nan"))
        ozimmu.dgemm_static(dA2, dB2, 5 + rep, C2)     # eager work on the same static array between the replays
        torch.cuda.synchronize()
        print(f"replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert bool(torch.equal(C, want)), f"replay {rep} differs from the eager call"
