"""Seeded synthetic inputs shaped like the paper's experiments.

This module only draws random matrices; it holds none of the method's arithmetic, so the
CPU oracle's tests and the GPU path's tests can both take their inputs from it.

Every generator returns ``(A, B)`` as float64 numpy arrays in column-major (Fortran)
order, ``A`` m-by-k and ``B`` k-by-n, drawn from ``numpy.random.default_rng(seed)``
(``A`` first, then ``B``).

Recipes (they stand in for data the paper does not ship):
  uniform        entries U[-1, 1)                      -- like the DLARNV squares of the
                                                          GPU benchmark section, signed
  lognormal      (U(0,1) - 0.5) * exp(phi * N(0,1))    -- eq. (rand-mat)
  pow2_scaled    U[-1,1) base, row i of A times 2^a_i, column j of B times 2^b_j,
                 a_i, b_j uniform integers in [-spread, spread]
  diag_scaled    A = Abar D, B = D^{-1} Bbar, Abar, Bbar ~ U(1,2), D geometric diagonal with
                 d_11 = kappa_D^{-1/2}, d_nn = kappa_D^{1/2}; optional circular rotation of
                 row i of A and column i of B by i places -- the badly scaled test of the
                 GPU benchmark section
"""
import numpy as np


def _fortran(rng_fill, rows, cols):
    """Fill a rows-by-cols column-major array column block by column block."""
    out = np.empty((cols, rows), dtype=np.float64)  # C-order (cols, rows) == F-order (rows, cols)
    step = max(1, (1 << 24) // max(rows, 1))
    for c0 in range(0, cols, step):
        c1 = min(cols, c0 + step)
        out[c0:c1, :] = rng_fill((c1 - c0, rows))
    return out.T


def uniform(m, n, k, seed):
    rng = np.random.default_rng(seed)
    f = lambda shape: rng.random(shape) * 2.0 - 1.0
    return _fortran(f, m, k), _fortran(f, k, n)


def lognormal(m, n, k, phi, seed):
    rng = np.random.default_rng(seed)

    def f(shape):
        u = rng.random(shape) - 0.5
        z = rng.standard_normal(shape)
        return u * np.exp(phi * z)

    return _fortran(f, m, k), _fortran(f, k, n)


def pow2_scaled(m, n, k, spread, seed):
    rng = np.random.default_rng(seed)
    f = lambda shape: rng.random(shape) * 2.0 - 1.0
    A = _fortran(f, m, k)
    B = _fortran(f, k, n)
    a = rng.integers(-spread, spread + 1, size=m)
    b = rng.integers(-spread, spread + 1, size=n)
    A *= np.ldexp(1.0, a)[:, None]
    B *= np.ldexp(1.0, b)[None, :]
    return A, B


def diag_scaled(n, kappa_d, seed, rotate=True):
    rng = np.random.default_rng(seed)
    f = lambda shape: rng.random(shape) + 1.0
    Abar = _fortran(f, n, n)
    Bbar = _fortran(f, n, n)
    if n > 1:
        d = kappa_d ** (-0.5 + np.arange(n) / (n - 1))
    else:
        d = np.ones(1)
    A = np.asfortranarray(Abar * d[None, :])
    B = np.asfortranarray(Bbar / d[:, None])
    if rotate:
        for i in range(n):
            A[i, :] = np.roll(A[i, :], i + 1)
            B[:, i] = np.roll(B[:, i], i + 1)
    return A, B


def lognormal_device(m, n, k, phi, seed, device="cuda"):
    """Same recipe as lognormal(), drawn on the GPU with torch's generator (for inputs too large to
    draw on the host in reasonable time).  Returns column-major torch tensors; a different random
    stream than lognormal(), so the two are not interchangeable for a given seed."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)

    def draw(rows, cols):
        out = torch.empty((cols, rows), dtype=torch.float64, device=device)   # column-major rows x cols
        step = max(1, (1 << 26) // max(rows, 1))
        for c0 in range(0, cols, step):
            c1 = min(cols, c0 + step)
            u = torch.rand((c1 - c0, rows), dtype=torch.float64, device=device, generator=g) - 0.5
            z = torch.randn((c1 - c0, rows), dtype=torch.float64, device=device, generator=g)
            out[c0:c1] = u * torch.exp(phi * z)
        return out.t()

    return draw(m, k), draw(k, n)


# The five benchmark configurations: name -> (generator thunk, slice counts)
CONFIGS = {
    "uniform_128": dict(m=128, n=128, k=128, gen=lambda: uniform(128, 128, 128, 1000), s=[3]),
    "lognormal_1024": dict(m=1024, n=1024, k=1024, gen=lambda: lognormal(1024, 1024, 1024, 0.5, 1001),
                           s=list(range(2, 9))),
    "lognormal_4096": dict(m=4096, n=4096, k=4096, gen=lambda: lognormal(4096, 4096, 4096, 1.0, 1002),
                           s=[7, 8, 9]),
    "pow2_scaled_8192": dict(m=8192, n=8192, k=8192, gen=lambda: pow2_scaled(8192, 8192, 8192, 30, 1003),
                             s=list(range(2, 10))),
    "lognormal_longk": dict(m=2048, n=2048, k=262144, gen=lambda: lognormal(2048, 2048, 262144, 2.0, 1004),
                            s=[7]),
}
