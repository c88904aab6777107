"""Seeded synthetic inputs with the shapes and value distributions of the paper's workloads.

This module holds input recipes only -- none of the method's arithmetic -- so that the CPU
oracle's tests and the GPU path's tests and benchmark can draw the same matrices.

* ``phi_matrix``: the accuracy experiment's generator, Eq. (6) of Section 4.2:
  element = uniform(-0.5, 0.5) * exp(phi * normal(0, 1)).
* ``gaussian_complex`` / ``unit_column_complex``: Gaussian complex matrices, the second with
  every column scaled to unit 2-norm; stands in for the d-qubit gate applied to a reshaped
  state vector in Section 4.4 (matmul-(2^(N-d), 2^d, 2^d)).
* adversarial sets used by the parity tests (saturating slices, powers of two, zero rows and
  columns, one dominant element per row, subnormals).

Host versions use ``numpy.random.default_rng(seed)``; device versions use a seeded
``torch.Generator`` on the GPU (rows and columns are then copied back for the oracle).
"""
from __future__ import annotations

import numpy as np

# (name, m, n, k, phi, slice counts, complex) -- the five configurations of the build's baseline
CONFIGS = {
    "c1_64": dict(m=64, n=64, k=64, phi=0.5, slices=(3, 5, 7), complex=False),
    "c2_1024": dict(m=1024, n=1024, k=1024, phi=(0.5, 1.0, 2.0), slices=tuple(range(3, 14)), complex=False),
    "c3_8192": dict(m=8192, n=8192, k=8192, phi=1.0, slices=(6, 8, 10), complex=False),
    "c4_longk": dict(m=4096, n=4096, k=131072, phi=2.0, slices=(8,), complex=False),
    "c5_complex": dict(m=4096, n=4096, k=256, phi=None, slices=(7,), complex=True),
}


def phi_matrix(rows: int, cols: int, phi: float, seed: int) -> np.ndarray:
    """Eq. (6): (U(0,1) - 0.5) * exp(phi * N(0,1)), FP64, row-major."""
    rng = np.random.default_rng(seed)
    u = rng.random((rows, cols))
    g = rng.standard_normal((rows, cols))
    return (u - 0.5) * np.exp(phi * g)


def phi_pair(m: int, n: int, k: int, phi: float, seed: int):
    """A (m x k) from seed 1000+seed, B (k x n) from seed 2000+seed."""
    return phi_matrix(m, k, phi, 1000 + seed), phi_matrix(k, n, phi, 2000 + seed)


def gaussian_complex(rows: int, cols: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.standard_normal((rows, cols)) + 1j * rng.standard_normal((rows, cols))


def unit_column_complex(rows: int, cols: int, seed: int) -> np.ndarray:
    z = gaussian_complex(rows, cols, seed)
    return z / np.sqrt((np.abs(z) ** 2).sum(axis=0, keepdims=True))


def integer_matrix(rows: int, cols: int, seed: int, bound: int = 127) -> np.ndarray:
    """Integer-valued FP64 matrix with |entry| <= bound (lives entirely in slice 1)."""
    rng = np.random.default_rng(seed)
    return rng.integers(-bound, bound + 1, size=(rows, cols)).astype(np.float64)


def saturating_matrix(rows: int, cols: int) -> np.ndarray:
    """All entries 1 - 2^-53: every slice chunk of every element is 127."""
    return np.full((rows, cols), 1.0 - 2.0 ** -53)


def adversarial_matrix(rows: int, cols: int, seed: int) -> np.ndarray:
    """Mix of cases the splitter must survive: a zero row, a zero column, exact powers of
    two, one dominant element per row, subnormals, negative zero, huge and tiny rows."""
    rng = np.random.default_rng(seed)
    M = (rng.random((rows, cols)) - 0.5) * np.exp(2.0 * rng.standard_normal((rows, cols)))
    if rows > 0 and cols > 0:
        M[0, :] = 0.0                                   # zero row
        M[:, cols // 2] = 0.0                           # zero column
    if rows > 1:
        M[1, :] = np.ldexp(1.0, rng.integers(-8, 8, size=cols)) * rng.choice([-1.0, 1.0], size=cols)
    if rows > 2:
        M[2, :] *= 1e-12
        M[2, cols // 3] = 3.0e9                         # one dominant element
    if rows > 3:
        M[3, :] = rng.integers(1, 1 << 20, size=cols) * 4.9406564584124654e-324  # subnormals
    if rows > 4:
        M[4, :] = -0.0
        M[4, 0] = 2.0 ** -1074
    if rows > 5:
        M[5, :] *= 2.0 ** 1000                          # near the top of the range
    if rows > 6:
        M[6, :] *= 2.0 ** -1000
    if rows > 7:
        M[7, :] = 1.0 - 2.0 ** -53                      # saturating chunks
    if rows > 8:
        M[8, :] = 2.0 ** 10                             # exact power of two as row maximum
    return M


# ----------------------------------------------------------------------------- device side
def phi_matrix_device(rows: int, cols: int, phi: float, seed: int, device="cuda"):
    """Eq. (6) generated on the GPU with a seeded torch.Generator (FP64)."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed)
    u = torch.rand((rows, cols), generator=g, device=device, dtype=torch.float64)
    z = torch.randn((rows, cols), generator=g, device=device, dtype=torch.float64)
    return (u - 0.5) * torch.exp(phi * z)


def unit_column_complex_device(rows: int, cols: int, seed: int, device="cuda"):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed)
    re = torch.randn((rows, cols), generator=g, device=device, dtype=torch.float64)
    im = torch.randn((rows, cols), generator=g, device=device, dtype=torch.float64)
    z = torch.complex(re, im)
    return z / torch.sqrt((z.abs() ** 2).sum(dim=0, keepdim=True))


def gaussian_complex_device(rows: int, cols: int, seed: int, device="cuda"):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed)
    re = torch.randn((rows, cols), generator=g, device=device, dtype=torch.float64)
    im = torch.randn((rows, cols), generator=g, device=device, dtype=torch.float64)
    return torch.complex(re, im)


def haar_unitary_device(dim: int, seed: int, device="cuda"):
    """A Haar-distributed dim x dim unitary (QR of a complex Gaussian matrix with the phases of R's
    diagonal divided out): the random gates of the circuit workload of Section 4.4."""
    import torch

    g = torch.Generator().manual_seed(seed)
    z = torch.complex(torch.randn((dim, dim), generator=g, dtype=torch.float64),
                      torch.randn((dim, dim), generator=g, dtype=torch.float64))
    q, r = torch.linalg.qr(z)
    d = torch.diagonal(r)
    return (q * (d / d.abs())).to(device)
