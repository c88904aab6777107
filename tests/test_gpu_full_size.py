"""Parity at the full size of the large workloads, in the launch configuration the benchmark times.

An entry C_ij depends only on row i of A and column j of B, so the oracle run on a few rows of A
against all of B reproduces exactly those rows of the full result: the sampled rows (one in every
64-row tile of C, tile edges, and random ones) must be bit-exact. Inputs are generated on the device
from a seed and the sampled rows copied back for the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_11975_amd import ozimmu
from paper_2306_11975_amd import workloads as wl

pytestmark = pytest.mark.gpu


def bits(x):
    return np.ascontiguousarray(x).view(np.uint64)


TILE_ROWS = 64   # rows of C one workgroup owns


def sample_rows(m, extra, seed, every_tile=False):
    edges = [0, 1, 63, 64, 127, 128, 255, 256, m // 2 - 1, m // 2, m - 257, m - 256, m - 65, m - 64, m - 1]
    rng = np.random.default_rng(seed)
    rows = set(int(r) for r in edges if 0 <= r < m) | set(int(r) for r in rng.choice(m, size=extra, replace=False))
    if every_tile:   # one row at a random position inside every tile row
        rows |= set(int(t * TILE_ROWS + rng.integers(0, min(TILE_ROWS, m - t * TILE_ROWS)))
                    for t in range((m + TILE_ROWS - 1) // TILE_ROWS))
    return np.array(sorted(rows), dtype=np.int64)


@pytest.fixture(scope="module")
def config3():
    m = n = k = 8192
    A = wl.phi_matrix_device(m, k, 1.0, 1003)
    B = wl.phi_matrix_device(k, n, 1.0, 2003)
    rows = sample_rows(m, 13, seed=3, every_tile=True)
    assert len(set(rows // TILE_ROWS)) == m // TILE_ROWS
    A_rows = A[torch.from_numpy(rows).cuda()].cpu().numpy()
    B_host = B.cpu().numpy()
    yield A, B, rows, A_rows, B_host
    del A, B
    torch.cuda.empty_cache()


@pytest.mark.parametrize("s", [6, 8, 10])
def test_config3_8192_cubed_sampled_rows_bit_exact(config3, s):
    A, B, rows, A_rows, B_host = config3
    m, k = A.shape
    n = B.shape[1]
    C = torch.full((m, n), float("nan"), dtype=torch.float64, device="cuda")
    ws = ozimmu.alloc_workspace(m, n, k, s)
    ozimmu.dgemm(A, B, C, s, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(C).any()
    got = C[torch.from_numpy(rows).cuda()].cpu().numpy()
    want = oracle.dgemm(A_rows, B_host, s)
    assert np.array_equal(bits(got), bits(want))
    # sampled accuracy against the double-double product, scaled by (|A||B|): below 2^-50 once s is large
    if s == 10:
        hi, lo = oracle.dd_gemm(A_rows, B_host)
        scale = oracle.abs_gemm(A_rows, B_host)
        assert np.max(np.abs((got - hi) - lo) / scale) <= 2.0 ** -50


def test_config4_long_k_wide_exponents_sampled_rows_bit_exact():
    """m = n = 4096, k = 131072, phi = 2, s = 8: every diagonal spans several INT32 blocks (INT64 sums)."""
    m, n, k, s = 4096, 4096, 131072, 8
    A = wl.phi_matrix_device(m, k, 2.0, 1004)
    B = wl.phi_matrix_device(k, n, 2.0, 2004)
    C = torch.full((m, n), float("nan"), dtype=torch.float64, device="cuda")
    ws = ozimmu.alloc_workspace(m, n, k, s)
    ozimmu.dgemm(A, B, C, s, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(C).any()
    rows = sample_rows(m, 0, seed=4, every_tile=True)
    assert len(set(rows // TILE_ROWS)) == m // TILE_ROWS
    A_rows = A[torch.from_numpy(rows).cuda()].cpu().numpy()
    got = C[torch.from_numpy(rows).cuda()].cpu().numpy()
    del A, C, ws
    B_host = B.cpu().numpy()
    del B
    torch.cuda.empty_cache()
    want = oracle.dgemm(A_rows, B_host, s)
    assert np.array_equal(bits(got), bits(want))


def test_config5_complex_small_k_sampled_rows_bit_exact():
    """Complex m = n = 4096, k = 256, s = 7: Gaussian A, unit-norm columns of B."""
    m, n, k, s = 4096, 4096, 256, 7
    A = wl.gaussian_complex_device(m, k, 1005)
    B = wl.unit_column_complex_device(k, n, 2005)
    C = torch.full((m, n), complex(float("nan"), float("nan")), dtype=torch.complex128, device="cuda")
    ws = ozimmu.alloc_workspace(m, n, k, s, is_complex=True)
    ozimmu.zgemm(A, B, C, s, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(torch.view_as_real(C)).any()
    rows = sample_rows(m, 117, seed=5)
    idx = torch.from_numpy(rows).cuda()
    got = C[idx].cpu().numpy()
    want = oracle.zgemm(A[idx].cpu().numpy(), B.cpu().numpy(), s)
    assert np.array_equal(bits(got.real.copy()), bits(want.real.copy()))
    assert np.array_equal(bits(got.imag.copy()), bits(want.imag.copy()))


@pytest.mark.parametrize("size,s", [(2048, 8), (3072, 7), (6144, 8)])
def test_tile_counts_that_do_not_fill_the_chip_sampled_rows_bit_exact(size, s):
    """512, 1152 and 4608 tiles on 256 CUs: 2, 4.5 and 18 rounds of workgroups, the last one partial at 3072."""
    m = n = k = size
    A = wl.phi_matrix_device(m, k, 1.0, 1006)
    B = wl.phi_matrix_device(k, n, 1.0, 2006)
    C = torch.full((m, n), float("nan"), dtype=torch.float64, device="cuda")
    ozimmu.dgemm(A, B, C, s, ozimmu.alloc_workspace(m, n, k, s))
    torch.cuda.synchronize()
    assert not torch.isnan(C).any()
    rows = sample_rows(m, 9, seed=size)
    idx = torch.from_numpy(rows).cuda()
    want = oracle.dgemm(A[idx].cpu().numpy(), B.cpu().numpy(), s)
    assert np.array_equal(bits(C[idx].cpu().numpy()), bits(want))


@pytest.mark.parametrize("s", range(1, 10))
def test_large_tile_kernels_up_to_nine_slices_sampled_rows_bit_exact(s):
    """Small shapes take 64 x 64 tiles up to nine slices; this one has 256 tiles of 64 x 128 and k > 512, so it
    runs the 64 x 128 kernels that the small parity cases no longer reach."""
    m, n, k = 1024, 2048, 544
    assert ozimmu.launch_plan(m, n, k, s)["tile_cols"] == 128
    A = wl.phi_matrix_device(m, k, 1.0, 1007)
    B = wl.phi_matrix_device(k, n, 1.0, 2007)
    C = torch.full((m, n), float("nan"), dtype=torch.float64, device="cuda")
    ozimmu.dgemm(A, B, C, s, ozimmu.alloc_workspace(m, n, k, s))
    torch.cuda.synchronize()
    assert not torch.isnan(C).any()
    rows = sample_rows(m, 5, seed=s, every_tile=True)
    idx = torch.from_numpy(rows).cuda()
    want = oracle.dgemm(A[idx].cpu().numpy(), B.cpu().numpy(), s)
    assert np.array_equal(bits(C[idx].cpu().numpy()), bits(want))


def test_small_tiles_are_chosen_for_short_k_and_for_grids_that_underfill_the_chip():
    assert ozimmu.launch_plan(4096, 4096, 256, 7)["tile_cols"] == 64      # short inner dimension
    assert ozimmu.launch_plan(1024, 1024, 1024, 8)["tile_cols"] == 64     # 128 tiles of 64 x 128 for 256 compute units
    assert ozimmu.launch_plan(4096, 4096, 4096, 8)["tile_cols"] == 128
    assert ozimmu.launch_plan(1024, 1024, 1024, 10)["tile_cols"] == 128   # no small kernels beyond nine slices
    assert ozimmu.launch_plan(64, 64, 200000, 2)["tile_cols"] == 128      # k-blocking keeps the large tiles


@pytest.mark.parametrize("m,n,k,s,cols", [(1024, 2048, 512, 8, 64), (960, 2048, 600, 5, 64), (1024, 2048, 600, 9, 128),
                                          (1000, 1000, 1000, 9, 64), (1000, 1000, 1000, 10, 128)])
def test_both_sides_of_the_tile_choice_sampled_rows_bit_exact(m, n, k, s, cols):
    """Shapes just on either side of the rule that picks 64 x 64 tiles (k <= 512, or fewer than 256 tiles of
    64 x 128, up to nine slices), with ragged edges."""
    assert ozimmu.launch_plan(m, n, k, s)["tile_cols"] == cols
    A = wl.phi_matrix_device(m, k, 1.0, 1008)
    B = wl.phi_matrix_device(k, n, 1.0, 2008)
    C = torch.full((m, n), float("nan"), dtype=torch.float64, device="cuda")
    ozimmu.dgemm(A, B, C, s, ozimmu.alloc_workspace(m, n, k, s))
    torch.cuda.synchronize()
    assert not torch.isnan(C).any()
    rows = sample_rows(m, 5, seed=s + k, every_tile=True)
    idx = torch.from_numpy(rows).cuda()
    want = oracle.dgemm(A[idx].cpu().numpy(), B.cpu().numpy(), s)
    assert np.array_equal(bits(C[idx].cpu().numpy()), bits(want))
