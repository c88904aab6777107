"""Double-double summing-up on the GPU (Section 2.3.4) against the oracle, bit for bit in both parts,
and its accuracy beyond FP64 against the double-double reference product."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_11975_amd import ozimmu
from paper_2306_11975_amd import workloads as wl

pytestmark = pytest.mark.gpu


def bits(x):
    return np.ascontiguousarray(x).view(np.uint64)


def gpu_dd(A, B, s, pad=0):
    m, k = A.shape
    n = B.shape[1]
    dA = torch.from_numpy(np.ascontiguousarray(A)).cuda()
    dB = torch.from_numpy(np.ascontiguousarray(B)).cuda()
    buf = torch.full((2, m, n + pad), float("nan"), dtype=torch.float64, device="cuda")
    hi, lo = buf[0, :, :n], buf[1, :, :n]
    ozimmu.dgemm_dd(dA, dB, hi, lo, s, ozimmu.alloc_workspace(m, n, k, s))
    torch.cuda.synchronize()
    if pad:
        assert torch.isnan(buf[:, :, n:]).all()
    return hi.cpu().numpy(), lo.cpu().numpy()


@pytest.mark.parametrize("m,n,k,s,phi,seed", [(64, 64, 64, 7, 0.5, 1), (300, 270, 517, 13, 1.0, 2),
                                              (257, 130, 1300, 16, 2.0, 3), (40, 50, 70000, 3, 2.0, 4),
                                              (1, 1, 1, 1, 1.0, 5)])
def test_dd_sum_bit_exact(m, n, k, s, phi, seed):
    A, B = wl.phi_pair(m, n, k, phi, seed)
    hi, lo = gpu_dd(A, B, s, pad=3)
    whi, wlo = oracle.dgemm_dd(A, B, s)
    assert np.array_equal(bits(hi), bits(whi))
    assert np.array_equal(bits(lo), bits(wlo))


def test_dd_sum_is_more_accurate_than_fp64():
    n = 512
    A, B = wl.phi_pair(n, n, n, 0.5, seed=7)
    rhi, rlo = oracle.dd_gemm(A, B)            # reference product in double-double
    G = oracle.abs_gemm(A, B)
    hi, lo = gpu_dd(A, B, 14)
    err_dd = np.max(np.abs(((hi - rhi) + (lo - rlo))) / G)
    dC = torch.empty((n, n), dtype=torch.float64, device="cuda")
    ozimmu.dgemm(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), dC, 14, ozimmu.alloc_workspace(n, n, n, 14))
    torch.cuda.synchronize()
    C64 = dC.cpu().numpy()
    err_64 = np.max(np.abs((C64 - rhi) - rlo) / G)
    assert err_dd <= 2.0 ** -70, err_dd
    assert err_64 >= 2.0 ** -62 and err_64 <= 2.0 ** -50


def test_dd_degenerate():
    hi = torch.full((3, 4), float("nan"), dtype=torch.float64, device="cuda")
    lo = torch.full((3, 4), float("nan"), dtype=torch.float64, device="cuda")
    ozimmu.dgemm_dd(torch.empty((3, 0), dtype=torch.float64, device="cuda"),
                    torch.empty((0, 4), dtype=torch.float64, device="cuda"), hi, lo, 5,
                    torch.empty(256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert not hi.cpu().numpy().any() and not lo.cpu().numpy().any()
