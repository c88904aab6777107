"""The paper's second accuracy workload on the GPU (Section 4.2, zero-cancellation evaluation): a
Gaussian matrix times its computed inverse, measured against the double-double product. With enough
slices the Ozaki product must be more accurate than the vendor FP64 GEMM on the same device."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_11975_amd import ozimmu

pytestmark = pytest.mark.gpu


def avg_rel_error(C, hi, lo):
    return float(np.mean(np.abs((C - hi) - lo) / np.abs(hi)))


def test_zero_cancellation_beats_native_fp64_gemm():
    n = 768
    g = torch.Generator(device="cuda")
    g.manual_seed(43)
    A = torch.randn((n, n), generator=g, device="cuda", dtype=torch.float64)
    X = torch.linalg.solve(A, torch.eye(n, dtype=torch.float64, device="cuda")).contiguous()
    Ah, Xh = A.cpu().numpy(), X.cpu().numpy()
    hi, lo = oracle.dd_gemm(Ah, Xh)
    e_native = avg_rel_error(torch.matmul(A, X).cpu().numpy(), hi, lo)
    errs = {}
    for s in (8, 10, 12, 13):
        C = torch.empty((n, n), dtype=torch.float64, device="cuda")
        ozimmu.dgemm(A, X, C, s, ozimmu.alloc_workspace(n, n, n, s))
        torch.cuda.synchronize()
        got = C.cpu().numpy()
        errs[s] = avg_rel_error(got, hi, lo)
        rows = np.arange(0, n, 97)
        assert np.array_equal(got[rows].view(np.uint64), oracle.dgemm(Ah[rows], Xh, s).view(np.uint64))
    assert errs[13] < e_native and errs[12] < e_native, (errs, e_native)
    assert errs[13] <= errs[12] <= errs[10] <= errs[8]
