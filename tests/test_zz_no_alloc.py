"""ozimmu_dgemm_static (the entry point for callers that cannot allocate or pass a workspace) against
ozimmu_dgemm with a caller-owned workspace: same bits, on calls that follow each other on one stream and
share the library's built-in scratch, the later ones on smaller inputs whose slice tensors overlap what
the earlier call left there."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2306_11975_amd import ozimmu
from paper_2306_11975_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda"


def bits(x):
    return np.ascontiguousarray(x).view(np.uint64)


def run_both(A, B, s):
    m, k = A.shape
    n = B.shape[1]
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    C_static = torch.full((m, n), float("nan"), dtype=torch.float64, device=DEV)
    ozimmu.dgemm_static(dA, dB, C_static, s)
    C_ws = torch.full((m, n), float("nan"), dtype=torch.float64, device=DEV)
    ozimmu.dgemm(dA, dB, C_ws, s, ozimmu.alloc_workspace(m, n, k, s))
    torch.cuda.synchronize()
    return C_static.cpu().numpy(), C_ws.cpu().numpy()


def test_static_scratch_matches_workspace_call_on_consecutive_calls():
    # first call: several tiles, ragged; second and third: smaller inputs, other slice counts
    for (m, n, k, s, phi, seed) in [(700, 520, 900, 8, 1.0, 71), (130, 70, 333, 5, 2.0, 72), (1, 3, 2, 11, 0.5, 73)]:
        print(f"static m={m} n={n} k={k} s={s}", flush=True)
        assert ozimmu.workspace_bytes(m, n, k, s) <= ozimmu.STATIC_SCRATCH_BYTES
        A, B = wl.phi_pair(m, n, k, phi, seed)
        got, ref = run_both(A, B, s)
        assert np.array_equal(bits(got), bits(ref)), (m, n, k, s)
        assert np.array_equal(bits(got), bits(oracle.dgemm(A, B, s))), (m, n, k, s)


def test_static_scratch_rejects_what_does_not_fit_and_handles_empty_products():
    L = ozimmu.lib()
    fake = ctypes.c_void_p(256)   # never dereferenced: the size check comes first
    assert ozimmu.workspace_bytes(8192, 8192, 8192, 8) > ozimmu.STATIC_SCRATCH_BYTES
    assert L.ozimmu_dgemm_static(8192, 8192, 8192, fake, 8192, fake, 8192, fake, 8192, 8, None) == ozimmu.ERR_TOO_LARGE
    assert L.ozimmu_dgemm_static(4, 4, 4, fake, 4, fake, 4, fake, 4, 0, None) == ozimmu.ERR_BAD_SLICES
    assert L.ozimmu_dgemm_static(-1, 4, 4, fake, 4, fake, 4, fake, 4, 3, None) == ozimmu.ERR_BAD_DIM
    assert L.ozimmu_dgemm_static(0, 4, 4, None, 4, None, 4, None, 4, 3, None) == ozimmu.OK
    C = torch.full((3, 4), float("nan"), dtype=torch.float64, device=DEV)
    ozimmu.dgemm_static(torch.empty((3, 0), dtype=torch.float64, device=DEV),
                        torch.empty((0, 4), dtype=torch.float64, device=DEV), C, 5)
    torch.cuda.synchronize()
    assert not C.cpu().numpy().any()
