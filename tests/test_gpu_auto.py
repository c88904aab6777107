"""Automatic choice of the number of slices (Section 4.4) on the GPU against the oracle: the sums
of lost mantissa bits per slice count are integers and must be identical, and so must the choice
(both sides decide sum <= T * count in double precision)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_11975_amd import ozimmu
from paper_2306_11975_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check(A, B, thresholds=(0.0, 0.5, 1.0, 3.0, 20.0), dA=None, dB=None):
    dA = dev(A) if dA is None else dA
    dB = dev(B) if dB is None else dB
    for T in thresholds:
        s_want, sums_want = oracle.auto_num_slices(A, B, T)
        s_got, sums_got = ozimmu.auto_num_slices(dA, dB, T)
        assert np.array_equal(sums_got, sums_want)
        assert s_got == s_want, T
    return ozimmu.auto_num_slices(dA, dB, 0.0)[0]


@pytest.mark.parametrize("m,n,k,phi,seed", [(64, 64, 64, 0.5, 1), (300, 270, 517, 2.0, 2), (257, 513, 130, 1.0, 3),
                                            (1, 1, 1, 1.0, 4), (7, 1000, 9000, 1.0, 5)])
def test_auto_matches_oracle(m, n, k, phi, seed):
    A, B = wl.phi_pair(m, n, k, phi, seed)
    check(A, B)


def test_auto_adversarial_values_and_strides():
    M = wl.adversarial_matrix(40, 333, seed=9)       # zero row/column, powers of two, subnormals, huge rows
    check(M, np.ascontiguousarray(M.T))
    big = wl.phi_matrix(50, 200, 1.0, seed=3)
    A = big[:, 11:151]                                # odd offset: rows are not 16-byte aligned
    B = wl.phi_matrix(140, 90, 2.0, seed=4)
    dbig = dev(big)
    check(np.ascontiguousarray(A), B, dA=dbig[:, 11:151])


def test_auto_single_binade_and_limits():
    rng = np.random.default_rng(3)
    A = 1.0 + rng.random((100, 300))
    B = 1.0 + rng.random((300, 50))
    dA, dB = dev(A), dev(B)
    assert ozimmu.auto_num_slices(dA, dB, 0.0)[0] == 8
    assert ozimmu.auto_num_slices(dA, dB, 4.0)[0] == 7
    assert ozimmu.auto_num_slices(dA, dB, 0.0, max_slices=6)[0] == 6
    # the chosen count makes the GPU product exact here: integers below 2^20 times 2^-20
    Ai = np.round(A * 2 ** 20) / 2 ** 20
    Bi = np.round(B * 2 ** 20) / 2 ** 20
    s = ozimmu.auto_num_slices(dev(Ai), dev(Bi), 0.0)[0]
    C = torch.empty((100, 50), dtype=torch.float64, device="cuda")
    ozimmu.dgemm(dev(Ai), dev(Bi), C, s, ozimmu.alloc_workspace(100, 50, 300, s))
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy(), oracle.dgemm(Ai, Bi, s))
    # degenerate shapes pick one slice
    e = torch.empty((0, 5), dtype=torch.float64, device="cuda")
    assert ozimmu.auto_num_slices(e, torch.empty((5, 3), dtype=torch.float64, device="cuda"), 0.0)[0] >= 1
    assert ozimmu.auto_num_slices(torch.empty((3, 0), dtype=torch.float64, device="cuda"),
                                  torch.empty((0, 3), dtype=torch.float64, device="cuda"), 0.0)[0] == 1


@pytest.mark.parametrize("m,k", [(20001, 100), (2500, 3000), (3, 20000)])
def test_auto_workgroups_that_walk_several_row_groups(m, k):
    """More row groups than the scan launches workgroups (four short rows per wavefront: 20001 x 100;
    one long row per workgroup: 2500 x 3000), and rows too long for the register cache (3 x 20000)."""
    A = wl.phi_matrix(m, k, 1.5, seed=21)
    B = wl.phi_matrix(k, 5, 1.0, seed=22)
    check(A, B, thresholds=(0.0, 1.0))


def test_auto_complex_planes():
    A = wl.gaussian_complex(130, 256, seed=1)
    B = wl.unit_column_complex(256, 70, seed=2)
    check(A, B, thresholds=(0.0, 1.0))


def test_auto_complex_rows_beyond_the_one_pass_scan():
    """Interleaved rows of more than 1024 elements are scanned one plane at a time (element stride 2);
    20000 short rows make the one-pass kernel's workgroups walk several row groups."""
    check(wl.gaussian_complex(40, 1500, seed=5), wl.unit_column_complex(1500, 33, seed=6), thresholds=(0.0, 1.0))
    check(wl.gaussian_complex(20000, 70, seed=7), wl.unit_column_complex(70, 9, seed=8), thresholds=(0.0, 1.0))


@pytest.mark.parametrize("m,k", [(20000, 64), (4099, 33), (70, 1), (5000, 128), (301, 65), (100000, 16)])
def test_auto_complex_short_rows(m, k):
    """Rows of up to 128 interleaved elements (the state vector under a gate of up to seven qubits) have a scan kernel
    of their own: one and two words per lane, wavefronts that walk several row groups, ragged last groups."""
    check(wl.gaussian_complex(m, k, seed=m + k), wl.unit_column_complex(k, 9, seed=k + 2), thresholds=(0.0, 1.0))


def test_auto_complex_short_rows_adversarial_values():
    """Zero rows, subnormal rows (the exponents then come from the full bit patterns, not from the high words), exact
    powers of two and huge elements, in both planes."""
    for m, k, n in ((96, 64, 64), (50, 128, 128), (33, 7, 100), (70, 100, 3)):
        A = wl.adversarial_matrix(m, k, seed=31) + 1j * wl.adversarial_matrix(m, k, seed=32)
        B = wl.adversarial_matrix(k, n, seed=33) + 1j * wl.adversarial_matrix(k, n, seed=34)   # a small operand scanned by columns: one launch for both planes
        check(A, B, thresholds=(0.0, 1.0))
        check(A, wl.unit_column_complex(k, n, seed=35), thresholds=(0.0, 1.0))


@pytest.mark.parametrize("k", [400, 900, 1024])
def test_auto_complex_rows_shared_by_two_and_four_wavefronts(k):
    """One-pass scan of interleaved rows with two (256 < k <= 512) and four (k <= 1024) wavefronts per row group."""
    check(wl.gaussian_complex(37, k, seed=k), wl.unit_column_complex(k, 21, seed=k + 1), thresholds=(0.0, 1.0))


def test_auto_full_size_matches_oracle():
    """m = n = k = 4096, phi = 1: the launch configuration of the large workloads (rows kept in
    registers, 256-row bands for the columns)."""
    A = wl.phi_matrix_device(4096, 4096, 1.0, 1003)
    B = wl.phi_matrix_device(4096, 4096, 1.0, 2003)
    check(A.cpu().numpy(), B.cpu().numpy(), thresholds=(0.0, 1.0), dA=A, dB=B)


@pytest.mark.parametrize("ta", ["N", "T", "C"])
@pytest.mark.parametrize("tb", ["N", "T"])
@pytest.mark.parametrize("cplx", [False, True])
def test_auto_for_column_major_operands_with_transposes(ta, tb, cplx):
    """The BLAS-style variant must see the same groups (rows of op(A), columns of op(B)) whichever way
    the operands are stored: sums and choice equal the oracle's on op(A), op(B)."""
    m, n, k = 70, 300, 190
    opA, opB = wl.phi_pair(m, n, k, 2.0, seed=21)
    if cplx:
        oA2, oB2 = wl.phi_pair(m, n, k, 0.5, seed=22)
        opA, opB = opA + 1j * oA2, opB + 1j * oB2
    A = {"N": opA, "T": opA.T, "C": opA.conj().T}[ta]
    B = {"N": opB, "T": opB.T, "C": opB.conj().T}[tb]
    lda, ldb = A.shape[0] + 3, B.shape[0] + 1

    def col_major(M, ld):
        buf = np.full((M.shape[1], ld), 1e300, dtype=M.dtype)   # padding rows would dominate every exponent if read
        buf[:, :M.shape[0]] = M.T
        return torch.from_numpy(buf).cuda()

    dA, dB = col_major(A, lda), col_major(B, ldb)
    for T in (0.0, 1.0, 6.0):
        s_want, sums_want = oracle.auto_num_slices(opA, opB, T)
        s_got, sums_got = ozimmu.auto_num_slices_blas(ta, tb, m, n, k, dA, lda, dB, ldb, cplx, T)
        assert np.array_equal(sums_got, sums_want)
        assert s_got == s_want


# ------------------------------------------------------------------ count and product in one call, general shapes
def bits(x):
    return np.ascontiguousarray(x).view(np.uint64)


@pytest.mark.parametrize("cplx", [False, True])
@pytest.mark.parametrize("m,n,k,phi,seed", [(300, 270, 517, 2.0, 2), (64, 64, 64, 0.5, 1), (130, 700, 300, 1.0, 3), (1, 1, 1, 1.0, 4)])
def test_gemm_auto_is_choice_then_product(cplx, m, n, k, phi, seed):
    """ozimmu_dgemm_auto / ozimmu_zgemm_auto on shapes of the general path: whatever the guess, the count is the oracle's
    choice and C the oracle's product with it; the guess is confirmed exactly when it was right. (The shapes of the
    one-kernel complex path are in test_gpu_gate.py.)"""
    A, B = wl.phi_pair(m, n, k, phi, seed)
    if cplx:
        Ai, Bi = wl.phi_pair(m, n, k, phi, seed + 100)
        A, B = A + 1j * Ai, B + 1j * Bi
    dA, dB = dev(A), dev(B)
    gemm_auto = ozimmu.zgemm_auto if cplx else ozimmu.dgemm_auto
    oracle_gemm = oracle.zgemm if cplx else oracle.dgemm
    for T in (0.0, 1.0):
        s_want = oracle.auto_num_slices(A, B, T)[0]
        want = oracle_gemm(A, B, s_want)
        for guess in (s_want, s_want - 1, s_want + 1, 0, 16):
            guess = min(max(guess, 0), 16)
            C = torch.full((m, n), float("nan"), dtype=dA.dtype, device="cuda")
            s_got, confirmed = gemm_auto(dA, dB, C, T, guess=guess)
            assert s_got == s_want, (T, guess)
            assert confirmed == (guess == s_want), (T, guess)
            assert np.array_equal(bits(C.cpu().numpy()), bits(want)), (T, guess)


@pytest.mark.parametrize("cplx,m,n,k", [(False, 6, 33, 8999), (False, 5, 40, 9000), (True, 20, 30, 5000), (True, 9, 70, 4097)])
def test_gemm_auto_long_rows(cplx, m, n, k):
    """Rows too long to stay in registers (read twice by the splitter; a complex operand then takes one strided pass
    per plane), odd leading dimensions: the counting variants of those splitters."""
    A, B = wl.phi_pair(m, n, k, 1.0, seed=k)
    if cplx:
        Ai, Bi = wl.phi_pair(m, n, k, 2.0, seed=k + 1)
        A, B = A + 1j * Ai, B + 1j * Bi
    dA, dB = dev(A), dev(B)
    s_want = oracle.auto_num_slices(A, B, 1.0)[0]
    want = (oracle.zgemm if cplx else oracle.dgemm)(A, B, s_want)
    for guess in (s_want, s_want + 1):
        C = torch.full((m, n), float("nan"), dtype=dA.dtype, device="cuda")
        s_got, confirmed = (ozimmu.zgemm_auto if cplx else ozimmu.dgemm_auto)(dA, dB, C, 1.0, guess=guess)
        assert (s_got, confirmed) == (s_want, guess == s_want)
        assert np.array_equal(bits(C.cpu().numpy()), bits(want))


def test_gemm_auto_rejects_a_workspace_too_small_for_the_largest_count():
    A, B = wl.phi_pair(200, 100, 300, 1.0, 7)
    dA, dB = dev(A), dev(B)
    C = torch.empty((200, 100), dtype=torch.float64, device="cuda")
    ws = torch.empty(ozimmu.workspace_bytes(200, 100, 300, 8), dtype=torch.uint8, device="cuda")
    with pytest.raises(ozimmu.OzimmuError):
        ozimmu.dgemm_auto(dA, dB, C, 1.0, guess=8, workspace=ws)                      # 16 slices would not fit
    s, _ = ozimmu.dgemm_auto(dA, dB, C, 1.0, guess=8, max_slices=8, workspace=ws)     # ... 8 do
    assert s == min(8, oracle.auto_num_slices(A, B, 1.0)[0])


def test_gemm_auto_degenerate_cases():
    A = torch.zeros((6, 0), dtype=torch.float64, device="cuda")
    B = torch.zeros((0, 9), dtype=torch.float64, device="cuda")
    C = torch.full((6, 9), float("nan"), dtype=torch.float64, device="cuda")
    assert ozimmu.dgemm_auto(A, B, C, 1.0, guess=4) == (1, False)      # k = 0: nothing to inspect, C = 0
    assert (C.cpu().numpy() == 0.0).all()
    Z = torch.zeros((40, 30), dtype=torch.float64, device="cuda")       # all-zero operands lose nothing: one slice
    C = torch.full((40, 50), float("nan"), dtype=torch.float64, device="cuda")
    assert ozimmu.dgemm_auto(Z, torch.zeros((30, 50), dtype=torch.float64, device="cuda"), C, 0.0, guess=1) == (1, True)
    assert (C.cpu().numpy() == 0.0).all()
