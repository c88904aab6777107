"""BLAS-style entry point (column-major, transposes, alpha/beta; Section 4.4) against the oracle,
bit for bit: the Ozaki product is the same fixed-order computation and the update has a fixed order
of roundings."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_11975_amd import ozimmu
from paper_2306_11975_amd import workloads as wl

pytestmark = pytest.mark.gpu


def bits(x):
    return np.ascontiguousarray(x).view(np.uint64)


def col_major_on_device(M, ld):
    """Mathematical matrix M (r x c) -> device buffer holding it column-major with leading dimension ld
    (padding rows poisoned)."""
    r, c = M.shape
    buf = np.full((max(c, 1), ld), 7.25e300)
    buf[:c, :r] = M.T
    return torch.from_numpy(buf).cuda()


def run(ta, tb, m, n, k, alpha, beta, s, phi=1.0, seed=1, pad=(0, 0, 0), c_nan=False):
    opA, opB = wl.phi_pair(m, n, k, phi, seed)
    A = opA.T.copy() if ta else opA
    B = opB.T.copy() if tb else opB
    rng = np.random.default_rng(seed + 100)
    C0 = np.full((m, n), np.nan) if c_nan else rng.standard_normal((m, n))
    lda, ldb, ldc = max(A.shape[0], 1) + pad[0], max(B.shape[0], 1) + pad[1], max(m, 1) + pad[2]
    dA, dB, dC = col_major_on_device(A, lda), col_major_on_device(B, ldb), col_major_on_device(C0, ldc)
    ws = ozimmu.alloc_workspace(n, m, k, s)
    ozimmu.dgemm_blas("T" if ta else "N", "T" if tb else "N", m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc, s, ws)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    got = out[:n, :m].T
    want = oracle.dgemm_blas(ta, tb, alpha, A, B, beta, C0, s)
    assert np.array_equal(bits(got), bits(want))
    assert (out[:, m:] == 7.25e300).all(), "padding of C must be untouched"


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
def test_blas_transposes_and_scalars_bit_exact(ta, tb):
    for alpha, beta in ((1.0, 0.0), (1.7, -0.3), (-2.0, 1.0), (0.5, 0.0)):
        run(ta, tb, 130, 70, 300, alpha, beta, 8, pad=(3, 5, 2))


@pytest.mark.parametrize("m,n,k,s", [(300, 270, 1300, 7), (33, 520, 2049, 5), (257, 64, 64, 13), (40, 50, 70000, 2)])
def test_blas_shapes_across_the_kernels(m, n, k, s):
    """Short k (sum kept in registers), long k (diagonal buffers) and INT64 k-blocking."""
    run(True, False, m, n, k, 1.25, 0.75, s, phi=2.0, seed=3, pad=(1, 0, 7))
    run(False, True, m, n, k, 1.0, 0.0, s, phi=0.5, seed=4)


def test_blas_beta_zero_does_not_read_c_and_degenerate_cases():
    run(False, False, 64, 48, 100, 2.0, 0.0, 6, c_nan=True)
    run(True, True, 64, 48, 2000, 1.0, 0.0, 6, c_nan=True)
    # alpha == 0 and k == 0: only the scaling of C remains
    for k, alpha in ((0, 1.0), (50, 0.0)):
        m, n = 37, 21
        C0 = np.random.default_rng(5).standard_normal((m, n))
        for beta in (0.0, -1.5):
            dC = col_major_on_device(C0, m + 2)
            dA = torch.zeros(max(m * max(k, 1), 1), dtype=torch.float64, device="cuda")
            ozimmu.dgemm_blas("N", "N", m, n, k, alpha, dA, m, dA, max(k, 1), beta, dC, m + 2, 4, None)
            torch.cuda.synchronize()
            got = dC.cpu().numpy()[:n, :m].T
            want = np.zeros((m, n)) if beta == 0.0 else beta * C0
            assert np.array_equal(bits(got), bits(want))
            assert not np.signbit(got).any() or beta != 0.0


# ------------------------------------------------------------------ complex call
def zcol_major_on_device(M, ld):
    r, c = M.shape
    buf = np.full((max(c, 1), ld), 7.25e300 + 3.5e299j, dtype=np.complex128)
    buf[:c, :r] = M.T
    return torch.from_numpy(buf).cuda()


def zrun(ta, tb, m, n, k, alpha, beta, s, seed=1, pad=(0, 0, 0), c_nan=False, scale_cols=True):
    rng = np.random.default_rng(seed)
    opA = rng.standard_normal((m, k)) * np.exp(rng.standard_normal((m, k))) + 1j * rng.standard_normal((m, k))
    opB = rng.standard_normal((k, n)) + 1j * rng.standard_normal((k, n)) * np.exp(0.5 * rng.standard_normal((k, n)))
    A = {"N": opA, "T": opA.T.copy(), "C": opA.conj().T.copy()}[ta]
    B = {"N": opB, "T": opB.T.copy(), "C": opB.conj().T.copy()}[tb]
    C0 = np.full((m, n), np.nan + 1j * np.nan) if c_nan else rng.standard_normal((m, n)) + 1j * rng.standard_normal((m, n))
    lda, ldb, ldc = max(A.shape[0], 1) + pad[0], max(B.shape[0], 1) + pad[1], max(m, 1) + pad[2]
    dA, dB, dC = zcol_major_on_device(A, lda), zcol_major_on_device(B, ldb), zcol_major_on_device(C0, ldc)
    ws = torch.empty(ozimmu.zgemm_blas_workspace_bytes(m, n, k, s, beta == 0), dtype=torch.uint8, device="cuda")
    ozimmu.zgemm_blas(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc, s, ws)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    got = out[:n, :m].T
    want = oracle.zgemm_blas(ta, tb, alpha, A, B, beta, C0, s)
    assert np.array_equal(bits(got), bits(want)), (ta, tb, alpha, beta)
    assert (out[:, m:] == 7.25e300 + 3.5e299j).all(), "padding of C must be untouched"


@pytest.mark.parametrize("ta", ["N", "T", "C"])
@pytest.mark.parametrize("tb", ["N", "T", "C"])
def test_complex_blas_transposes_and_scalars_bit_exact(ta, tb):
    for alpha, beta in ((1.0, 0.0), (1.3 - 0.4j, -0.2 + 0.9j), (-2.0, 1.0), (0.5j, 0.0)):
        zrun(ta, tb, 130, 70, 300, alpha, beta, 8, pad=(3, 5, 2))


@pytest.mark.parametrize("m,n,k,s", [(300, 270, 1300, 7), (33, 520, 2049, 5), (257, 64, 64, 13), (40, 50, 70000, 2)])
def test_complex_blas_shapes_across_the_kernels(m, n, k, s):
    """Short k (both products of a part in one launch), long k (four launches) and INT64 k-blocking."""
    zrun("C", "N", m, n, k, 1.25 + 0.5j, 0.75j, s, seed=3, pad=(1, 0, 7))
    zrun("N", "C", m, n, k, 1.0, 0.0, s, seed=4)


@pytest.mark.parametrize("m,n,k,s", [(64, 1000, 64, 8), (32, 300, 32, 5), (17, 129, 40, 7), (64, 200, 64, 9), (128, 300, 100, 8),
                                     (100, 150, 128, 12)])
def test_complex_blas_small_gate_on_a_wide_state(m, n, k, s):
    """Neither operand transposed, A at most 128 x 128: the state (B, whose columns are the rows of the row-major
    product) is split inside the product kernel; with a general alpha and beta the update follows as for every other
    shape."""
    zrun("N", "N", m, n, k, 1.0, 0.0, s, seed=6, c_nan=True)
    zrun("N", "N", m, n, k, 1.0, 0.0, s, seed=7, pad=(3, 2, 5), c_nan=True)
    zrun("N", "N", m, n, k, 0.75 - 0.5j, 0.25 + 1.0j, s, seed=8, pad=(0, 1, 2))


def test_complex_blas_beta_zero_does_not_read_c_and_degenerate_cases():
    zrun("N", "N", 64, 48, 100, 2.0 - 1j, 0.0, 6, c_nan=True)
    zrun("C", "C", 64, 48, 2000, 1.0, 0.0, 6, c_nan=True)
    for k, alpha in ((0, 1.0), (50, 0.0)):
        m, n = 37, 21
        rng = np.random.default_rng(5)
        C0 = rng.standard_normal((m, n)) + 1j * rng.standard_normal((m, n))
        for beta in (0.0, -1.5 + 0.25j):
            dC = zcol_major_on_device(C0, m + 2)
            dA = torch.zeros(max(m * max(k, 1), 1), dtype=torch.complex128, device="cuda")
            ozimmu.zgemm_blas("N", "N", m, n, k, alpha, dA, m, dA, max(k, 1), beta, dC, m + 2, 4, None)
            torch.cuda.synchronize()
            got = dC.cpu().numpy()[:n, :m].T
            want = oracle.zgemm_blas("N", "N", alpha, np.zeros((m, k), dtype=complex), np.zeros((k, n), dtype=complex),
                                     beta, C0, 4)
            assert np.array_equal(bits(got), bits(want))


# ------------------------------------------------------------------ slice count chosen inside the BLAS-style call
@pytest.mark.parametrize("cplx,ta,tb", [(False, "N", "N"), (False, "T", "N"), (False, "N", "T"), (False, "T", "T"),
                                        (True, "N", "N"), (True, "T", "N"), (True, "N", "T"), (True, "T", "T"),
                                        (True, "C", "N"), (True, "N", "C")])
def test_blas_auto_is_choice_then_product(cplx, ta, tb):
    """ozimmu_dgemm_blas_auto / ozimmu_zgemm_blas_auto: count = the oracle's choice for op(A), op(B); C = the oracle's
    update with that count, whatever the guess; a guess can only be confirmed when beta is zero."""
    m, n, k = 90, 140, 260
    rng = np.random.default_rng(41)
    if cplx:
        opA = rng.standard_normal((m, k)) * np.exp(rng.standard_normal((m, k))) + 1j * rng.standard_normal((m, k))
        opB = rng.standard_normal((k, n)) + 1j * rng.standard_normal((k, n)) * np.exp(0.5 * rng.standard_normal((k, n)))
        A = {"N": opA, "T": opA.T.copy(), "C": opA.conj().T.copy()}[ta]
        B = {"N": opB, "T": opB.T.copy(), "C": opB.conj().T.copy()}[tb]
        C0 = rng.standard_normal((m, n)) + 1j * rng.standard_normal((m, n))
        on_device, ref = zcol_major_on_device, lambda al, be, s: oracle.zgemm_blas(ta, tb, al, A, B, be, C0, s)
        scalars = ((1.0, 0.0), (0.5 - 1.5j, 0.0), (1.0, 0.25j))
    else:
        opA, opB = wl.phi_pair(m, n, k, 1.5, 42)
        A = opA.T.copy() if ta == "T" else opA
        B = opB.T.copy() if tb == "T" else opB
        C0 = rng.standard_normal((m, n))
        on_device, ref = col_major_on_device, lambda al, be, s: oracle.dgemm_blas(ta == "T", tb == "T", al, A, B, be, C0, s)
        scalars = ((1.0, 0.0), (-1.5, 0.0), (1.0, 0.5))
    lda, ldb, ldc = A.shape[0] + 3, B.shape[0] + 1, m + 2
    dA, dB = on_device(A, lda), on_device(B, ldb)
    for threshold in (0.0, 1.0):
        s_want = oracle.auto_num_slices(opA, opB, threshold)[0]
        for alpha, beta in scalars:
            want = ref(alpha, beta, s_want)
            for guess in (s_want, s_want - 1, 0):
                dC = on_device(C0, ldc)
                s_got, confirmed = ozimmu.gemm_blas_auto(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc, cplx,
                                                         threshold, guess=guess)
                assert s_got == s_want
                assert confirmed == (guess == s_want and beta == 0), (alpha, beta, guess)
                assert np.array_equal(bits(dC.cpu().numpy()[:n, :m].T), bits(want)), (threshold, alpha, beta, guess)


def test_complex_blas_auto_small_gate_on_a_wide_state():
    """Untransposed plain product with a small first operand: the one-kernel path inside the BLAS-style one-call form."""
    m, n, k = 64, 700, 64
    rng = np.random.default_rng(43)
    opA = wl.unit_column_complex(m, k, seed=44)
    opB = rng.standard_normal((k, n)) + 1j * rng.standard_normal((k, n))
    opB /= np.linalg.norm(opB)
    C0 = np.zeros((m, n), dtype=np.complex128)
    dA, dB = zcol_major_on_device(opA, m), zcol_major_on_device(opB, k)
    s_want = oracle.auto_num_slices(opA, opB, 1.0)[0]
    want = oracle.zgemm_blas("N", "N", 1.0, opA, opB, 0.0, C0, s_want)
    for guess in (s_want, s_want + 1):
        dC = zcol_major_on_device(C0, m)
        assert ozimmu.gemm_blas_auto("N", "N", m, n, k, 1.0, dA, m, dB, k, 0.0, dC, m, True, 1.0, guess=guess) == (s_want, guess == s_want)
        assert np.array_equal(bits(dC.cpu().numpy()[:n, :m].T), bits(want))


def test_blas_auto_degenerate_cases():
    """k = 0 (C is only scaled), an empty C, alpha = 0: the one-call forms return what the two calls give."""
    rng = np.random.default_rng(45)
    C0 = rng.standard_normal((5, 4))
    dA, dB = col_major_on_device(np.zeros((5, 1)), 5), col_major_on_device(np.zeros((1, 4)), 1)
    dC = col_major_on_device(C0, 5)
    s, confirmed = ozimmu.gemm_blas_auto("N", "N", 5, 4, 0, 1.0, dA, 5, dB, 1, 2.0, dC, 5, False, 1.0, guess=3)
    assert (s, confirmed) == (1, False)
    assert np.array_equal(bits(dC.cpu().numpy()[:4, :5].T), bits(2.0 * C0))
    dC = col_major_on_device(C0, 5)
    A = rng.standard_normal((5, 7))
    B = rng.standard_normal((7, 4))
    s, confirmed = ozimmu.gemm_blas_auto("N", "N", 5, 4, 7, 0.0, col_major_on_device(A, 5), 5, col_major_on_device(B, 7), 7, 0.0,
                                         dC, 5, False, 1.0, guess=3)
    assert not confirmed and s == oracle.auto_num_slices(A, B, 1.0)[0]
    assert (dC.cpu().numpy()[:4, :5] == 0.0).all()
    assert ozimmu.gemm_blas_auto("N", "N", 0, 4, 7, 1.0, dA, 1, col_major_on_device(B, 7), 7, 0.0, dC, 1, False, 1.0, guess=3)[0] >= 1
