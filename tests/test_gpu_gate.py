"""GPU parity of the one-kernel complex product for a small gate on a tall state (Section 4.4: a d-qubit gate on an
N-qubit state vector is the complex product 2^(N-d) x 2^d x 2^d). ozimmu_zgemm takes that path when k and n are
at most 128 (256 with up to eight slices); the state is then split inside the product kernel (tiles of 32 rows; one
step of 64 positions and eight fragments of the gate while k and n are at most 64, two steps and sixteen fragments up to
128, four steps, 32 fragments and sixteen wavefronts up to 256; four wavefronts per SIMD up to eight slices, two beyond). Compared bit for bit with the oracle, which splits first and multiplies afterwards."""
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


def gpu_zgemm(A, B, s, lda_extra=0, ldb_extra=0, ldc_extra=0):
    m, k = A.shape
    n = B.shape[1]
    nan = complex(float("nan"), float("nan"))
    Ad = torch.full((m, k + lda_extra), nan, dtype=torch.complex128, device=DEV)
    Bd = torch.full((k, n + ldb_extra), nan, dtype=torch.complex128, device=DEV)
    Cd = torch.full((m, n + ldc_extra), nan, dtype=torch.complex128, device=DEV)
    Ad[:, :k] = torch.from_numpy(A)
    Bd[:, :n] = torch.from_numpy(B)
    ozimmu.zgemm(Ad[:, :k], Bd[:, :n], Cd[:, :n], s, ozimmu.alloc_workspace(m, n, k, s, is_complex=True))
    torch.cuda.synchronize()
    out = Cd.cpu().numpy()
    assert np.all(np.isnan(out[:, n:].real)) and np.all(np.isnan(out[:, n:].imag)), "wrote outside C"
    return out[:, :n]


def assert_same(got, want):
    assert np.array_equal(bits(got.real.copy()), bits(want.real.copy()))
    assert np.array_equal(bits(got.imag.copy()), bits(want.imag.copy()))


@pytest.mark.parametrize("s", range(1, 17))
@pytest.mark.parametrize("k", [32, 64])
def test_gate_every_slice_count(s, k):
    """Every slice count of the kernel for k, n <= 64, with half a step and a whole one; five row tiles with a ragged last one."""
    m, n = 150, 64
    A = wl.gaussian_complex(m, k, seed=100 + s)
    B = wl.unit_column_complex(k, n, seed=200 + s)
    assert_same(gpu_zgemm(A, B, s), oracle.zgemm(A, B, s))


@pytest.mark.parametrize("s", range(1, 17))
def test_gate_every_slice_count_two_steps(s):
    """The instantiations for k or n above 64: five row tiles of 32 with a ragged last one, sixteen fragments of B."""
    m, n, k = 150, 128, 128
    A = wl.gaussian_complex(m, k, seed=300 + s)
    B = wl.unit_column_complex(k, n, seed=400 + s)
    assert_same(gpu_zgemm(A, B, s), oracle.zgemm(A, B, s))


@pytest.mark.parametrize("m,n,k,s", [(33, 128, 65, 8), (100, 65, 64, 7), (31, 70, 20, 3), (97, 113, 127, 6), (64, 128, 1, 2),
                                     (200, 81, 100, 8)])
def test_gate_ragged_shapes_two_steps(m, n, k, s):
    """k or n between 65 and 128 (k short of the two steps is padded with zero slices; fragments past the last
    column are skipped)."""
    A = wl.gaussian_complex(m, k, seed=m + k)
    B = wl.unit_column_complex(k, n, seed=n + k + 1)
    assert_same(gpu_zgemm(A, B, s, lda_extra=1, ldb_extra=2, ldc_extra=3), oracle.zgemm(A, B, s))


@pytest.mark.parametrize("s", range(1, 9))
def test_gate_every_slice_count_four_steps(s):
    """k and n up to 256 with up to eight slices: workgroups of sixteen wavefronts, 32 lanes per row, 32 fragments of B."""
    m, n, k = 70, 256, 256
    A = wl.gaussian_complex(m, k, seed=500 + s)
    B = wl.unit_column_complex(k, n, seed=600 + s)
    assert_same(gpu_zgemm(A, B, s), oracle.zgemm(A, B, s))


@pytest.mark.parametrize("m,n,k,s", [(33, 200, 129, 5), (70, 130, 64, 8), (31, 64, 250, 3), (100, 255, 193, 7), (64, 256, 1, 2),
                                     (40, 129, 129, 9)])
def test_gate_ragged_shapes_four_steps(m, n, k, s):
    """k or n between 129 and 256 (zero rows among the adversarial values take the 64-bit maxima over 32 lanes);
    nine slices at that size take the general path."""
    A = wl.gaussian_complex(m, k, seed=m + k)
    A[m // 2, :] = 0.0
    B = wl.unit_column_complex(k, n, seed=n + k + 1)
    assert_same(gpu_zgemm(A, B, s, lda_extra=1, ldb_extra=2, ldc_extra=3), oracle.zgemm(A, B, s))


def test_eight_qubit_gate_sampled_rows():
    """An 8-qubit gate on 20 qubits (4096 x 256 x 256), rows sampled over the whole state."""
    m, k, s = 1 << 12, 256, 8
    A = wl.gaussian_complex_device(m, k, seed=26)
    A = A / A.abs().pow(2).sum().sqrt()
    U = wl.haar_unitary_device(k, seed=27).contiguous()
    C = torch.empty((m, k), dtype=torch.complex128, device=DEV)
    ozimmu.zgemm(A, U, C, s, ozimmu.alloc_workspace(m, k, k, s, is_complex=True))
    torch.cuda.synchronize()
    rng = np.random.default_rng(28)
    rows = np.unique(np.concatenate([[0, 31, 32, m - 32, m - 1], rng.integers(0, m, 60)]))
    idx = torch.from_numpy(rows).to(DEV)
    assert_same(C[idx].cpu().numpy(), oracle.zgemm(A[idx].cpu().numpy(), U.cpu().numpy(), s))


@pytest.mark.parametrize("m,n,k,s", [(1, 1, 1, 3), (64, 64, 64, 8), (65, 63, 33, 7), (63, 17, 31, 5), (130, 16, 64, 8),
                                     (200, 15, 17, 2), (31, 33, 1, 4), (300, 48, 40, 6), (129, 32, 32, 8), (64, 49, 64, 1)])
def test_gate_ragged_shapes(m, n, k, s):
    """Rows, columns and inner dimension on both sides of the boundaries the kernel has: 32 rows per workgroup, 16 per
    wavefront, 8 columns per patch (patches past the last column are skipped), 64 positions per step."""
    A = wl.gaussian_complex(m, k, seed=m + k)
    B = wl.unit_column_complex(k, n, seed=n + k + 1)
    assert_same(gpu_zgemm(A, B, s), oracle.zgemm(A, B, s))


def test_gate_respects_leading_dimensions():
    A = wl.gaussian_complex(100, 50, seed=3)
    B = wl.unit_column_complex(50, 40, seed=4)
    assert_same(gpu_zgemm(A, B, 7, lda_extra=5, ldb_extra=3, ldc_extra=9), oracle.zgemm(A, B, 7))


def test_gate_adversarial_values():
    """Zero rows and columns, exact powers of two, one huge element per row, subnormals, in both planes."""
    m, n, k = 96, 64, 64
    A = wl.adversarial_matrix(m, k, seed=5) + 1j * wl.adversarial_matrix(m, k, seed=6)
    B = wl.adversarial_matrix(k, n, seed=7) + 1j * wl.adversarial_matrix(k, n, seed=8)
    for s in (3, 8):
        assert_same(gpu_zgemm(A, B, s), oracle.zgemm(A, B, s))


def test_gate_purely_real_and_purely_imaginary_operands():
    """Each of the four real products on its own: a part that must come out as an exact zero does."""
    A = wl.gaussian_complex(70, 64, seed=9)
    B = wl.unit_column_complex(64, 64, seed=10)
    for Ax, Bx in ((A.real + 0j, B.real + 0j), (1j * A.imag, 1j * B.imag), (A.real + 0j, 1j * B.imag), (1j * A.imag, B.real + 0j)):
        got = gpu_zgemm(np.ascontiguousarray(Ax), np.ascontiguousarray(Bx), 6)
        assert_same(got, oracle.zgemm(Ax, Bx, 6))


def test_seven_qubit_gate_sampled_rows():
    """A 7-qubit gate on 20 qubits (8192 x 128 x 128), rows sampled over the whole state."""
    m, k, s = 1 << 13, 128, 8
    A = wl.gaussian_complex_device(m, k, seed=16)
    A = A / A.abs().pow(2).sum().sqrt()
    U = wl.haar_unitary_device(k, seed=17).contiguous()
    C = torch.empty((m, k), dtype=torch.complex128, device=DEV)
    ozimmu.zgemm(A, U, C, s, ozimmu.alloc_workspace(m, k, k, s, is_complex=True))
    torch.cuda.synchronize()
    rng = np.random.default_rng(18)
    rows = np.unique(np.concatenate([[0, 31, 32, m - 32, m - 1], rng.integers(0, m, 100)]))
    idx = torch.from_numpy(rows).to(DEV)
    assert_same(C[idx].cpu().numpy(), oracle.zgemm(A[idx].cpu().numpy(), U.cpu().numpy(), s))


def test_gate_adversarial_values_many_slices():
    """The wide fixed-point fraction (more than nine slices) on zero rows, powers of two, huge elements, subnormals."""
    m, n, k = 70, 100, 90
    A = wl.adversarial_matrix(m, k, seed=21) + 1j * wl.adversarial_matrix(m, k, seed=22)
    B = wl.adversarial_matrix(k, n, seed=23) + 1j * wl.adversarial_matrix(k, n, seed=24)
    for s in (10, 13, 16):
        assert_same(gpu_zgemm(A, B, s), oracle.zgemm(A, B, s))


def test_wider_products_take_the_general_path():
    A = wl.gaussian_complex(70, 64, seed=11)
    B = wl.unit_column_complex(64, 140, seed=12)
    assert_same(gpu_zgemm(A, B, 8), oracle.zgemm(A, B, 8))


def test_gate_on_a_long_state_sampled_rows():
    """A 6-qubit gate on 22 qubits (65536 x 64 x 64): rows sampled over the whole state, among them the first and
    last of the first and last workgroup (separability: an entry of the result depends on one row of the state only)."""
    m, k, s = 1 << 16, 64, 8
    A = wl.gaussian_complex_device(m, k, seed=13)
    A = A / A.abs().pow(2).sum().sqrt()
    U = wl.haar_unitary_device(k, seed=14).contiguous()
    C = torch.empty((m, k), dtype=torch.complex128, device=DEV)
    ozimmu.zgemm(A, U, C, s, ozimmu.alloc_workspace(m, k, k, s, is_complex=True))
    torch.cuda.synchronize()
    rng = np.random.default_rng(15)
    rows = np.unique(np.concatenate([[0, 31, 32, 63, 64, m - 32, m - 1], rng.integers(0, m, 200)]))
    idx = torch.from_numpy(rows).to(DEV)
    want = oracle.zgemm(A[idx].cpu().numpy(), U.cpu().numpy(), s)
    assert_same(C[idx].cpu().numpy(), want)


def test_gate_call_captured_in_a_graph_replays_correctly():
    """The gate path only enqueues two kernels on the caller's stream, so a call can be captured and replayed: each
    replay runs on new data written into the captured buffers, with eager work and synchronisations in between."""
    m, k, s = 3000, 64, 8
    A = torch.empty((m, k), dtype=torch.complex128, device=DEV)
    U = torch.empty((k, k), dtype=torch.complex128, device=DEV)
    C = torch.empty((m, k), dtype=torch.complex128, device=DEV)
    ws = ozimmu.alloc_workspace(m, k, k, s, is_complex=True)
    A.copy_(torch.from_numpy(wl.gaussian_complex(m, k, seed=40)))
    U.copy_(torch.from_numpy(wl.unit_column_complex(k, k, seed=41)))
    ozimmu.zgemm(A, U, C, s, ws)            # warm-up outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            ozimmu.zgemm(A, U, C, s, ws, stream=side)
    for seed in (42, 43, 44):
        Ah, Uh = wl.gaussian_complex(m, k, seed=seed), wl.unit_column_complex(k, k, seed=seed + 10)
        A.copy_(torch.from_numpy(Ah))
        U.copy_(torch.from_numpy(Uh))
        C.fill_(complex(float("nan"), float("nan")))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_same(C.cpu().numpy(), oracle.zgemm(Ah, Uh, s))


def test_gate_seeded_random_shapes_and_values():
    """Forty seeded shapes over the whole range the one-kernel path serves (k, n up to 256 with up to eight slices, up to
    128 beyond), with Gaussian, wide-exponent and adversarial values in turn."""
    rng = np.random.default_rng(2024)
    for it in range(40):
        s = int(rng.integers(1, 17))
        lim = 256 if s <= 8 else 128
        k, n, m = int(rng.integers(1, lim + 1)), int(rng.integers(1, lim + 1)), int(rng.integers(1, 300))
        if it % 3 == 0:
            A, B = wl.gaussian_complex(m, k, seed=it), wl.unit_column_complex(k, n, seed=1000 + it)
        elif it % 3 == 1:
            A = wl.phi_matrix(m, k, 2.0, seed=it) + 1j * wl.phi_matrix(m, k, 0.5, seed=it + 7)
            B = wl.phi_matrix(k, n, 1.0, seed=it + 3) + 1j * wl.phi_matrix(k, n, 2.0, seed=it + 5)
        else:
            A = wl.adversarial_matrix(m, k, seed=it) + 1j * wl.adversarial_matrix(m, k, seed=it + 1)
            B = wl.adversarial_matrix(k, n, seed=it + 2) + 1j * wl.adversarial_matrix(k, n, seed=it + 3)
        got = gpu_zgemm(np.ascontiguousarray(A), np.ascontiguousarray(B), s)
        want = oracle.zgemm(A, B, s)
        assert np.array_equal(bits(got.real.copy()), bits(want.real.copy())), (it, m, n, k, s)
        assert np.array_equal(bits(got.imag.copy()), bits(want.imag.copy())), (it, m, n, k, s)


# ------------------------------------------------------------------ slice count chosen and product formed in one call
def check_zgemm_auto(A, B, threshold, guesses):
    """ozimmu_zgemm_auto must return the count ozimmu_auto_num_slices chooses (= the oracle's) and the product with that
    count, whatever the guess; a guess is confirmed exactly when it was right."""
    s_want, _ = oracle.auto_num_slices(A, B, threshold)
    want = oracle.zgemm(A, B, s_want)
    m, k = A.shape
    n = B.shape[1]
    dA, dB = torch.from_numpy(np.ascontiguousarray(A)).to(DEV), torch.from_numpy(np.ascontiguousarray(B)).to(DEV)
    for guess in guesses:
        guess = s_want + guess[1] if isinstance(guess, tuple) else guess
        C = torch.full((m, n), complex(float("nan"), float("nan")), dtype=torch.complex128, device=DEV)
        s_got, confirmed = ozimmu.zgemm_auto(dA, dB, C, threshold, guess=guess)
        torch.cuda.synchronize()
        assert s_got == s_want, (guess, s_got, s_want)
        assert_same(C.cpu().numpy(), want)
        assert confirmed == (guess == s_want), (guess, s_want, confirmed)


@pytest.mark.parametrize("m,n,k", [(3000, 64, 64), (500, 128, 100), (200, 256, 256), (70, 16, 16), (33, 1, 5)])
@pytest.mark.parametrize("threshold", [0.0, 1.0, 6.0])
def test_zgemm_auto_with_right_and_wrong_guesses(m, n, k, threshold):
    A = wl.gaussian_complex(m, k, seed=m + n)
    A /= np.linalg.norm(A)
    B = wl.unit_column_complex(k, n, seed=k + 3)
    check_zgemm_auto(A, B, threshold, guesses=[("rel", 0), ("rel", 1), ("rel", -1), 0, 1, 16])


def test_zgemm_auto_adversarial_values_and_other_shapes():
    """Zero and subnormal rows in the counters of the product kernel; shapes the one-kernel path does not serve."""
    A = wl.adversarial_matrix(96, 64, seed=51) + 1j * wl.adversarial_matrix(96, 64, seed=52)
    B = wl.adversarial_matrix(64, 40, seed=53) + 1j * wl.adversarial_matrix(64, 40, seed=54)
    for threshold in (0.0, 2.0, 30.0):
        check_zgemm_auto(A, B, threshold, guesses=[("rel", 0), ("rel", -1), 7])
    A = wl.gaussian_complex(70, 300, seed=55)
    B = wl.unit_column_complex(300, 50, seed=56)
    check_zgemm_auto(A, B, 1.0, guesses=[("rel", 0), 0])


@pytest.mark.parametrize("k,s", [(128, 8), (128, 9), (128, 10), (64, 16), (64, 12), (64, 8), (33, 5), (256, 8)])
@pytest.mark.parametrize("signs", ["same", "mixed"])
def test_gate_largest_integer_sums(k, s, signs):
    """Every slice +-127 (elements of magnitude 1 - 2^-53 under a power-of-two maximum): the integer sums of the
    diagonals take their largest magnitude, which is what the fold's 32-bit merge of neighbouring diagonals must hold."""
    m, n = 40, min(k, 128)
    x = 1.0 - 2.0 ** -53
    rng = np.random.default_rng(k + s)
    def plane(r, c):
        sg = np.ones((r, c)) if signs == "same" else rng.choice([-1.0, 1.0], size=(r, c))
        return sg * x
    A = plane(m, k) + 1j * plane(m, k)
    B = plane(k, n) + 1j * plane(k, n)
    assert_same(gpu_zgemm(A, B, s), oracle.zgemm(A, B, s))
