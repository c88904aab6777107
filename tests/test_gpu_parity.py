"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element.

Integer results (exponents, INT8 slices, INT32 slice products) must be bit-exact; the final FP64
C must be bit-exact as well, because the order of the FP64 sum is fixed by the contract
(diagonals least significant first, one ldexp at the end). No tolerance is used anywhere except
in the accuracy test, whose bound 2^-50 (|A||B|) is the one the build's target states.
"""
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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_split_rows(A, s):
    m, k = A.shape
    mp, kp = ozimmu.slice_geometry(m, k)
    S = torch.full((s, mp, kp), 77, dtype=torch.int8, device=DEV)  # poison: padding must be written
    E = torch.full((max(m, 1),), -12345, dtype=torch.int32, device=DEV)
    ozimmu.split_rows(dev(A), s, S, E)
    torch.cuda.synchronize()
    return E.cpu().numpy()[:m], ozimmu.unpack_slices(S.cpu().numpy(), s, m, k), S


def gpu_split_cols(B, s):
    k, n = B.shape
    npad, kp = ozimmu.slice_geometry(n, k)
    S = torch.full((s, npad, kp), 77, dtype=torch.int8, device=DEV)
    E = torch.full((max(n, 1),), -12345, dtype=torch.int32, device=DEV)
    scratch = torch.empty(max(npad, 1), dtype=torch.int64, device=DEV)
    ozimmu.split_cols(dev(B), s, S, E, scratch)
    torch.cuda.synchronize()
    return E.cpu().numpy()[:n], ozimmu.unpack_slices(S.cpu().numpy(), s, n, k), S


def gpu_dgemm(A, B, s, ldc_extra=0):
    m, k = A.shape
    n = B.shape[1]
    Cbuf = torch.full((m, n + ldc_extra), float("nan"), dtype=torch.float64, device=DEV)
    C = Cbuf[:, :n]
    ws = ozimmu.alloc_workspace(m, n, k, s)
    ozimmu.dgemm(dev(A), dev(B), C, s, ws)
    torch.cuda.synchronize()
    if ldc_extra:
        assert torch.isnan(Cbuf[:, n:]).all()
    return C.cpu().numpy()


def check_split(Eg, Sg, Eo, So, rows, k):
    assert np.array_equal(Eg, Eo)
    assert np.array_equal(Sg[:, :rows, :k], So)
    pad = Sg.copy()
    pad[:, :rows, :k] = 0
    assert not pad.any(), "padding of the slice tensor must be zero"


# ------------------------------------------------------------------ splitter
@pytest.mark.parametrize("m,k,s,phi,seed", [(64, 64, 7, 0.5, 1), (300, 517, 5, 2.0, 2), (257, 128, 16, 1.0, 3),
                                            (1, 1, 3, 1.0, 4), (5, 1030, 13, 4.0, 5)])
def test_split_rows_matches_oracle(m, k, s, phi, seed):
    A = wl.phi_matrix(m, k, phi, seed)
    Eo, So = oracle.split_rows(A, s)
    Eg, Sg, _ = gpu_split_rows(A, s)
    check_split(Eg, Sg, Eo, So, m, k)


@pytest.mark.parametrize("k,n,s,phi,seed", [(64, 64, 7, 0.5, 1), (517, 300, 5, 2.0, 2), (128, 257, 16, 1.0, 3),
                                            (1, 1, 3, 1.0, 4), (1030, 70, 13, 4.0, 5), (700, 3, 8, 1.0, 6)])
def test_split_cols_matches_oracle(k, n, s, phi, seed):
    B = wl.phi_matrix(k, n, phi, seed)
    Eo, So = oracle.split_cols(B, s)
    Eg, Sg, _ = gpu_split_cols(B, s)
    check_split(Eg, Sg, Eo, So, n, k)


def test_split_adversarial_values():
    A = wl.adversarial_matrix(40, 333, seed=9)
    for s in (1, 8, 16):
        Eo, So = oracle.split_rows(A, s)
        Eg, Sg, _ = gpu_split_rows(A, s)
        check_split(Eg, Sg, Eo, So, 40, 333)
        Bt = np.ascontiguousarray(A.T)
        Eo, So = oracle.split_cols(Bt, s)
        Eg, Sg, _ = gpu_split_cols(Bt, s)
        check_split(Eg, Sg, Eo, So, 40, 333)


def random_bit_patterns(shape, seed, exp_lo=0, exp_hi=2046):
    """Doubles drawn as raw bit patterns: random sign and 52-bit fraction, exponent field uniform in
    [exp_lo, exp_hi] (0 = subnormals and zeros, 2046 = the largest finite binade)."""
    rng = np.random.default_rng(seed)
    frac = rng.integers(0, 1 << 52, size=shape, dtype=np.uint64)
    expo = rng.integers(exp_lo, exp_hi + 1, size=shape, dtype=np.uint64)
    sign = rng.integers(0, 2, size=shape, dtype=np.uint64)
    return ((sign << np.uint64(63)) | (expo << np.uint64(52)) | frac).view(np.float64)


@pytest.mark.parametrize("s", [3, 9, 16])
def test_split_of_random_bit_patterns(s):
    """Every finite binade, subnormals included, in one matrix: rows whose largest element is near
    DBL_MAX next to subnormal rows, most elements far below their row's first slice."""
    M = random_bit_patterns((70, 333), seed=5)
    M[3, :] = random_bit_patterns((333,), seed=6, exp_lo=0, exp_hi=0)       # a subnormal row
    M[4, :] = 0.0
    Eo, So = oracle.split_rows(M, s)
    Eg, Sg, _ = gpu_split_rows(M, s)
    check_split(Eg, Sg, Eo, So, 70, 333)
    Eo, So = oracle.split_cols(np.ascontiguousarray(M.T), s)
    Eg, Sg, _ = gpu_split_cols(np.ascontiguousarray(M.T), s)
    check_split(Eg, Sg, Eo, So, 70, 333)


def test_dgemm_of_random_bit_patterns_bit_exact():
    """Exponent fields spread over 600 binades (the result stays finite), and over all binades (the scale
    2^(EA+EB) overflows for part of the outputs: both sides must then give the same infinities, never NaN)."""
    for lo, hi, seed in ((723, 1323, 7), (0, 2046, 8)):
        A = random_bit_patterns((130, 200), seed, lo, hi)
        B = random_bit_patterns((200, 90), seed + 100, lo, hi)
        got, want = gpu_dgemm(A, B, 8), oracle.dgemm(A, B, 8)
        assert not np.isnan(want).any() and np.array_equal(bits(got), bits(want))
    assert np.isinf(want).any()


def test_split_respects_leading_dimension():
    big = wl.phi_matrix(50, 200, 1.0, seed=3)
    view = big[:, 10:150]
    t = dev(big)[:, 10:150]
    s = 6
    mp, kp = ozimmu.slice_geometry(50, 140)
    S = torch.zeros((s, mp, kp), dtype=torch.int8, device=DEV)
    E = torch.zeros(50, dtype=torch.int32, device=DEV)
    ozimmu.split_rows(t, s, S, E)
    Eo, So = oracle.split_rows(view, s)
    assert np.array_equal(E.cpu().numpy(), Eo)
    assert np.array_equal(ozimmu.unpack_slices(S.cpu().numpy(), s, 50, 140)[:, :50, :140], So)
    npad, kp = ozimmu.slice_geometry(140, 50)
    S = torch.zeros((s, npad, kp), dtype=torch.int8, device=DEV)
    E = torch.zeros(140, dtype=torch.int32, device=DEV)
    ozimmu.split_cols(t, s, S, E, torch.empty(npad, dtype=torch.int64, device=DEV))
    Eo, So = oracle.split_cols(view, s)
    assert np.array_equal(E.cpu().numpy(), Eo)
    assert np.array_equal(ozimmu.unpack_slices(S.cpu().numpy(), s, 140, 50)[:, :140, :50], So)


# ------------------------------------------------------------------ INT32 slice products
@pytest.mark.parametrize("m,n,k,s,seed", [(64, 64, 64, 3, 1), (300, 270, 517, 4, 2), (513, 255, 1024, 2, 3)])
def test_slice_products_bit_exact(m, n, k, s, seed):
    A, B = wl.phi_pair(m, n, k, 1.0, seed)
    _, SAo = oracle.split_rows(A, s)
    _, SBo = oracle.split_cols(B, s)
    _, _, SA = gpu_split_rows(A, s)
    _, _, SB = gpu_split_cols(B, s)
    P = torch.full((m, n + 3), -7, dtype=torch.int32, device=DEV)
    for p in range(1, s + 1):
        for q in range(1, s + 1):
            ozimmu.slice_gemm(m, n, k, SA, SB, p, q, 0, k, P[:, :n])
            torch.cuda.synchronize()
            got = P.cpu().numpy()
            assert np.array_equal(got[:, :n].astype(np.int64), oracle.pair_product(SAo[p - 1], SBo[q - 1])), (p, q)
            assert (got[:, n:] == -7).all()


def test_slice_product_k_blocks():
    m, n, k, s = 70, 90, 1000, 2
    A, B = wl.phi_pair(m, n, k, 2.0, seed=5)
    _, SAo = oracle.split_rows(A, s)
    _, SBo = oracle.split_cols(B, s)
    _, _, SA = gpu_split_rows(A, s)
    _, _, SB = gpu_split_cols(B, s)
    P = torch.zeros((m, n), dtype=torch.int32, device=DEV)
    for k0, klen in [(0, 128), (128, 512), (640, 360), (896, 104), (0, 0), (896, 0), (0, 1000)]:
        ozimmu.slice_gemm(m, n, k, SA, SB, 2, 1, k0, klen, P)
        torch.cuda.synchronize()
        assert np.array_equal(P.cpu().numpy().astype(np.int64), oracle.pair_product(SAo[1], SBo[0], k0, klen)), (k0, klen)


def test_int32_block_limit_with_saturating_slices():
    """All chunks 127: one INT32 sum holds 2^17 products without overflow (127^2 2^17 < 2^31)."""
    k = ozimmu.INT32_BLOCK + 256
    A = wl.saturating_matrix(3, k)
    B = wl.saturating_matrix(k, 2)
    A[1, :] *= -1.0
    _, _, SA = gpu_split_rows(A, 2)
    _, _, SB = gpu_split_cols(B, 2)
    P = torch.zeros((3, 2), dtype=torch.int32, device=DEV)
    ozimmu.slice_gemm(3, 2, k, SA, SB, 1, 1, 128, ozimmu.INT32_BLOCK, P)
    torch.cuda.synchronize()
    want = np.array([[1, 1], [-1, -1], [1, 1]], dtype=np.int64) * (ozimmu.INT32_BLOCK * 16129)
    assert np.array_equal(P.cpu().numpy().astype(np.int64), want)
    _, SAo = oracle.split_rows(A, 2)
    _, SBo = oracle.split_cols(B, 2)
    assert np.array_equal(want, oracle.pair_product(SAo[0], SBo[0], 128, ozimmu.INT32_BLOCK))


# ------------------------------------------------------------------ end to end
@pytest.mark.parametrize("s", [3, 5, 7])
def test_config1_64_cubed_bit_exact(s):
    A, B = wl.phi_pair(64, 64, 64, 0.5, seed=1)
    assert np.array_equal(bits(gpu_dgemm(A, B, s)), bits(oracle.dgemm(A, B, s)))


@pytest.mark.parametrize("m,n,k,s,phi,seed", [(300, 270, 517, 8, 1.0, 2), (257, 513, 130, 13, 2.0, 3),
                                              (1, 1, 1, 1, 1.0, 4), (255, 256, 128, 16, 0.5, 5),
                                              (520, 100, 2000, 2, 4.0, 6),
                                              # a few more shapes with ragged tiles in every dimension
                                              (300, 270, 1024, 8, 1.0, 7), (300, 270, 1025, 8, 1.0, 8),
                                              (513, 385, 1300, 7, 2.0, 9), (129, 640, 3000, 11, 1.0, 10)])
def test_dgemm_ragged_shapes_bit_exact(m, n, k, s, phi, seed):
    A, B = wl.phi_pair(m, n, k, phi, seed)
    assert np.array_equal(bits(gpu_dgemm(A, B, s, ldc_extra=5)), bits(oracle.dgemm(A, B, s)))


def random_shapes(count, seed, budget=1.5e9):
    """Seeded shapes and slice counts, ragged on purpose, with the oracle's work (pairs * m * n * k) bounded."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        s = int(rng.integers(1, 17))
        m, n = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        k = int(rng.choice([rng.integers(1, 200), rng.integers(200, 1100), rng.integers(1100, 6000)]))
        if s * (s + 1) // 2 * m * n * k <= budget:
            out.append((m, n, k, s, float(rng.choice([0.5, 1.0, 2.0, 4.0]))))
    return out


@pytest.mark.parametrize("case", range(20))
def test_dgemm_seeded_random_shapes_bit_exact(case):
    m, n, k, s, phi = random_shapes(20, seed=2024)[case]
    print(f"m={m} n={n} k={k} s={s} phi={phi}", flush=True)
    A, B = wl.phi_pair(m, n, k, phi, seed=100 + case)
    assert np.array_equal(bits(gpu_dgemm(A, B, s, ldc_extra=case % 3)), bits(oracle.dgemm(A, B, s)))


@pytest.mark.parametrize("m,n,k,s", [(300000, 2, 3, 8), (2, 300000, 3, 8), (3, 2, 200000, 8), (70000, 3, 1500, 4),
                                     (1, 1, 140000, 16)])
def test_dgemm_extreme_aspect_ratios_bit_exact(m, n, k, s):
    """Thousands of tiles along one dimension and a single ragged one along the other; very long k with a
    handful of outputs (INT64 diagonal sums, two bands at 16 slices)."""
    A, B = wl.phi_pair(m, n, k, 1.0, seed=41)
    assert np.array_equal(bits(gpu_dgemm(A, B, s)), bits(oracle.dgemm(A, B, s)))


@pytest.mark.parametrize("m,n,k", [(4194304, 1, 1), (1, 4194304, 2), (1, 2, 4194304)])
def test_dgemm_at_the_largest_accepted_dimension(m, n, k):
    """OZIMMU_MAX_DIM = 2^22 in each position (65536 tiles along m, 32768 along n; 131072 k-steps in one INT64-summed walk)."""
    s = 3
    print(f"m={m} n={n} k={k}", flush=True)
    A, B = wl.phi_pair(m, n, k, 1.0, seed=43)
    assert np.array_equal(bits(gpu_dgemm(A, B, s)), bits(oracle.dgemm(A, B, s)))


@pytest.mark.parametrize("phi", [0.5, 1.0, 2.0])
def test_config2_1024_cubed_bit_exact_and_accuracy(phi):
    """Every slice count of the sweep s = 3 .. 13; sampled rows (at least one in every 64-row tile) bit
    for bit against the oracle; the scaled error against the double-double product must not grow with s
    until it has reached the 2^-50 level, and must stay there."""
    A, B = wl.phi_pair(1024, 1024, 1024, phi, seed=2)
    hi, lo = oracle.dd_gemm(A, B)
    G = oracle.abs_gemm(A, B)
    rows = np.arange(0, 1024, 37)
    assert len(set(rows // 64)) == 16
    floor = 2.0 ** -50
    prev = None
    for s in range(3, 14):
        C = gpu_dgemm(A, B, s)
        ref = oracle.dgemm(A[rows], B, s)  # separability: rows of C depend on the same rows of A only
        assert np.array_equal(bits(C[rows]), bits(ref)), s
        err = float(np.max(np.abs((C - hi) - lo) / G))
        if prev is not None:
            assert err <= prev if prev > floor else err <= floor, (s, err, prev)
        prev = err
    assert prev <= floor  # accuracy target once s is large enough (s = 13)


def test_dgemm_adversarial_values_bit_exact():
    A = wl.adversarial_matrix(40, 300, seed=1)
    B = np.ascontiguousarray(wl.adversarial_matrix(35, 300, seed=2).T)
    A[5, :] *= 2.0 ** -600   # keep products of the extreme rows finite
    for s in (1, 4, 9):
        assert np.array_equal(bits(gpu_dgemm(A, B, s)), bits(oracle.dgemm(A, B, s)))


def test_dgemm_integer_matrices_equal_plain_matmul():
    A = wl.integer_matrix(130, 400, seed=1)
    B = wl.integer_matrix(400, 90, seed=2)
    C = gpu_dgemm(A, B, 4)
    assert np.array_equal(C, (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64))


def test_dgemm_subnormal_and_overflowing_scale():
    A = np.array([[1.2345678901234567e-160, -3.3e-161, 2e-162]])
    B = np.array([[7.7e-160], [1.1e-159], [5e-158]])
    assert np.array_equal(bits(gpu_dgemm(A, B, 10)), bits(oracle.dgemm(A, B, 10)))
    A = np.array([[1.5e200, 1.0e200]])
    B = np.array([[1.5e200], [1.0e200]])
    got, want = gpu_dgemm(A, B, 6), oracle.dgemm(A, B, 6)
    assert np.isinf(want[0, 0]) and np.array_equal(bits(got), bits(want))


def test_dgemm_k_blocking_long_diagonals():
    """s * k_pad > 2^17 forces the INT64 path: registers are flushed every 2^17 products."""
    m, n, k, s = 40, 50, 70000, 2
    A, B = wl.phi_pair(m, n, k, 2.0, seed=7)
    assert s * ozimmu.slice_geometry(m, k)[1] > ozimmu.INT32_BLOCK
    assert np.array_equal(bits(gpu_dgemm(A, B, s)), bits(oracle.dgemm(A, B, s)))
    # saturating slices across a block boundary: a single INT32 would overflow here
    k = ozimmu.INT32_BLOCK + 640
    A = wl.saturating_matrix(2, k)
    B = wl.saturating_matrix(k, 2)
    assert np.array_equal(bits(gpu_dgemm(A, B, 3)), bits(oracle.dgemm(A, B, 3)))


def test_degenerate_shapes():
    ws = torch.empty(256, dtype=torch.uint8, device=DEV)
    C = torch.full((3, 4), float("nan"), dtype=torch.float64, device=DEV)
    ozimmu.dgemm(torch.empty((3, 0), dtype=torch.float64, device=DEV),
                 torch.empty((0, 4), dtype=torch.float64, device=DEV), C, 5, ws)
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    assert not got.any() and not np.signbit(got).any()
    ozimmu.dgemm(torch.empty((0, 7), dtype=torch.float64, device=DEV),
                 torch.empty((7, 4), dtype=torch.float64, device=DEV),
                 torch.empty((0, 4), dtype=torch.float64, device=DEV), 5, None)
    torch.cuda.synchronize()


def test_two_runs_identical_and_stream_argument():
    A, B = wl.phi_pair(300, 300, 700, 1.0, seed=11)
    C1 = gpu_dgemm(A, B, 8)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        C2 = gpu_dgemm(A, B, 8)
    assert np.array_equal(bits(C1), bits(C2))


# ------------------------------------------------------------------ complex
@pytest.mark.parametrize("m,n,k,s", [(64, 64, 64, 7), (130, 70, 256, 7), (33, 300, 100, 11),
                                     # longer k, INT32 and INT64 sums
                                     (70, 50, 1300, 6), (300, 260, 1100, 9), (20, 30, 70000, 2)])
def test_zgemm_bit_exact(m, n, k, s):
    A = wl.gaussian_complex(m, k, seed=1)
    B = wl.unit_column_complex(k, n, seed=2)
    C = torch.full((m, n), complex(float("nan"), float("nan")), dtype=torch.complex128, device=DEV)
    ws = ozimmu.alloc_workspace(m, n, k, s, is_complex=True)
    ozimmu.zgemm(dev(A), dev(B), C, s, ws)
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    want = oracle.zgemm(A, B, s)
    assert np.array_equal(bits(got.real.copy()), bits(want.real.copy()))
    assert np.array_equal(bits(got.imag.copy()), bits(want.imag.copy()))


@pytest.mark.parametrize("s", range(1, 17))
@pytest.mark.parametrize("k", [96, 128, 200])
def test_zgemm_one_launch_every_slice_count(s, k):
    """The four real products walked by one workgroup per tile, for every kernel instantiation: one
    continuous stream of steps up to eight slices (k = 96: exactly the three steps the walk runs ahead, k = 128:
    one more),
    a pipeline per band beyond; two tile rows and columns with ragged edges."""
    m, n = 70, 140
    A = wl.gaussian_complex(m, k, seed=10 + s)
    B = wl.unit_column_complex(k, n, seed=30 + s)
    C = torch.full((m, n), complex(float("nan"), float("nan")), dtype=torch.complex128, device=DEV)
    ozimmu.zgemm(dev(A), dev(B), C, s, ozimmu.alloc_workspace(m, n, k, s, is_complex=True))
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    want = oracle.zgemm(A, B, s)
    assert np.array_equal(bits(got.real.copy()), bits(want.real.copy()))
    assert np.array_equal(bits(got.imag.copy()), bits(want.imag.copy()))


# ------------------------------------------------------------------ HIP graph capture
def test_dgemm_captured_in_a_graph_replays_correctly():
    """The library only enqueues kernels on the caller's stream (no memsets, no allocation, no
    synchronisation), so a call can be captured and replayed. Each replay runs on new input data
    written into the captured buffers, with eager work and synchronisations in between, and is
    checked against the oracle and against the eager call."""
    m, n, k, s = 300, 270, 1300, 8
    A = torch.empty((m, k), dtype=torch.float64, device=DEV)
    B = torch.empty((k, n), dtype=torch.float64, device=DEV)
    C = torch.empty((m, n), dtype=torch.float64, device=DEV)
    ws = ozimmu.alloc_workspace(m, n, k, s)
    A0, B0 = wl.phi_pair(m, n, k, 1.0, seed=50)
    A.copy_(dev(A0)); B.copy_(dev(B0))
    ozimmu.dgemm(A, B, C, s, ws)            # warm-up outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            ozimmu.dgemm(A, B, C, s, ws, stream=side)
    for seed in (51, 52, 53):
        Ah, Bh = wl.phi_pair(m, n, k, 2.0, seed=seed)
        A.copy_(dev(Ah)); B.copy_(dev(Bh))
        C.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = C.cpu().numpy()
        assert np.array_equal(bits(got), bits(oracle.dgemm(Ah, Bh, s))), seed
        assert np.array_equal(bits(got), bits(gpu_dgemm(Ah, Bh, s))), seed


def test_standalone_cpp_example_runs():
    """The C ABI without Python or a framework: a small HIP host program (built with the library) picks
    the lossless slice count, multiplies and checks itself against a plain FP64 loop."""
    import subprocess
    from pathlib import Path

    exe = Path(ozimmu.__file__).resolve().parent / "example_dgemm"
    if not exe.exists():
        pytest.skip("example_dgemm has not been built (python -m paper_2306_11975_amd.build)")
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "lossless split" in res.stdout
