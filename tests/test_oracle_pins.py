"""Pins for the CPU oracle: it is checked against what the paper and the mathematics fix,
never against itself. Every check here uses an independent formulation (Python integers on
raw bit patterns, exact rationals, closed forms, a library integer matmul) so that a dropped
term, a wrong sign or index, or a transposed operand in oracle/ozaki_oracle.c fails a test.
"""
import math
import struct
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest

import oracle
from paper_2306_11975_amd import workloads as wl

W = 7
GOLDEN = Path(__file__).parent / "golden" / "paper_closed_forms.txt"


def golden():
    out = {}
    for line in GOLDEN.read_text().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        key, val, _ = [t.strip() for t in line.split("|", 2)]
        out[key] = float(val)
    return out


# ------------------------------------------------------------------ independent helpers
def decompose(x: float):
    """double -> (sign, M, ex) with |x| = M * 2^ex exactly, M a Python integer."""
    bits = struct.unpack("<Q", struct.pack("<d", x))[0]
    sign = bits >> 63
    e = (bits >> 52) & 0x7FF
    mant = bits & ((1 << 52) - 1)
    if e == 0:
        return sign, mant, -1074
    return sign, mant | (1 << 52), e - 1075


def brute_exponent(row):
    """Smallest E with max|x| < 2^E, from integer bit lengths (0 for a zero row)."""
    best = None
    for x in row:
        _, M, ex = decompose(float(x))
        if M == 0:
            continue
        e = M.bit_length() + ex
        best = e if best is None else max(best, e)
    return 0 if best is None else best


def brute_chunks(x: float, E: int, s: int):
    """7-bit chunks of |x| 2^-E below the binary point, by integer shifts only."""
    sign, M, ex = decompose(float(x))
    out = []
    for p in range(1, s + 1):
        sh = ex - E + W * p  # floor(M * 2^sh) mod 128
        v = (M << sh) if sh >= 0 else (M >> (-sh))
        v &= 127
        out.append(-v if sign else v)
    return out


def exact_product(A, B):
    """Exact A.B as Fractions via one common power-of-two scale per matrix."""
    def ints(Mx):
        parts = [[decompose(float(v)) for v in row] for row in Mx]
        emin = min(ex for row in parts for (_, _, ex) in row)
        return [[(-1 if sg else 1) * (Mi << (ex - emin)) for (sg, Mi, ex) in row] for row in parts], emin

    Ai, ea = ints(A)
    Bi, eb = ints(B)
    m, k, n = len(Ai), len(Ai[0]), len(Bi[0])
    scale = Fraction(2) ** (ea + eb)
    return [[Fraction(sum(Ai[i][l] * Bi[l][j] for l in range(k))) * scale for j in range(n)] for i in range(m)]


def frac_matrix(C):
    return [[Fraction(float(v)) for v in row] for row in C]


# ------------------------------------------------------------------ closed forms (Sec. 2.3, 3.2)
def test_alpha_and_bps_closed_forms_match_paper_text():
    g = golden()
    # Eq. (3) with u_acc = 2^-24 equals Eq. (4) with l_acc = 24
    assert oracle.alpha(24, 4096) == g["alpha_fp32_k4096"]
    # plain FP16 arithmetic: alpha stays positive up to k = 2^9 and not beyond
    assert oracle.alpha(11, 2 ** g["fp16_arith_max_log2k"]) >= 1
    assert oracle.alpha(11, 2 ** (g["fp16_arith_max_log2k"] + 1)) < 1
    # FP16 Tensor Core (FP32 inside): positive up to 2^22
    assert oracle.alpha(24, 2 ** g["fp16_tc_max_log2k"]) >= 1
    assert oracle.alpha(24, 2 ** (g["fp16_tc_max_log2k"] + 1)) < 1
    lin, lacc = int(g["int8_lin"]), int(g["int8_lacc"])
    for lg in range(1, int(g["int8_bps_full_below_log2k"])):
        assert oracle.bps(lin, lacc, 2.0 ** lg) == lin
    assert oracle.bps(lin, lacc, 2.0 ** g["int8_bps_full_below_log2k"]) == lin - 1
    # BPS never exceeds either bound
    for lg in range(1, 25):
        b = oracle.bps(lin, lacc, 2.0 ** lg)
        assert b == min(lin, (lacc - lg) // 2)


def test_pair_count_closed_form():
    g = golden()
    assert oracle.num_pairs(9) == g["pairs_s9"]
    assert oracle.num_pairs(10) == g["pairs_s10"]
    assert oracle.num_pairs(20) == g["pairs_s20"]
    for s in range(1, 21):
        assert oracle.num_pairs(s) == s * (s + 1) // 2


def test_int8_vs_int12_operation_ratio():
    """Mantissa space 70: INT8 needs 10 slices (55 products); INT12 at k = 2^12 has BPS 9,
    8 slices, 36 products: ratio 1.52...; from 2^16 on both have BPS 7."""
    g = golden()
    space = 70
    k = 2.0 ** 12
    s8 = math.ceil(space / oracle.bps(7, 31, k))
    s12 = math.ceil(space / oracle.bps(int(g["int12_lin"]), 31, k))
    ratio = oracle.num_pairs(s8) / oracle.num_pairs(s12)
    assert math.floor(ratio * 100) / 100 == g["int8_over_int12_ops"]
    for lg in range(int(g["int8_int12_same_from_log2k"]), 21):
        assert oracle.bps(7, 31, 2.0 ** lg) == oracle.bps(11, 31, 2.0 ** lg)


# ------------------------------------------------------------------ exponents
def test_row_exponent_convention_and_invariants():
    A = wl.adversarial_matrix(12, 40, seed=3)
    E, S = oracle.split_rows(A, 4)
    for i in range(A.shape[0]):
        assert E[i] == brute_exponent(A[i]), i
        mu = np.abs(A[i]).max()
        if mu == 0:
            assert E[i] == 0 and not S[:, i, :].any()
        else:
            assert mu < math.ldexp(1.0, int(E[i])) if E[i] < 1024 else True
            assert mu >= math.ldexp(1.0, int(E[i]) - 1)
            # the element that sets the exponent has a leading chunk of at least 64
            assert np.abs(S[0, i, :]).max() >= 64
    assert np.abs(S.astype(np.int32)).max() <= 127
    # exact power of two as row maximum: frexp exponent is one above log2
    assert E[8] == 11


def test_scaling_a_row_by_power_of_two_moves_only_the_exponent():
    A = wl.phi_matrix(6, 50, 1.0, seed=5)
    E0, S0 = oracle.split_rows(A, 6)
    shift = np.array([3, -7, 100, -300, 0, 17])
    E1, S1 = oracle.split_rows(np.ldexp(A, shift[:, None]), 6)
    assert np.array_equal(S0, S1)
    assert np.array_equal(E1 - E0, shift)


def test_split_cols_is_split_rows_of_the_transpose():
    B = wl.adversarial_matrix(9, 33, seed=11).T.copy()  # 33 x 9
    Er, Sr = oracle.split_rows(np.ascontiguousarray(B.T), 5)
    Ec, Sc = oracle.split_cols(B, 5)
    assert np.array_equal(Er, Ec) and np.array_equal(Sr, Sc)
    # and it really reduces over the column: changing one entry of column j changes only row j
    B2 = B.copy()
    B2[4, 2] = 1e30
    Ec2, Sc2 = oracle.split_cols(B2, 5)
    changed = [j for j in range(B.shape[1]) if Ec2[j] != Ec[j] or not np.array_equal(Sc2[:, j], Sc[:, j])]
    assert changed == [2]


# ------------------------------------------------------------------ slices
@pytest.mark.parametrize("seed,phi", [(1, 0.5), (2, 2.0)])
def test_slices_match_integer_brute_force_on_bit_patterns(seed, phi):
    A = wl.phi_matrix(5, 37, phi, seed)
    s = 16
    E, S = oracle.split_rows(A, s)
    for i in range(A.shape[0]):
        for l in range(A.shape[1]):
            assert list(S[:, i, l]) == brute_chunks(A[i, l], int(E[i]), s), (i, l)


def test_slices_brute_force_adversarial():
    A = wl.adversarial_matrix(12, 24, seed=7)
    s = 12
    E, S = oracle.split_rows(A, s)
    for i in range(A.shape[0]):
        for l in range(A.shape[1]):
            assert list(S[:, i, l]) == brute_chunks(A[i, l], int(E[i]), s), (i, l)


def test_slices_brute_force_on_raw_bit_patterns_of_every_binade():
    """Doubles drawn as raw 64-bit patterns (exponent field uniform over 0 .. 2046: subnormals to the
    largest binade; one all-subnormal row), rows and columns, against the Python-integer cut."""
    rng = np.random.default_rng(12)
    shape = (9, 21)
    bits = ((rng.integers(0, 2, size=shape, dtype=np.uint64) << np.uint64(63)) |
            (rng.integers(0, 2047, size=shape, dtype=np.uint64) << np.uint64(52)) |
            rng.integers(0, 1 << 52, size=shape, dtype=np.uint64))
    bits[2, :] &= np.uint64((1 << 52) - 1) | np.uint64(1 << 63)     # subnormal row
    A = bits.view(np.float64)
    s = 16
    E, S = oracle.split_rows(A, s)
    Ec, Sc = oracle.split_cols(np.ascontiguousarray(A.T), s)
    assert np.array_equal(E, Ec) and np.array_equal(S, Sc)          # B is split as its transpose
    for i in range(shape[0]):
        for l in range(shape[1]):
            assert list(S[:, i, l]) == brute_chunks(A[i, l], int(E[i]), s), (i, l)


def test_slice_prefix_property_and_truncation_residual():
    A = wl.phi_matrix(8, 64, 1.0, seed=9)
    E, S13 = oracle.split_rows(A, 13)
    prev = None
    for s in range(1, 14):
        Es, Ss = oracle.split_rows(A, s)
        assert np.array_equal(Es, E)
        assert np.array_equal(Ss, S13[:s])  # slice p does not depend on s
        # residual: same sign, 0 <= |x| - |recon| < 2^(E - 7 s), non-increasing in s
        res = np.zeros(A.shape, dtype=object)
        for i in range(A.shape[0]):
            for l in range(A.shape[1]):
                recon = sum(Fraction(int(Ss[p, i, l])) * Fraction(2) ** (int(E[i]) - W * (p + 1)) for p in range(s))
                x = Fraction(float(A[i, l]))
                r = abs(x) - abs(recon)
                assert 0 <= r < Fraction(2) ** (int(E[i]) - W * s)
                assert recon == 0 or (recon > 0) == (x > 0)
                res[i, l] = r
        if prev is not None:
            assert all(res[i, l] <= prev[i, l] for i in range(A.shape[0]) for l in range(A.shape[1]))
        prev = res


def test_exact_reconstruction_with_enough_slices():
    # a row of equal-exponent values needs ceil(53/7) = 8 slices and not fewer
    rng = np.random.default_rng(4)
    A = (1.0 + rng.random((4, 32))) * rng.choice([-1.0, 1.0], size=(4, 32))  # all in [1,2)
    A[:, 0] = np.nextafter(2.0, 0.0)  # full 53-bit significand present
    for s, exact in [(7, False), (8, True), (11, True)]:
        E, S = oracle.split_rows(A, s)
        recon = np.zeros_like(A)
        for p in range(s):
            recon += np.ldexp(S[p].astype(np.float64), (E - W * (p + 1))[:, None])
        assert (np.array_equal(recon, A)) == exact
    # general rule: exact iff 7 s >= 53 + E_i - frexp_exp(x) for the elements present
    A = wl.phi_matrix(6, 40, 2.0, seed=21)
    s = 10
    E, S = oracle.split_rows(A, s)
    for i in range(A.shape[0]):
        for l in range(A.shape[1]):
            recon = sum(Fraction(int(S[p, i, l])) * Fraction(2) ** (int(E[i]) - W * (p + 1)) for p in range(s))
            _, M, ex = decompose(float(A[i, l]))
            lowest_bit = ex + ((M & -M).bit_length() - 1)  # place of the last set bit
            assert (recon == Fraction(float(A[i, l]))) == (lowest_bit >= int(E[i]) - W * s)


# ------------------------------------------------------------------ integer products
def test_pair_products_match_library_integer_matmul_and_bounds():
    A, B = wl.phi_pair(23, 19, 77, 1.0, seed=2)
    s = 5
    EA, SA = oracle.split_rows(A, s)
    EB, SB = oracle.split_cols(B, s)
    for p in range(s):
        for q in range(s):
            P = oracle.pair_product(SA[p], SB[q])
            ref = SA[p].astype(np.int64) @ SB[q].astype(np.int64).T
            assert np.array_equal(P, ref)
            assert np.abs(P).max() <= 77 * 127 * 127
    # k-range blocks add up to the whole
    P = oracle.pair_product(SA[1], SB[2])
    parts = oracle.pair_product(SA[1], SB[2], 0, 30) + oracle.pair_product(SA[1], SB[2], 30, 40) + \
        oracle.pair_product(SA[1], SB[2], 70, 7)
    assert np.array_equal(P, parts)
    # a transposed operand would fail here: m != n and values are asymmetric
    assert P.shape == (23, 19)


def test_diagonal_sums_are_sums_of_pairs():
    A, B = wl.phi_pair(9, 11, 45, 0.5, seed=6)
    s = 6
    _, SA = oracle.split_rows(A, s)
    _, SB = oracle.split_cols(B, s)
    S = oracle.diagonal_sums(SA, SB)
    for d in range(2, s + 2):
        ref = sum(SA[p - 1].astype(np.int64) @ SB[d - p - 1].astype(np.int64).T for p in range(1, d))
        assert np.array_equal(S[d - 2], ref)


def test_k_permutation_invariance_of_integers_and_final_bits():
    A, B = wl.phi_pair(12, 10, 96, 1.0, seed=8)
    perm = np.random.default_rng(0).permutation(96)
    s = 7
    C0 = oracle.dgemm(A, B, s)
    C1 = oracle.dgemm(A[:, perm], B[perm, :], s)
    assert np.array_equal(C0.view(np.uint64), C1.view(np.uint64))


def test_int32_overflow_bound():
    """All entries 1 - 2^-53: every chunk is 127, so P_{1,1} = 127^2 k. That fits INT32 for
    k = 133144 and not for k = 133145; the contract block length 2^17 fits."""
    lim = 2 ** 31 - 1
    for k, fits in [(133144, True), (133145, False), (2 ** 17, True)]:
        A = wl.saturating_matrix(1, k)
        B = wl.saturating_matrix(k, 1)
        EA, SA = oracle.split_rows(A, 7)
        EB, SB = oracle.split_cols(B, 7)
        assert EA[0] == 0 and EB[0] == 0
        assert (SA == 127).all() and (SB == 127).all()
        P = oracle.pair_product(SA[0], SB[0])
        assert P[0, 0] == k * 16129
        assert (P[0, 0] <= lim) == fits


# ------------------------------------------------------------------ scale + sum
@pytest.mark.parametrize("s", [1, 2, 5, 9])
def test_integer_matrices_reduce_to_plain_integer_matmul(s):
    """|entry| <= 127 integers live entirely in slice 1, so C must be the exact integer
    product, which plain FP64 matmul also delivers bit for bit."""
    A = wl.integer_matrix(17, 40, seed=1)
    B = wl.integer_matrix(40, 13, seed=2)
    A[3, :] = 0
    exact = A.astype(np.int64) @ B.astype(np.int64)
    C = oracle.dgemm(A, B, s)
    assert np.array_equal(C, exact.astype(np.float64))
    assert np.array_equal(C.view(np.uint64), (A @ B).view(np.uint64))
    E, S = oracle.split_rows(A, max(s, 2))
    assert not S[1:].any()


def test_full_square_of_pairs_with_exact_arithmetic_is_the_exact_product():
    """With enough slices for exact reconstruction, summing ALL s^2 pair products with the
    scale 2^(-7(p+q)) 2^(EA+EB) in exact arithmetic gives exactly A.B (checks the scale
    formula, the exponent vectors, the slices and the pair products together)."""
    A, B = wl.phi_pair(5, 4, 12, 0.5, seed=12)
    s = 16
    EA, SA = oracle.split_rows(A, s)
    EB, SB = oracle.split_cols(B, s)
    exact = exact_product(A.tolist(), B.tolist())
    tot = [[Fraction(0)] * 4 for _ in range(5)]
    for p in range(1, s + 1):
        for q in range(1, s + 1):
            P = oracle.pair_product(SA[p - 1], SB[q - 1])
            for i in range(5):
                for j in range(4):
                    tot[i][j] += Fraction(int(P[i, j])) * Fraction(2) ** (int(EA[i]) + int(EB[j]) - W * (p + q))
    assert tot == exact


def test_accumulate_order_and_rounding_against_exact_rational_replay():
    """Replay the fixed order with exact rationals and one correctly rounded addition per
    step (Fraction -> float is correctly rounded in CPython)."""
    A, B = wl.phi_pair(7, 6, 33, 2.0, seed=14)
    s = 9
    EA, SA = oracle.split_rows(A, s)
    EB, SB = oracle.split_cols(B, s)
    S = oracle.diagonal_sums(SA, SB)
    C = oracle.accumulate(S, EA, EB)
    for i in range(7):
        for j in range(6):
            acc = 0.0
            for d in range(s + 1, 1, -1):
                term = Fraction(int(S[d - 2, i, j])) / Fraction(2) ** (W * d)
                acc = float(Fraction(acc) + term)
            want = float(Fraction(acc) * Fraction(2) ** (int(EA[i]) + int(EB[j])))
            assert C[i, j] == want
    # the end-to-end entry agrees with its own stages
    assert np.array_equal(oracle.dgemm(A, B, s), C)


def test_final_scale_rounds_once_into_the_subnormal_range():
    A = np.array([[1.2345678901234567e-160, -3.3e-161]])
    B = np.array([[7.7e-160], [1.1e-159]])
    C = oracle.dgemm(A, B, 10)
    exact = exact_product(A.tolist(), B.tolist())[0][0]
    assert abs(Fraction(float(C[0, 0])) - exact) <= Fraction(2) ** -1074


# ------------------------------------------------------------------ accuracy of the method
def scaled_errors(A, B, C):
    exact = exact_product(A.tolist(), B.tolist())
    G = oracle.abs_gemm(A, B)
    worst = Fraction(0)
    for i in range(A.shape[0]):
        for j in range(B.shape[1]):
            if G[i, j] == 0:
                continue
            worst = max(worst, abs(Fraction(float(C[i, j])) - exact[i][j]) / Fraction(float(G[i, j])))
    return float(worst)


def test_a_priori_bound_and_monotone_error_and_fp64_floor():
    A, B = wl.phi_pair(24, 24, 64, 0.5, seed=1)
    k = 64
    exact = exact_product(A.tolist(), B.tolist())
    prev = None
    for s in range(2, 14):
        C = oracle.dgemm(A, B, s)
        EA, _ = oracle.split_rows(A, s)
        EB, _ = oracle.split_cols(B, s)
        worst = 0.0
        for i in range(24):
            for j in range(24):
                err = abs(Fraction(float(C[i, j])) - exact[i][j])
                scale = Fraction(2) ** (int(EA[i]) + int(EB[j]))
                bound = k * (s + 1) * Fraction(2) ** (-W * s) * scale * (1 + Fraction(1, 32))
                # truncated pairs + at most s-1 roundings of a sum bounded by k*scale
                bound += (s - 1) * Fraction(2) ** -53 * k * scale
                assert err <= bound, (s, i, j)
        e = scaled_errors(A, B, C)
        if prev is not None:
            assert e <= prev or e <= 2.0 ** -51
        prev = e
    assert prev <= 2.0 ** -50  # the target accuracy once s is large enough


def test_dd_reference_matches_exact_rational_product():
    A, B = wl.phi_pair(10, 9, 50, 2.0, seed=3)
    hi, lo = oracle.dd_gemm(A, B)
    exact = exact_product(A.tolist(), B.tolist())
    G = oracle.abs_gemm(A, B)
    for i in range(10):
        for j in range(9):
            got = Fraction(float(hi[i, j])) + Fraction(float(lo[i, j]))
            assert abs(got - exact[i][j]) <= Fraction(float(G[i, j])) * Fraction(2) ** -98
            assert hi[i, j] == float(exact[i][j])  # hi is the correctly rounded product here
    # |A||B| itself within k ulp of the exact value
    exact_abs = exact_product(np.abs(A).tolist(), np.abs(B).tolist())
    for i in range(10):
        for j in range(9):
            assert abs(Fraction(float(G[i, j])) - exact_abs[i][j]) <= exact_abs[i][j] * 51 * Fraction(2) ** -53


def test_pairwise_order_cross_check_agrees_within_rounding():
    A, B = wl.phi_pair(16, 16, 80, 1.0, seed=4)
    s = 8
    C = oracle.dgemm(A, B, s)
    Cp = oracle.dgemm_pairwise_order(A, B, s)
    G = oracle.abs_gemm(A, B)
    EA, _ = oracle.split_rows(A, s)
    EB, _ = oracle.split_cols(B, s)
    tol = oracle.num_pairs(s) * 2.0 ** -53 * 80 * np.ldexp(1.0, EA[:, None] + EB[None, :])
    assert (np.abs(C - Cp) <= tol).all()
    assert np.abs(C - Cp).max() <= 2.0 ** -45 * G.max()


# ------------------------------------------------------------------ complex
def test_complex_product_against_exact_rational():
    A = wl.gaussian_complex(6, 20, seed=1)
    B = wl.unit_column_complex(20, 5, seed=2)
    s = 11
    C = oracle.zgemm(A, B, s)
    rr = exact_product(A.real.tolist(), B.real.tolist())
    ii = exact_product(A.imag.tolist(), B.imag.tolist())
    ri = exact_product(A.real.tolist(), B.imag.tolist())
    ir = exact_product(A.imag.tolist(), B.real.tolist())
    G = oracle.abs_gemm(np.abs(A.real) + np.abs(A.imag), np.abs(B.real) + np.abs(B.imag))
    for i in range(6):
        for j in range(5):
            assert abs(Fraction(float(C[i, j].real)) - (rr[i][j] - ii[i][j])) <= Fraction(float(G[i, j])) * Fraction(2) ** -50
            assert abs(Fraction(float(C[i, j].imag)) - (ri[i][j] + ir[i][j])) <= Fraction(float(G[i, j])) * Fraction(2) ** -50
    # structure: it is exactly the four real products combined with one rounding each
    Cr = oracle.dgemm(A.real, B.real, s) - oracle.dgemm(A.imag, B.imag, s)
    Ci = oracle.dgemm(A.real, B.imag, s) + oracle.dgemm(A.imag, B.real, s)
    assert np.array_equal(C.real, Cr) and np.array_equal(C.imag, Ci)
    # a sign error in the real part would show: purely imaginary inputs give a negative real product
    Z = oracle.zgemm(np.array([[1j]]), np.array([[1j]]), 3)
    assert Z[0, 0] == -1.0


def test_degenerate_shapes():
    assert oracle.dgemm(np.zeros((0, 5)), np.zeros((5, 3)), 4).shape == (0, 3)
    C = oracle.dgemm(np.ones((3, 0)), np.ones((0, 2)), 4)
    assert C.shape == (3, 2) and not C.any() and not np.signbit(C).any()
    C = oracle.dgemm(np.array([[1.5, -1.5]]), np.array([[2.0], [2.0]]), 6)
    assert C[0, 0] == 0.0 and not np.signbit(C[0, 0])


# ------------------------------------------------------------------ INT8-AUTO (Section 4.4)
def brute_loss_sums(M, by_columns, s_max=16):
    """Lost mantissa bits per slice count from the raw bit patterns: every stored bit of the
    significand is placed at its position after the binary point of |x| 2^-E and counted if it
    lies beyond the 7 s positions that s slices keep."""
    M = np.asarray(M, dtype=np.float64)
    vecs = M.T if by_columns else M
    sums = [0] * s_max
    for vec in vecs:
        E = brute_exponent(vec)
        for x in vec:
            _, Mi, ex = decompose(float(x))
            if Mi == 0:
                continue
            nbits = 53 if Mi >> 52 else Mi.bit_length()     # stored significant bits
            # bit i of Mi has weight 2^(ex + i); its position after the binary point is E - ex - i
            positions = [E - ex - i for i in range(Mi.bit_length() - nbits, Mi.bit_length())]
            assert min(positions) >= 1
            for s in range(1, s_max + 1):
                sums[s - 1] += sum(1 for q in positions if q > W * s)
    return np.array(sums, dtype=np.uint64)


def test_auto_loss_sums_match_bit_position_brute_force():
    A, B = wl.phi_pair(9, 11, 13, 2.0, seed=21)
    assert np.array_equal(oracle.auto_loss_sums(A, False), brute_loss_sums(A, False))
    assert np.array_equal(oracle.auto_loss_sums(B, True), brute_loss_sums(B, True))
    M = wl.adversarial_matrix(12, 17, seed=5)    # zeros, powers of two, subnormals, huge and tiny rows
    assert np.array_equal(oracle.auto_loss_sums(M, False), brute_loss_sums(M, False))
    assert np.array_equal(oracle.auto_loss_sums(M, True), brute_loss_sums(M, True))


def test_auto_single_binade_closed_form():
    """All entries in [1, 2): no leading zeros anywhere, every element loses max(0, 53 - 7 s) bits,
    so the choice is ceil((53 - T) / 7) whatever the shape."""
    rng = np.random.default_rng(3)
    A = 1.0 + rng.random((20, 30))
    B = -(1.0 + rng.random((30, 10)))
    sums = oracle.auto_loss_sums(A, False)
    assert [int(v) for v in sums] == [A.size * max(0, 53 - 7 * s) for s in range(1, 17)]
    for T, want in ((0, 8), (3, 8), (4, 7), (10.99, 7), (11, 6), (25, 4), (46, 1), (60, 1)):
        assert oracle.auto_num_slices(A, B, T)[0] == want, T
    assert oracle.auto_num_slices(A, B, 0, s_max=6)[0] == 6      # nothing qualifies: the maximum is returned


def test_auto_threshold_zero_means_exact_split_and_is_minimal():
    A, B = wl.phi_pair(15, 12, 20, 1.5, seed=8)
    s, sums = oracle.auto_num_slices(A, B, 0.0)
    assert (sums[:, s - 1] == 0).all() and (sums[:, s - 2] > 0).any()
    EA, SA = oracle.split_rows(A, s)
    EB, SB = oracle.split_cols(B, s)
    for (E, S, M) in ((EA, SA, A), (EB, SB, B.T)):
        for i in range(M.shape[0]):
            for l in range(M.shape[1]):
                rec = sum(Fraction(int(S[p, i, l])) * Fraction(2) ** (int(E[i]) - W * (p + 1)) for p in range(s))
                assert rec == Fraction(float(M[i, l]))


def test_auto_monotone_and_scale_invariant():
    A, B = wl.phi_pair(30, 25, 40, 2.0, seed=4)
    picks = [oracle.auto_num_slices(A, B, T)[0] for T in (0, 0.25, 0.5, 1, 2, 4, 8, 16, 32, 53)]
    assert picks == sorted(picks, reverse=True) and picks[-1] == 1
    sums = oracle.auto_loss_sums(A, False)
    assert all(int(sums[i]) >= int(sums[i + 1]) for i in range(15))
    assert all(int(sums[i]) - int(sums[i + 1]) <= 7 * A.size for i in range(15))
    A2 = A * np.ldexp(1.0, np.arange(30) % 9 - 4)[:, None]       # rows scaled by powers of two
    assert np.array_equal(oracle.auto_loss_sums(A2, False), sums)
    # a complex input is judged plane by plane
    Z = A + 1j * A[::-1]
    s_c, sums_c = oracle.auto_num_slices(Z, B, 1.0)
    assert sums_c.shape == (3, 16)
    assert s_c == max(oracle.auto_num_slices(A, B, 1.0)[0], oracle.auto_num_slices(A[::-1].copy(), B, 1.0)[0])


def test_auto_on_random_unitary_gate_is_in_the_range_the_paper_reports():
    """Section 4.4 reports 12-13 slices at T = 0 and 8-9 at T = 1 for its random-unitary circuits.
    Those circuits are defined in a figure that is not available, so this is a plausibility check
    on the same kind of input (Haar-like unitary from the QR of a complex Gaussian matrix applied to
    a normalised random state reshaped to 2^(N-d) x 2^d), not a like-for-like pin."""
    rng = np.random.default_rng(5)
    d, N = 7, 16
    G = rng.standard_normal((2 ** d, 2 ** d)) + 1j * rng.standard_normal((2 ** d, 2 ** d))
    Q, _ = np.linalg.qr(G)
    psi = rng.standard_normal(2 ** N) + 1j * rng.standard_normal(2 ** N)
    psi /= np.linalg.norm(psi)
    A = psi.reshape(2 ** (N - d), 2 ** d)
    g = golden()
    # one slice of slack below the reported range: the paper's state vectors are larger (wider spread)
    assert g["auto_t0_slices_low"] - 1 <= oracle.auto_num_slices(A, Q, 0.0)[0] <= g["auto_t0_slices_high"]
    assert g["auto_t1_slices_low"] <= oracle.auto_num_slices(A, Q, 1.0)[0] <= g["auto_t1_slices_high"]


# ------------------------------------------------------------------ BLAS-style call (Section 4.4)
@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
def test_blas_call_reduces_to_plain_integer_arithmetic(ta, tb):
    """Integer matrices |x| <= 127 live in slice 1, so G is the exact integer product for any s, and
    with integer alpha, beta and C every operation of the update is exact: the whole call must equal
    numpy's integer arithmetic. A transposed operand, a wrong leading dimension or swapped m/n fails."""
    rng = np.random.default_rng(17)
    m, n, k = 5, 7, 9
    opA = rng.integers(-127, 128, size=(m, k))
    opB = rng.integers(-127, 128, size=(k, n))
    C0 = rng.integers(-1000, 1000, size=(m, n))
    A = opA.T if ta else opA
    B = opB.T if tb else opB
    for alpha, beta in ((1, 0), (3, 0), (1, 1), (-2, 5), (0, 4), (0, 0)):
        got = oracle.dgemm_blas(ta, tb, alpha, A.astype(float), B.astype(float), beta, C0.astype(float), 3)
        want = alpha * (opA @ opB) + beta * C0
        assert np.array_equal(got, want.astype(float)), (alpha, beta)
    # beta = 0 must not read C (BLAS convention): NaN there does not propagate
    got = oracle.dgemm_blas(ta, tb, 1.0, A.astype(float), B.astype(float), 0.0, np.full((m, n), np.nan), 2)
    assert np.array_equal(got, (opA @ opB).astype(float))


def test_blas_call_rounding_order_against_exact_rationals():
    """General values: G from the plain routine (pinned above), then the update replayed in exact
    rationals with the three roundings made explicit."""
    A, B = wl.phi_pair(4, 5, 6, 1.0, seed=31)
    rng = np.random.default_rng(2)
    C0 = rng.standard_normal((4, 5))
    alpha, beta = 1.7, -0.3
    G = oracle.dgemm(A, B, 9)
    got = oracle.dgemm_blas(False, False, alpha, A, B, beta, C0, 9)
    for i in range(4):
        for j in range(5):
            t1 = float(Fraction(alpha) * Fraction(float(G[i, j])))      # float(Fraction) rounds to nearest even
            t2 = float(Fraction(beta) * Fraction(float(C0[i, j])))
            assert got[i, j] == float(Fraction(t1) + Fraction(t2))
    # transposed inputs give the same bits as the plain call on the transposed data
    got_t = oracle.dgemm_blas(True, True, alpha, A.T.copy(), B.T.copy(), beta, C0, 9)
    assert np.array_equal(got_t.view(np.uint64), got.view(np.uint64))


@pytest.mark.parametrize("ta", ["N", "T", "C"])
@pytest.mark.parametrize("tb", ["N", "T", "C"])
def test_complex_blas_call_reduces_to_gaussian_integer_arithmetic(ta, tb):
    """Gaussian-integer matrices with parts |x| <= 127 live in slice 1 of each plane, so the four real
    products are exact integers for any s; with Gaussian-integer alpha, beta and C every operation of
    the update is exact and the call must equal Python's exact complex integer arithmetic. A wrong
    sign of a conjugation, a swapped plane or a transposed operand fails."""
    rng = np.random.default_rng(23)
    m, n, k = 4, 6, 5

    def gauss(shape, lim):
        return rng.integers(-lim, lim + 1, size=shape) + 1j * rng.integers(-lim, lim + 1, size=shape)

    opA, opB, C0 = gauss((m, k), 127), gauss((k, n), 127), gauss((m, n), 500)
    A = {"N": opA, "T": opA.T, "C": opA.conj().T}[ta]
    B = {"N": opB, "T": opB.T, "C": opB.conj().T}[tb]
    for alpha, beta in ((1, 0), (2 - 3j, 0), (1, 1), (-1 + 2j, 3 - 1j), (0, 2j), (0, 0), (1j, 1j)):
        got = oracle.zgemm_blas(ta, tb, alpha, A, B, beta, C0, 3)
        want = alpha * (opA @ opB) + beta * C0      # all parts are integers far below 2^53: exact in complex128
        assert np.array_equal(got, want), (alpha, beta)
    got = oracle.zgemm_blas(ta, tb, 1.0, A, B, 0.0, np.full((m, n), np.nan + 1j * np.nan), 2)
    assert np.array_equal(got, opA @ opB)


def test_complex_blas_call_rounding_order_against_exact_rationals():
    """General values: G from the plain complex routine (pinned elsewhere), then the update replayed in
    exact rationals with every rounding of the stated order made explicit."""
    rng = np.random.default_rng(5)
    m, n, k = 3, 4, 6
    A = rng.standard_normal((m, k)) + 1j * rng.standard_normal((m, k))
    B = rng.standard_normal((k, n)) + 1j * rng.standard_normal((k, n))
    C0 = rng.standard_normal((m, n)) + 1j * rng.standard_normal((m, n))
    alpha, beta = 1.3 - 0.4j, -0.2 + 0.9j
    G = oracle.zgemm(A, B, 9)
    got = oracle.zgemm_blas("N", "N", alpha, A, B, beta, C0, 9)

    def rn(x):
        return float(x)                          # float(Fraction) rounds to nearest even

    def cmul(a, z):
        F = Fraction
        re = rn(F(rn(F(a.real) * F(z.real))) - F(rn(F(a.imag) * F(z.imag))))
        im = rn(F(rn(F(a.real) * F(z.imag))) + F(rn(F(a.imag) * F(z.real))))
        return re, im

    for i in range(m):
        for j in range(n):
            tr, ti = cmul(alpha, complex(G[i, j]))
            ur, ui = cmul(beta, complex(C0[i, j]))
            assert got[i, j].real == rn(Fraction(tr) + Fraction(ur))
            assert got[i, j].imag == rn(Fraction(ti) + Fraction(ui))
    # beta == 0: t alone; alpha == 1 leaves G's bits untouched
    def bits(z):
        return np.ascontiguousarray(z).view(np.uint64)

    assert np.array_equal(bits(oracle.zgemm_blas("N", "N", 1.0, A, B, 0.0, C0, 9)), bits(G))
    # the product is odd in each operand plane, so a conjugate transpose equals the plain call on
    # the explicitly conjugated and transposed data
    got_c = oracle.zgemm_blas("C", "T", alpha, A.conj().T.copy(), B.T.copy(), beta, C0, 9)
    assert np.array_equal(bits(got_c), bits(got))


# ------------------------------------------------------------------ accuracy trends of Section 4.2
def avg_rel_error(C, hi, lo):
    """Eq. (7), averaged: |C - C_dd| / |C_dd| with the double-double reference (hi + lo)."""
    return float(np.mean(np.abs((C - hi) - lo) / np.abs(hi)))


def test_accuracy_trends_the_paper_reports_for_the_exponent_range():
    """Section 4.2 (exponent distribution range): with phi = 0.1 nine slices already beat plain FP64
    DGEMM; with 11 and 13 slices the error is below or about at the level of DGEMM up to phi = 4."""
    n = 192
    for phi, s, factor in ((0.1, 9, 1.0), (1.0, 11, 1.0), (2.0, 13, 1.0), (4.0, 13, 4.0)):
        A = wl.phi_matrix(n, n, phi, seed=41)
        B = wl.phi_matrix(n, n, phi, seed=42)
        hi, lo = oracle.dd_gemm(A, B)
        e_oz = avg_rel_error(oracle.dgemm(A, B, s), hi, lo)
        e_fp = avg_rel_error(A @ B, hi, lo)
        assert e_oz <= factor * e_fp, (phi, s, e_oz, e_fp)
    # and too few slices for a wide range are worse than DGEMM (the disadvantage of Section 3.3)
    A = wl.phi_matrix(n, n, 4.0, seed=41)
    B = wl.phi_matrix(n, n, 4.0, seed=42)
    hi, lo = oracle.dd_gemm(A, B)
    assert avg_rel_error(oracle.dgemm(A, B, 9), hi, lo) > avg_rel_error(A @ B, hi, lo)


def test_zero_cancellation_product_is_more_accurate_than_fp64_gemm():
    """Section 4.2 (zero-cancellation): A ~ N(0,1) times its computed inverse; the reference is the
    double-double product, not the identity. The scheme resolves the cancelling leading digits
    exactly, so with enough slices its error is below that of FP64 DGEMM."""
    n = 160
    rng = np.random.default_rng(43)
    A = rng.standard_normal((n, n))
    X = np.linalg.solve(A, np.eye(n))
    hi, lo = oracle.dd_gemm(A, X)
    e_fp = avg_rel_error(A @ X, hi, lo)
    errs = {s: avg_rel_error(oracle.dgemm(A, X, s), hi, lo) for s in (8, 10, 12, 13)}
    assert errs[12] < e_fp and errs[13] < e_fp
    assert errs[13] <= errs[12] <= errs[10] <= errs[8]


# ------------------------------------------------------------------ double-double summing-up (Section 2.3.4)
def test_dd_summing_up_against_exact_rational_sum():
    """The pair (hi, lo) must represent the exact sum of the scaled integer diagonal sums to about
    2^-104 (double-double addition), and hi must be that sum rounded to nearest."""
    rng = np.random.default_rng(61)
    s, m, n = 14, 6, 5
    S = rng.integers(-(1 << 40), 1 << 40, size=(s, m, n))
    S[3] = 0
    S[:, 0, 0] = 0                                 # an exactly zero element
    S[:, 1, 1] = [(-1) ** d * (1 << 45) for d in range(s)]   # heavy cancellation between diagonals
    EA = rng.integers(-30, 30, size=m)
    EB = rng.integers(-30, 30, size=n)
    hi, lo = oracle.accumulate_dd(S, EA, EB)
    for i in range(m):
        for j in range(n):
            exact = sum(Fraction(int(S[d - 2, i, j])) * Fraction(2) ** (-W * d) for d in range(2, s + 2))
            exact *= Fraction(2) ** int(EA[i] + EB[j])
            got = Fraction(float(hi[i, j])) + Fraction(float(lo[i, j]))
            assert abs(got - exact) <= abs(exact) * Fraction(2) ** -100
            assert hi[i, j] == float(exact)        # float(Fraction) is correctly rounded
            if exact == 0:
                assert hi[i, j] == 0.0 and lo[i, j] == 0.0
    # with few diagonals the exact sum fits 106 bits and the pair is exact
    hi2, lo2 = oracle.accumulate_dd(S[:5], EA, EB)
    for i in range(m):
        for j in range(n):
            exact = sum(Fraction(int(S[d - 2, i, j])) * Fraction(2) ** (-W * d) for d in range(2, 7))
            exact *= Fraction(2) ** int(EA[i] + EB[j])
            assert Fraction(float(hi2[i, j])) + Fraction(float(lo2[i, j])) == exact


def test_dd_product_is_more_accurate_than_fp64_allows():
    """With 14 slices the kept products carry about 2^-80 of |A||B|; the FP64 summing-up throws that
    away (2^-53), the double-double one keeps it: the advantage 'precision higher than FP64'."""
    A, B = wl.phi_pair(24, 20, 200, 0.5, seed=62)
    ref = exact_product(A, B)
    G = oracle.abs_gemm(A, B)
    hi, lo = oracle.dgemm_dd(A, B, 14)
    C64 = oracle.dgemm(A, B, 14)
    worst_dd = max(abs(Fraction(float(hi[i, j])) + Fraction(float(lo[i, j])) - ref[i][j]) / Fraction(float(G[i, j]))
                   for i in range(24) for j in range(20))
    worst_64 = max(abs(Fraction(float(C64[i, j])) - ref[i][j]) / Fraction(float(G[i, j]))
                   for i in range(24) for j in range(20))
    assert worst_dd <= Fraction(2) ** -75
    assert worst_64 >= Fraction(2) ** -60          # FP64 cannot do better than about half an ulp
    assert np.array_equal(hi, C64) or np.max(np.abs(hi - C64) / G) <= 2.0 ** -52


# ------------------------------------------------------------------ structural invariants of the method
def test_transpose_symmetry_and_power_of_two_scaling_are_exact():
    """(A B)^T = B^T A^T holds bit for bit in the scheme: the slices of a row do not depend on which
    operand the row belongs to, the integer diagonal sums are symmetric under swapping the roles, and the
    FP64 order is per element. Likewise scaling rows of A and columns of B by powers of two only moves
    the exponents: the result is scaled exactly (no rounding changes), unlike a re-association in FP64."""
    A, B = wl.phi_pair(13, 11, 37, 2.0, seed=71)
    for s in (3, 8, 13):
        C = oracle.dgemm(A, B, s)
        Ct = oracle.dgemm(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T), s)
        assert np.array_equal(C.T.copy().view(np.uint64), Ct.view(np.uint64))
        ra = np.ldexp(1.0, (np.arange(13) % 7) - 3)
        cb = np.ldexp(1.0, (np.arange(11) % 5) - 2)
        Cs = oracle.dgemm(A * ra[:, None], B * cb[None, :], s)
        assert np.array_equal(Cs.view(np.uint64), (C * ra[:, None] * cb[None, :]).view(np.uint64))
