"""CPU oracle for the Ozaki-scheme DGEMM on an INT8 integer matrix unit.

TEST INFRASTRUCTURE ONLY: only the tests, the smoke check and the CPU-baseline leg of the
benchmark may import this package. It compiles ``ozaki_oracle.c`` with gcc (no GPU code,
nothing shared with the HIP library) and exposes thin numpy wrappers; all arithmetic of the
method lives in the C file, which cites the passages of the paper it follows.

Pins (see tests/test_oracle_*.py): closed forms of Section 3.2, exact reconstruction and
truncation bounds of the slices, brute force on raw bit patterns with Python integers,
exact-rational products on tiny inputs, the INT32 overflow bound, and the integer-matrix
special case in which the result must equal a plain integer matrix product.
The automatic slice count (Section 4.4) is pinned by a bit-position brute force on raw
patterns, the single-binade closed form, exact reconstruction at threshold 0 and monotonicity.
Unpinned: the paper's error curves and its Table 3 figures, and the slice counts its
automatic mode picked for its circuits (plots and circuit configurations are not available
in text form) -- parity unpinned for those.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "ozaki_oracle.c"
_LIB = _HERE / "_build" / "libozaki_oracle.so"

W = 7  # magnitude bits per slice (Table 2: INT8-INT32 input mantissa length)


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc; returns the path of the shared object."""
    if not force and _LIB.exists() and _LIB.stat().st_mtime >= _SRC.stat().st_mtime:
        return _LIB
    _LIB.parent.mkdir(exist_ok=True)
    tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
    cmd = ["gcc", "-std=c99", "-O2", "-ftree-vectorize", "-ffp-contract=off", "-fno-fast-math",
           "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-Wno-maybe-uninitialized", str(_SRC), "-o", str(tmp), "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(str(build()))
        i64, i32, dbl, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        lib.oz_oracle_threads.restype = i32
        lib.oz_alpha.restype = i32
        lib.oz_alpha.argtypes = [i32, dbl]
        lib.oz_bps.restype = i32
        lib.oz_bps.argtypes = [i32, i32, dbl]
        lib.oz_num_pairs.restype = i32
        lib.oz_num_pairs.argtypes = [i32]
        lib.oz_split_rows.restype = None
        lib.oz_split_rows.argtypes = [i64, i64, vp, i64, i32, vp, vp]
        lib.oz_split_cols.restype = None
        lib.oz_split_cols.argtypes = [i64, i64, vp, i64, i32, vp, vp]
        lib.oz_pair_product.restype = None
        lib.oz_pair_product.argtypes = [i64, i64, i64, vp, vp, i64, i64, vp]
        lib.oz_diagonal_sums.restype = None
        lib.oz_diagonal_sums.argtypes = [i64, i64, i64, i32, vp, vp, vp]
        lib.oz_accumulate.restype = None
        lib.oz_accumulate.argtypes = [i64, i64, i32, vp, vp, vp, vp, i64]
        for name in ("oz_dgemm", "oz_dgemm_pairwise_order", "oz_zgemm"):
            f = getattr(lib, name)
            f.restype = i32
            f.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, i32]
        lib.oz_dd_gemm.restype = None
        lib.oz_dd_gemm.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, vp]
        lib.oz_auto_loss_sums.restype = None
        lib.oz_auto_loss_sums.argtypes = [i64, i64, vp, i64, i64, i32, i32, vp]
        lib.oz_auto_num_slices.restype = i32
        lib.oz_auto_num_slices.argtypes = [i32, i32, vp, vp, dbl]
        lib.oz_accumulate_dd.restype = None
        lib.oz_accumulate_dd.argtypes = [i64, i64, i32, vp, vp, vp, vp, vp, i64]
        lib.oz_dgemm_dd.restype = i32
        lib.oz_dgemm_dd.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, vp, i64, i32]
        lib.oz_dgemm_blas.restype = i32
        lib.oz_dgemm_blas.argtypes = [i32, i32, i64, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, i32]
        lib.oz_zgemm_blas.restype = i32
        lib.oz_zgemm_blas.argtypes = [i32, i32, i64, i64, i64, vp, vp, i64, vp, i64, vp, vp, i64, i32]
        lib.oz_abs_gemm.restype = None
        lib.oz_abs_gemm.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp]
        _lib = lib
    return _lib


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def _f64(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if not np.all(np.isfinite(a)):
        raise ValueError("oracle inputs must be finite")
    return a


def threads() -> int:
    return int(_load().oz_oracle_threads())


def alpha(l_acc: int, k: float) -> int:
    """Eq. (4)."""
    return int(_load().oz_alpha(int(l_acc), float(k)))


def bps(l_in: int, l_acc: int, k: float) -> int:
    """Eq. (5)."""
    return int(_load().oz_bps(int(l_in), int(l_acc), float(k)))


def num_pairs(s: int) -> int:
    return int(_load().oz_num_pairs(int(s)))


def split_rows(A, s: int):
    """SplitInt on the rows of A (m x k): returns (EA[m] int32, SA[s][m][k] int8)."""
    A = _f64(A)
    m, k = A.shape
    E = np.zeros(m, dtype=np.int32)
    S = np.zeros((s, m, k), dtype=np.int8)
    _load().oz_split_rows(m, k, _p(A), k, s, _p(E), _p(S))
    return E, S


def split_cols(B, s: int):
    """SplitInt on M = B^T for B (k x n): returns (EB[n] int32, SB[s][n][k] int8)."""
    B = _f64(B)
    k, n = B.shape
    E = np.zeros(n, dtype=np.int32)
    S = np.zeros((s, n, k), dtype=np.int8)
    _load().oz_split_cols(k, n, _p(B), n, s, _p(E), _p(S))
    return E, S


def pair_product(SAp, SBq, k0: int = 0, klen: int | None = None) -> np.ndarray:
    """Exact INT64 product of one slice pair over the k-range [k0, k0+klen)."""
    SAp = np.ascontiguousarray(SAp, dtype=np.int8)
    SBq = np.ascontiguousarray(SBq, dtype=np.int8)
    m, k = SAp.shape
    n, k2 = SBq.shape
    assert k == k2
    if klen is None:
        klen = k - k0
    assert 0 <= k0 and k0 + klen <= k
    P = np.zeros((m, n), dtype=np.int64)
    _load().oz_pair_product(m, n, k, _p(SAp), _p(SBq), k0, klen, _p(P))
    return P


def diagonal_sums(SA, SB) -> np.ndarray:
    """S[d-2] = sum over p+q=d of A^(p).B^(q), INT64, for d = 2..s+1."""
    SA = np.ascontiguousarray(SA, dtype=np.int8)
    SB = np.ascontiguousarray(SB, dtype=np.int8)
    s, m, k = SA.shape
    s2, n, k2 = SB.shape
    assert s == s2 and k == k2
    S = np.zeros((s, m, n), dtype=np.int64)
    _load().oz_diagonal_sums(m, n, k, s, _p(SA), _p(SB), _p(S))
    return S


def accumulate(S, EA, EB) -> np.ndarray:
    """Fixed-order FP64 sum of the scaled diagonal sums (summing-up step of the IMMU algorithm)."""
    S = np.ascontiguousarray(S, dtype=np.int64)
    EA = np.ascontiguousarray(EA, dtype=np.int32)
    EB = np.ascontiguousarray(EB, dtype=np.int32)
    s, m, n = S.shape
    C = np.zeros((m, n), dtype=np.float64)
    _load().oz_accumulate(m, n, s, _p(S), _p(EA), _p(EB), _p(C), n)
    return C


def _gemm(name, A, B, s, complex_=False):
    if complex_:
        A = np.ascontiguousarray(A, dtype=np.complex128)
        B = np.ascontiguousarray(B, dtype=np.complex128)
        if not (np.all(np.isfinite(A)) and np.all(np.isfinite(B))):
            raise ValueError("oracle inputs must be finite")
        C = np.zeros((A.shape[0], B.shape[1]), dtype=np.complex128)
    else:
        A, B = _f64(A), _f64(B)
        C = np.zeros((A.shape[0], B.shape[1]), dtype=np.float64)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    rc = getattr(_load(), name)(m, n, k, _p(A), k, _p(B), n, _p(C), n, int(s))
    if rc != 0:
        raise MemoryError("oracle could not allocate its slices")
    return C


def dgemm(A, B, s: int) -> np.ndarray:
    """The method end to end (split, integer products, fixed-order FP64 sum)."""
    return _gemm("oz_dgemm", A, B, s)


def dgemm_pairwise_order(A, B, s: int) -> np.ndarray:
    """Cross-check: literal pair-by-pair FP64 accumulation order of the IMMU algorithm."""
    return _gemm("oz_dgemm_pairwise_order", A, B, s)


def zgemm(A, B, s: int) -> np.ndarray:
    """Complex product as four real Ozaki products (Section 4.4)."""
    return _gemm("oz_zgemm", A, B, s, complex_=True)


def dd_gemm(A, B):
    """Double-double reference product: returns (hi, lo)."""
    A, B = _f64(A), _f64(B)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    hi = np.zeros((m, n), dtype=np.float64)
    lo = np.zeros((m, n), dtype=np.float64)
    _load().oz_dd_gemm(m, n, k, _p(A), k, _p(B), n, _p(hi), _p(lo))
    return hi, lo


def abs_gemm(A, B) -> np.ndarray:
    """(|A||B|) in FP64, the denominator of the scaled error."""
    A, B = _f64(A), _f64(B)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    G = np.zeros((m, n), dtype=np.float64)
    _load().oz_abs_gemm(m, n, k, _p(A), k, _p(B), n, _p(G))
    return G


def auto_loss_sums(M, by_columns: bool, s_max: int = 16) -> np.ndarray:
    """Section 4.4 (INT8-AUTO): sum over the elements of the real matrix M of the mantissa bits
    lost with s = 1 .. s_max slices, exponents per row (A) or per column (B). uint64[s_max]."""
    M = _f64(M)
    rows, cols = M.shape
    out = np.zeros(s_max, dtype=np.uint64)
    _load().oz_auto_loss_sums(rows, cols, _p(M), cols, 1, int(bool(by_columns)), s_max, _p(out))
    return out


def auto_num_slices(A, B, T: float, s_max: int = 16):
    """Section 4.4 (INT8-AUTO): the smallest number of slices whose average mantissa loss is <= T
    for every input plane. A (m x k) and B (k x n) real or complex. Returns (s, sums[planes][s_max])."""
    A = np.asarray(A)
    B = np.asarray(B)
    planes = []
    for M, by_cols in ((A, False), (B, True)):
        if np.iscomplexobj(M):
            planes += [(np.ascontiguousarray(M.real), by_cols), (np.ascontiguousarray(M.imag), by_cols)]
        else:
            planes.append((M, by_cols))
    sums = np.stack([auto_loss_sums(M, bc, s_max) for M, bc in planes])
    counts = np.array([M.size for M, _ in planes], dtype=np.int64)
    s = int(_load().oz_auto_num_slices(len(planes), s_max, _p(np.ascontiguousarray(sums)), _p(counts), float(T)))
    return s, sums


def dgemm_blas(transa: bool, transb: bool, alpha: float, A, B, beta: float, C, s: int) -> np.ndarray:
    """BLAS-style call: returns alpha op(A) op(B) + beta C for 2-D arrays given as mathematical
    matrices (A is m x k, or k x m if transa; B likewise; C is m x n). They are handed to the C
    routine in column-major storage."""
    Af = np.asfortranarray(np.asarray(A, dtype=np.float64))
    Bf = np.asfortranarray(np.asarray(B, dtype=np.float64))
    Cf = np.array(C, dtype=np.float64, order="F", copy=True)
    m, n = Cf.shape
    k = Af.shape[0] if transa else Af.shape[1]
    rc = _load().oz_dgemm_blas(int(transa), int(transb), m, n, k, float(alpha), _p(Af), max(Af.shape[0], 1), _p(Bf),
                               max(Bf.shape[0], 1), float(beta), _p(Cf), max(m, 1), int(s))
    if rc:
        raise MemoryError
    return Cf


def zgemm_blas(transa: str, transb: str, alpha: complex, A, B, beta: complex, C, s: int) -> np.ndarray:
    """Complex BLAS-style call: returns alpha op(A) op(B) + beta C; transa / transb are 'N', 'T' or 'C'
    (conjugate transpose). A, B, C are 2-D complex arrays as stored (A is m x k for 'N', k x m otherwise;
    B likewise; C is m x n). They are handed to the C routine in column-major storage."""
    code = {"N": 0, "T": 1, "C": 2}
    ta, tb = code[transa.upper()], code[transb.upper()]
    Af = np.asfortranarray(np.asarray(A, dtype=np.complex128))
    Bf = np.asfortranarray(np.asarray(B, dtype=np.complex128))
    Cf = np.array(C, dtype=np.complex128, order="F", copy=True)
    m, n = Cf.shape
    k = Af.shape[0] if ta else Af.shape[1]
    al = np.array([complex(alpha).real, complex(alpha).imag], dtype=np.float64)
    be = np.array([complex(beta).real, complex(beta).imag], dtype=np.float64)
    rc = _load().oz_zgemm_blas(ta, tb, m, n, k, _p(al), _p(Af), max(Af.shape[0], 1), _p(Bf), max(Bf.shape[0], 1),
                               _p(be), _p(Cf), max(m, 1), int(s))
    if rc:
        raise MemoryError
    return Cf


def accumulate_dd(S, EA, EB):
    """Double-double summing-up of the scaled diagonal sums: returns (hi, lo)."""
    S = np.ascontiguousarray(S, dtype=np.int64)
    EA = np.ascontiguousarray(EA, dtype=np.int32)
    EB = np.ascontiguousarray(EB, dtype=np.int32)
    s, m, n = S.shape
    hi = np.zeros((m, n), dtype=np.float64)
    lo = np.zeros((m, n), dtype=np.float64)
    _load().oz_accumulate_dd(m, n, s, _p(S), _p(EA), _p(EB), _p(hi), _p(lo), n)
    return hi, lo


def dgemm_dd(A, B, s: int):
    """The Ozaki product with the double-double summing-up: returns (hi, lo), C = hi + lo."""
    A = _f64(A)
    B = _f64(B)
    m, k = A.shape
    n = B.shape[1]
    hi = np.zeros((m, n), dtype=np.float64)
    lo = np.zeros((m, n), dtype=np.float64)
    if _load().oz_dgemm_dd(m, n, k, _p(A), max(k, 1), _p(B), max(n, 1), _p(hi), _p(lo), max(n, 1), int(s)):
        raise MemoryError
    return hi, lo
