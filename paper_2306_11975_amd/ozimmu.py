"""Thin binding over the C ABI of libozimmu (include/ozimmu.h): argument marshalling only.

Every function has the name of the C entry point it calls; tensors are torch CUDA tensors used
purely as device memory, and the stream is torch's current HIP stream unless one is given.
There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

_LIB_PATH = Path(__file__).resolve().parent / "libozimmu.so"

(OK, ERR_BAD_DIM, ERR_BAD_LD, ERR_BAD_SLICES, ERR_NULL, ERR_WORKSPACE, ERR_HIP, ERR_NOT_IMPLEMENTED,
 ERR_TOO_LARGE) = range(9)
MAX_SLICES = 16
ROW_ALIGN = 128
K_ALIGN = 32
FRAG_ROWS = 32
INT32_BLOCK = 131072
WORKSPACE_ALIGN = 256
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = (
    "ozimmu_status_string", "ozimmu_slice_geometry", "ozimmu_slice_offset", "ozimmu_split_rows", "ozimmu_split_cols",
    "ozimmu_slice_gemm", "ozimmu_workspace_bytes", "ozimmu_dgemm", "ozimmu_zgemm", "ozimmu_dgemm_static", "ozimmu_dgemm_stage",
    "ozimmu_launch_plan", "ozimmu_dgemm_dd", "ozimmu_dgemm_blas", "ozimmu_zgemm_blas_workspace_bytes", "ozimmu_zgemm_blas",
    "ozimmu_auto_scratch_bytes", "ozimmu_auto_num_slices", "ozimmu_auto_num_slices_blas", "ozimmu_zgemm_auto",
    "ozimmu_dgemm_auto", "ozimmu_dgemm_blas_auto", "ozimmu_zgemm_blas_auto",
)
PROBE_EXPORTS = ("ozimmu_probe_int8_mfma",)      # include/ozimmu_probe.h: measurement utility, not the product path


class OzimmuError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"ozimmu error {code}: {what}")
        self.code = code


class Plan(ctypes.Structure):
    """ozimmu_plan_t of include/ozimmu.h."""
    _fields_ = [("tile_rows", ctypes.c_int), ("tile_cols", ctypes.c_int), ("workgroups", ctypes.c_int64),
                ("bands", ctypes.c_int), ("int32_block_steps", ctypes.c_int)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libozimmu.so (built by ``python -m paper_2306_11975_amd.build``)."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2306_11975_amd.build` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(str(_LIB_PATH))
        i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        L.ozimmu_status_string.restype = ctypes.c_char_p
        L.ozimmu_status_string.argtypes = [i32]
        L.ozimmu_slice_geometry.restype = i32
        L.ozimmu_slice_geometry.argtypes = [i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.ozimmu_slice_offset.restype = i64
        L.ozimmu_slice_offset.argtypes = [i64, i64, i32, i64, i64]
        L.ozimmu_split_rows.restype = i32
        L.ozimmu_split_rows.argtypes = [i64, i64, vp, i64, i32, vp, vp, vp]
        L.ozimmu_split_cols.restype = i32
        L.ozimmu_split_cols.argtypes = [i64, i64, vp, i64, i32, vp, vp, vp, vp]
        L.ozimmu_slice_gemm.restype = i32
        L.ozimmu_slice_gemm.argtypes = [i64, i64, i64, vp, vp, i32, i32, i64, i64, vp, i64, vp]
        L.ozimmu_workspace_bytes.restype = i32
        L.ozimmu_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, ctypes.POINTER(sz)]
        for name in ("ozimmu_dgemm", "ozimmu_zgemm"):
            f = getattr(L, name)
            f.restype = i32
            f.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp, sz, vp]
        L.ozimmu_dgemm_static.restype = i32
        L.ozimmu_dgemm_static.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp]
        L.ozimmu_dgemm_stage.restype = i32
        L.ozimmu_dgemm_stage.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp, sz, vp]
        L.ozimmu_launch_plan.restype = i32
        L.ozimmu_launch_plan.argtypes = [i64, i64, i64, i32, ctypes.POINTER(Plan)]
        L.ozimmu_dgemm_dd.restype = i32
        L.ozimmu_dgemm_dd.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, vp, i64, i32, vp, sz, vp]
        L.ozimmu_dgemm_blas.restype = i32
        L.ozimmu_dgemm_blas.argtypes = [ctypes.c_char, ctypes.c_char, i64, i64, i64, ctypes.c_double, vp, i64, vp, i64,
                                        ctypes.c_double, vp, i64, i32, vp, sz, vp]
        L.ozimmu_zgemm_blas_workspace_bytes.restype = i32
        L.ozimmu_zgemm_blas_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, ctypes.POINTER(sz)]
        L.ozimmu_zgemm_blas.restype = i32
        L.ozimmu_zgemm_blas.argtypes = [ctypes.c_char, ctypes.c_char, i64, i64, i64, vp, vp, i64, vp, i64, vp, vp, i64,
                                        i32, vp, sz, vp]
        L.ozimmu_auto_scratch_bytes.restype = i32
        L.ozimmu_auto_scratch_bytes.argtypes = [i64, ctypes.POINTER(sz)]
        L.ozimmu_auto_num_slices.restype = i32
        L.ozimmu_auto_num_slices.argtypes = [i64, i64, i64, vp, i64, vp, i64, i32, ctypes.c_double, i32, vp, sz,
                                             ctypes.POINTER(i32), vp, vp]
        L.ozimmu_auto_num_slices_blas.restype = i32
        L.ozimmu_auto_num_slices_blas.argtypes = [ctypes.c_char, ctypes.c_char, i64, i64, i64, vp, i64, vp, i64, i32,
                                                  ctypes.c_double, i32, vp, sz, ctypes.POINTER(i32), vp, vp]
        L.ozimmu_zgemm_auto.restype = i32
        L.ozimmu_zgemm_auto.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, ctypes.c_double, i32, i32, vp, sz, vp, sz,
                                        ctypes.POINTER(i32), ctypes.POINTER(i32), vp]
        L.ozimmu_dgemm_auto.restype = i32
        L.ozimmu_dgemm_auto.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, ctypes.c_double, i32, i32, vp, sz, vp, sz,
                                        ctypes.POINTER(i32), ctypes.POINTER(i32), vp]
        L.ozimmu_dgemm_blas_auto.restype = i32
        L.ozimmu_dgemm_blas_auto.argtypes = [ctypes.c_char, ctypes.c_char, i64, i64, i64, ctypes.c_double, vp, i64, vp, i64,
                                             ctypes.c_double, vp, i64, ctypes.c_double, i32, i32, vp, sz, vp, sz,
                                             ctypes.POINTER(i32), ctypes.POINTER(i32), vp]
        L.ozimmu_zgemm_blas_auto.restype = i32
        L.ozimmu_zgemm_blas_auto.argtypes = [ctypes.c_char, ctypes.c_char, i64, i64, i64, vp, vp, i64, vp, i64, vp, vp, i64,
                                             ctypes.c_double, i32, i32, vp, sz, vp, sz, ctypes.POINTER(i32),
                                             ctypes.POINTER(i32), vp]
        dp = ctypes.POINTER(ctypes.c_double)
        L.ozimmu_probe_int8_mfma.restype = i32
        L.ozimmu_probe_int8_mfma.argtypes = [i32, i32, i32, dp, dp]
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().ozimmu_status_string(int(code)).decode()


def _check(code: int) -> None:
    if code != OK:
        raise OzimmuError(code, status_string(code))


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _stream(stream) -> int:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _ld(t, cols):
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a 2-D row-major tensor (unit stride along the second dimension)")
    return t.stride(0) if t.shape[0] > 1 else max(cols, 1)


def slice_geometry(rows: int, k: int):
    rp, kp = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().ozimmu_slice_geometry(rows, k, ctypes.byref(rp), ctypes.byref(kp)))
    return rp.value, kp.value


def slice_offset(rows_padded: int, k_padded: int, slice_: int, row: int, l: int) -> int:
    return int(lib().ozimmu_slice_offset(rows_padded, k_padded, slice_, row, l))


def unpack_slices(raw, num_slices: int, rows: int, k: int):
    """Re-order the bytes of a slice tensor (as the library stores it, any 1-D or N-D int8 numpy
    array of num_slices * rows_padded * k_padded elements) into a plain [slice][row][l] numpy
    array of the padded shape. Pure index permutation: the block geometry is queried from the
    library through ozimmu_slice_offset, no arithmetic of the method happens here."""
    import numpy as np

    rp, kp = slice_geometry(rows, k)
    flat = np.ascontiguousarray(raw).reshape(-1)
    assert flat.size == num_slices * rp * kp
    if flat.size == 0:
        return flat.reshape(num_slices, rp, kp)
    # offsets are separable: offset(s, r, l) = s * rp * kp + f(r - r % 32, 0) + g(r % 32, l % 32) + h(0, l - l % 32)
    row_part = np.array([slice_offset(rp, kp, 0, r, 0) for r in range(0, rp, FRAG_ROWS)], dtype=np.int64)
    in_frag = np.array([[slice_offset(rp, kp, 0, rr, l) for l in range(K_ALIGN)] for rr in range(FRAG_ROWS)],
                       dtype=np.int64)                       # [32][32], fragment 0
    slab_part = np.array([slice_offset(rp, kp, 0, 0, l) for l in range(0, kp, K_ALIGN)], dtype=np.int64)
    idx = (row_part[:, None, None, None] + in_frag[None, :, None, :] + slab_part[None, None, :, None])
    idx = idx.reshape(rp, kp)                                # [row][l]
    out = np.empty((num_slices, rp, kp), dtype=flat.dtype)
    for s_ in range(num_slices):
        out[s_] = flat[s_ * rp * kp + idx]
    return out


def workspace_bytes(m: int, n: int, k: int, num_slices: int, is_complex: bool = False) -> int:
    out = ctypes.c_size_t()
    _check(lib().ozimmu_workspace_bytes(m, n, k, num_slices, int(is_complex), ctypes.byref(out)))
    return out.value


def split_rows(A, num_slices: int, slices, exps, stream=None) -> None:
    """A: (m, k) float64 device tensor with unit column stride; slices: int8 device buffer of
    num_slices * rows_padded * k_padded bytes; exps: int32 device tensor of m entries."""
    m, k = A.shape
    _check(lib().ozimmu_split_rows(m, k, _ptr(A), _ld(A, k), num_slices,
                                   _ptr(slices), _ptr(exps), _stream(stream)))


def split_cols(B, num_slices: int, slices, exps, col_scratch, stream=None) -> None:
    k, n = B.shape
    _check(lib().ozimmu_split_cols(k, n, _ptr(B), _ld(B, n), num_slices,
                                   _ptr(slices), _ptr(exps), _ptr(col_scratch), _stream(stream)))


def slice_gemm(m: int, n: int, k: int, SA, SB, p: int, q: int, k0: int, klen: int, P, stream=None) -> None:
    _check(lib().ozimmu_slice_gemm(m, n, k, _ptr(SA), _ptr(SB), p, q, k0, klen, _ptr(P),
                                   _ld(P, n), _stream(stream)))


def dgemm(A, B, C, num_slices: int, workspace, stream=None) -> None:
    """C = A . B by the Ozaki scheme on the INT8 matrix cores (A: m x k, B: k x n, C: m x n,
    float64 device tensors with unit column stride; workspace: uint8 device tensor)."""
    m, k = A.shape
    n = B.shape[1]
    _check(lib().ozimmu_dgemm(m, n, k, _ptr(A), _ld(A, k), _ptr(B), _ld(B, n), _ptr(C), _ld(C, n), num_slices,
                              _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))


def dgemm_static(A, B, C, num_slices: int, stream=None) -> None:
    """ozimmu_dgemm without a workspace argument: the library's built-in scratch is used (see ozimmu.h)."""
    m, k = A.shape
    n = B.shape[1]
    _check(lib().ozimmu_dgemm_static(m, n, k, _ptr(A), _ld(A, k), _ptr(B), _ld(B, n), _ptr(C), _ld(C, n),
                                     num_slices, _stream(stream)))


def dgemm_stage(stage: int, A, B, C, num_slices: int, workspace, stream=None) -> None:
    m, k = A.shape
    n = B.shape[1]
    _check(lib().ozimmu_dgemm_stage(stage, m, n, k, _ptr(A), _ld(A, k), _ptr(B), _ld(B, n), _ptr(C), _ld(C, n),
                                    num_slices, _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                    _stream(stream)))


def zgemm(A, B, C, num_slices: int, workspace, stream=None) -> None:
    """Complex128 device tensors (interleaved re, im), otherwise as dgemm."""
    m, k = A.shape
    n = B.shape[1]
    _check(lib().ozimmu_zgemm(m, n, k, _ptr(A), _ld(A, k), _ptr(B), _ld(B, n), _ptr(C), _ld(C, n), num_slices,
                              _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))


def launch_plan(m: int, n: int, k: int, num_slices: int) -> dict:
    """How ozimmu_dgemm runs a shape (ozimmu_plan_t as a dict; see ozimmu.h)."""
    plan = Plan()
    _check(lib().ozimmu_launch_plan(m, n, k, num_slices, ctypes.byref(plan)))
    return {name: getattr(plan, name) for name, _ in Plan._fields_}


def dgemm_dd(A, B, C_hi, C_lo, num_slices: int, workspace, stream=None) -> None:
    """C_hi + C_lo = A . B with the diagonal sums added in double-double (see ozimmu.h)."""
    m, k = A.shape
    n = B.shape[1]
    ldc = _ld(C_hi, n)
    if _ld(C_lo, n) != ldc:
        raise ValueError("C_hi and C_lo must have the same leading dimension")
    _check(lib().ozimmu_dgemm_dd(m, n, k, _ptr(A), _ld(A, k), _ptr(B), _ld(B, n), _ptr(C_hi), _ptr(C_lo), ldc,
                                 num_slices, _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                 _stream(stream)))


def dgemm_blas(transa: str, transb: str, m: int, n: int, k: int, alpha: float, A, lda: int, B, ldb: int,
               beta: float, C, ldc: int, num_slices: int, workspace, stream=None) -> None:
    """Column-major C = alpha op(A) op(B) + beta C; A, B, C are device tensors used as raw
    column-major storage with the given leading dimensions (see ozimmu.h)."""
    _check(lib().ozimmu_dgemm_blas(transa.encode()[:1], transb.encode()[:1], m, n, k, float(alpha), _ptr(A), lda,
                                   _ptr(B), ldb, float(beta), _ptr(C), ldc, num_slices, _ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream(stream)))


def zgemm_blas_workspace_bytes(m: int, n: int, k: int, num_slices: int, beta_is_zero: bool) -> int:
    out = ctypes.c_size_t()
    _check(lib().ozimmu_zgemm_blas_workspace_bytes(m, n, k, num_slices, int(bool(beta_is_zero)), ctypes.byref(out)))
    return out.value


def zgemm_blas(transa: str, transb: str, m: int, n: int, k: int, alpha: complex, A, lda: int, B, ldb: int,
               beta: complex, C, ldc: int, num_slices: int, workspace, stream=None) -> None:
    """Column-major complex C = alpha op(A) op(B) + beta C; A, B, C are complex128 device tensors used as
    raw column-major storage with the given leading dimensions in complex elements (see ozimmu.h)."""
    al = (ctypes.c_double * 2)(complex(alpha).real, complex(alpha).imag)
    be = (ctypes.c_double * 2)(complex(beta).real, complex(beta).imag)
    _check(lib().ozimmu_zgemm_blas(transa.encode()[:1], transb.encode()[:1], m, n, k, ctypes.addressof(al), _ptr(A), lda,
                                   _ptr(B), ldb, ctypes.addressof(be), _ptr(C), ldc, num_slices, _ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream(stream)))


def auto_scratch_bytes(n: int) -> int:
    out = ctypes.c_size_t()
    _check(lib().ozimmu_auto_scratch_bytes(n, ctypes.byref(out)))
    return out.value


def auto_num_slices(A, B, threshold: float, max_slices: int = MAX_SLICES, scratch=None, stream=None):
    """Number of slices whose average mantissa loss is within `threshold` (see ozimmu.h) for the
    float64 or complex128 device tensors A (m x k) and B (k x n). Returns (s, sums) with sums a
    numpy uint64 array [planes][16]. Waits for the stream."""
    import numpy as np
    import torch

    m, k = A.shape
    n = B.shape[1]
    cplx = A.is_complex()
    assert cplx == B.is_complex()
    if scratch is None:
        scratch = torch.empty(max(auto_scratch_bytes(n), WORKSPACE_ALIGN), dtype=torch.uint8, device=A.device)
    planes = 4 if cplx else 2
    sums = np.zeros((planes, MAX_SLICES), dtype=np.uint64)
    s = ctypes.c_int()
    _check(lib().ozimmu_auto_num_slices(m, n, k, _ptr(A), _ld(A, k), _ptr(B), _ld(B, n), int(cplx), float(threshold),
                                        int(max_slices), _ptr(scratch), scratch.numel(), ctypes.byref(s),
                                        sums.ctypes.data, _stream(stream)))
    return s.value, sums


def _gemm_auto(cplx, A, B, C, threshold, guess, max_slices, workspace, scratch, stream):
    import torch

    m, k = A.shape
    n = B.shape[1]
    if workspace is None:
        need = max(workspace_bytes(m, n, k, s, cplx) for s in range(1, max_slices + 1))
        workspace = torch.empty(max(need, WORKSPACE_ALIGN), dtype=torch.uint8, device=A.device)
    if scratch is None:
        scratch = torch.empty(max(auto_scratch_bytes(n), WORKSPACE_ALIGN), dtype=torch.uint8, device=A.device)
    s, confirmed = ctypes.c_int(), ctypes.c_int()
    f = lib().ozimmu_zgemm_auto if cplx else lib().ozimmu_dgemm_auto
    _check(f(m, n, k, _ptr(A), _ld(A, k), _ptr(B), _ld(B, n), _ptr(C), _ld(C, n), float(threshold), int(max_slices),
             int(guess), _ptr(workspace), workspace.numel(), _ptr(scratch), scratch.numel(), ctypes.byref(s),
             ctypes.byref(confirmed), _stream(stream)))
    return s.value, bool(confirmed.value)


def dgemm_auto(A, B, C, threshold: float, guess: int = 0, max_slices: int = MAX_SLICES, workspace=None, scratch=None,
               stream=None):
    """C = A . B (float64 device tensors) with the slice count ozimmu_auto_num_slices would choose, in one call (see
    ozimmu.h); `guess` is the expected count (0: none). Returns (s, guess_confirmed). Waits for the stream."""
    return _gemm_auto(False, A, B, C, threshold, guess, max_slices, workspace, scratch, stream)


def zgemm_auto(A, B, C, threshold: float, guess: int = 0, max_slices: int = MAX_SLICES, workspace=None, scratch=None,
               stream=None):
    """The same for complex128 device tensors."""
    return _gemm_auto(True, A, B, C, threshold, guess, max_slices, workspace, scratch, stream)


def gemm_blas_auto(transa: str, transb: str, m: int, n: int, k: int, alpha, A, lda: int, B, ldb: int, beta, C, ldc: int,
                   is_complex: bool, threshold: float, guess: int = 0, max_slices: int = MAX_SLICES, stream=None):
    """The BLAS-style call with the slice count chosen inside it (see ozimmu.h); A, B, C are device tensors used as raw
    column-major storage. Returns (s, guess_confirmed). Waits for the stream."""
    import torch

    beta_zero = complex(beta) == 0
    if is_complex:
        need = max(zgemm_blas_workspace_bytes(m, n, k, s, beta_zero) for s in range(1, max_slices + 1))
    else:
        need = max(workspace_bytes(n, m, k, s) for s in range(1, max_slices + 1))
    workspace = torch.empty(max(need, WORKSPACE_ALIGN), dtype=torch.uint8, device=C.device)
    scratch = torch.empty(max(auto_scratch_bytes(max(m, n)), WORKSPACE_ALIGN), dtype=torch.uint8, device=C.device)
    s, confirmed = ctypes.c_int(), ctypes.c_int()
    common = (float(threshold), int(max_slices), int(guess), _ptr(workspace), workspace.numel(), _ptr(scratch),
              scratch.numel(), ctypes.byref(s), ctypes.byref(confirmed), _stream(stream))
    if is_complex:
        al = (ctypes.c_double * 2)(complex(alpha).real, complex(alpha).imag)
        be = (ctypes.c_double * 2)(complex(beta).real, complex(beta).imag)
        _check(lib().ozimmu_zgemm_blas_auto(transa.encode()[:1], transb.encode()[:1], m, n, k, ctypes.addressof(al), _ptr(A),
                                            lda, _ptr(B), ldb, ctypes.addressof(be), _ptr(C), ldc, *common))
    else:
        _check(lib().ozimmu_dgemm_blas_auto(transa.encode()[:1], transb.encode()[:1], m, n, k, float(alpha), _ptr(A), lda,
                                            _ptr(B), ldb, float(beta), _ptr(C), ldc, *common))
    return s.value, bool(confirmed.value)


def auto_num_slices_blas(transa: str, transb: str, m: int, n: int, k: int, A, lda: int, B, ldb: int, is_complex: bool,
                         threshold: float, max_slices: int = MAX_SLICES, scratch=None, stream=None):
    """The same choice for column-major operands with transposes (see ozimmu.h); A and B are device
    tensors used as raw storage. Returns (s, sums). Waits for the stream."""
    import numpy as np
    import torch

    if scratch is None:
        scratch = torch.empty(max(auto_scratch_bytes(max(m, n)), WORKSPACE_ALIGN), dtype=torch.uint8, device=A.device)
    planes = 4 if is_complex else 2
    sums = np.zeros((planes, MAX_SLICES), dtype=np.uint64)
    s = ctypes.c_int()
    _check(lib().ozimmu_auto_num_slices_blas(transa.encode()[:1], transb.encode()[:1], m, n, k, _ptr(A), lda, _ptr(B), ldb,
                                             int(bool(is_complex)), float(threshold), int(max_slices), _ptr(scratch),
                                             scratch.numel(), ctypes.byref(s), sums.ctypes.data, _stream(stream)))
    return s.value, sums


def probe_int8_mfma(pattern: int, shape: int = 0, iters: int = 200000):
    """(10^12 INT8 ops/s, shader MHz) of a register-only MFMA issue loop; see ozimmu_probe.h."""
    tops, mhz = ctypes.c_double(), ctypes.c_double()
    _check(lib().ozimmu_probe_int8_mfma(pattern, shape, iters, ctypes.byref(tops), ctypes.byref(mhz)))
    return tops.value, mhz.value


def alloc_workspace(m: int, n: int, k: int, num_slices: int, is_complex: bool = False, device="cuda"):
    """Convenience for callers that use torch for device memory: a uint8 tensor of the right size
    (torch's caching allocator returns 512-byte aligned blocks)."""
    import torch

    nbytes = max(workspace_bytes(m, n, k, num_slices, is_complex), WORKSPACE_ALIGN)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    assert ws.data_ptr() % WORKSPACE_ALIGN == 0
    return ws
