"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2306_11975_amd import ozimmu

HEADER = Path(__file__).resolve().parents[1] / "include" / "ozimmu.h"
PROBE_HEADER = HEADER.with_name("ozimmu_probe.h")


def declared_functions(header=HEADER):
    text = header.read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ozimmu_[a-z_0-9]+)\s*\(", text)))


def test_header_and_binding_agree_and_library_exports_everything():
    names = declared_functions()
    assert set(names) == set(ozimmu.EXPORTS)
    probes = declared_functions(PROBE_HEADER)
    assert set(probes) == set(ozimmu.PROBE_EXPORTS)
    L = ozimmu.lib()
    for name in names + probes:
        assert getattr(L, name) is not None


def test_status_strings():
    assert ozimmu.status_string(0) == "ok"
    seen = {ozimmu.status_string(c) for c in range(9)}
    assert len(seen) == 9
    assert ozimmu.status_string(99) == "unknown status"


def test_geometry_and_workspace_size():
    assert ozimmu.slice_geometry(1, 1) == (128, 32)
    assert ozimmu.slice_geometry(128, 32) == (128, 32)
    assert ozimmu.slice_geometry(129, 33) == (256, 64)
    assert ozimmu.slice_geometry(0, 0) == (0, 0)
    s, m, n, k = 8, 8192, 8192, 8192
    ws = ozimmu.workspace_bytes(m, n, k, s)
    # slices of A and B, exponents, column maxima and the counters of the splitters that count for the slice-count
    # check (2 operands x 2048 slots x 5 x 8 bytes): every integer sum stays in registers
    lower = s * m * k * 2
    assert lower <= ws <= lower + 4 * (m + n) + 8 * n + 2 * 2048 * 5 * 8 + 16 * 256
    # long k: a diagonal no longer fits one INT32 block, INT64 diagonal sums are kept in the workspace
    ws_wide = ozimmu.workspace_bytes(4096, 4096, 131072, 8)
    assert ws_wide >= 8 * 4096 * 131072 * 2 + 8 * 4096 * 4096 * 8
    assert ozimmu.workspace_bytes(64, 64, 64, 3, True) > ozimmu.workspace_bytes(64, 64, 64, 3, False)


def test_slice_offset_is_a_bijection_with_contiguous_fragments():
    import numpy as np

    rp, kp = ozimmu.slice_geometry(300, 200)   # 384 x 224
    assert (rp, kp) == (384, 224)
    offs = np.array([[ozimmu.slice_offset(rp, kp, 0, r, l) for l in range(kp)] for r in range(rp)])
    assert sorted(offs.reshape(-1).tolist()) == list(range(rp * kp))
    # a fragment of 32 rows x 32 positions is one contiguous 1 KiB run; a row's 32 positions are 32
    # contiguous bytes; 16 bytes stay together
    frag = offs[64:96, 32:64]
    assert frag.min() == (2 * (kp // 32) + 1) * 1024 and frag.max() == frag.min() + 1023
    assert all(frag[r].max() - frag[r].min() == 31 and frag[r].min() == frag.min() + 32 * r for r in range(32))
    assert (np.diff(offs[:, :16], axis=1) == 1).all()
    assert ozimmu.slice_offset(rp, kp, 2, 0, 0) == 2 * rp * kp
    assert ozimmu.slice_offset(rp, kp, 0, rp, 0) == -1 and ozimmu.slice_offset(rp, kp, 0, 0, kp) == -1
    # unpack_slices inverts it
    raw = np.zeros(2 * rp * kp, dtype=np.int8)
    raw[ozimmu.slice_offset(rp, kp, 1, 299, 199)] = 5
    un = ozimmu.unpack_slices(raw, 2, 300, 200)
    assert un[1, 299, 199] == 5 and np.count_nonzero(un) == 1


def test_argument_errors_are_reported_before_any_launch():
    L = ozimmu.lib()
    out = ctypes.c_size_t()
    assert L.ozimmu_workspace_bytes(-1, 1, 1, 3, 0, ctypes.byref(out)) == 1
    assert L.ozimmu_workspace_bytes(1, 1, 1, 0, 0, ctypes.byref(out)) == 3
    assert L.ozimmu_workspace_bytes(1, 1, 1, 17, 0, ctypes.byref(out)) == 3
    assert L.ozimmu_workspace_bytes(1, 1, 1, 3, 0, None) == 4
    fake = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    # negative dimension, bad slice count, small leading dimensions, null pointers, workspace
    assert L.ozimmu_dgemm(-1, 4, 4, fake, 4, fake, 4, fake, 4, 3, fake, 1 << 30, None) == 1
    assert L.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 0, fake, 1 << 30, None) == 3
    assert L.ozimmu_dgemm(4, 4, 4, fake, 3, fake, 4, fake, 4, 3, fake, 1 << 30, None) == 2
    assert L.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 3, fake, 4, 3, fake, 1 << 30, None) == 2
    assert L.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 3, 3, fake, 1 << 30, None) == 2
    assert L.ozimmu_dgemm(4, 4, 4, None, 4, fake, 4, fake, 4, 3, fake, 1 << 30, None) == 4
    assert L.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, None, 4, 3, fake, 1 << 30, None) == 4
    assert L.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 3, None, 1 << 30, None) == 5
    assert L.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 3, ctypes.c_void_p(264), 1 << 30, None) == 5
    assert L.ozimmu_dgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 3, fake, 16, None) == 5
    assert L.ozimmu_zgemm(4, 4, 4, fake, 4, fake, 4, fake, 4, 3, fake, 16, None) == 5
    # dimensions beyond OZIMMU_MAX_DIM (2^22) are refused
    assert L.ozimmu_dgemm((1 << 22) + 1, 4, 4, fake, 4, fake, 4, fake, 4, 3, fake, 1 << 30, None) == 1
    assert L.ozimmu_workspace_bytes(4, 4, (1 << 22) + 1, 3, 0, ctypes.byref(out)) == 1
    # empty products are no-ops
    assert L.ozimmu_dgemm(0, 4, 4, None, 4, None, 4, None, 4, 3, None, 0, None) == 0
    assert L.ozimmu_dgemm(4, 0, 4, None, 4, None, 0, None, 0, 3, None, 0, None) == 0
    # staged entry points
    assert L.ozimmu_split_rows(4, 4, fake, 3, 3, fake, fake, None) == 2
    assert L.ozimmu_split_rows(4, 4, fake, 4, 3, fake, None, None) == 4
    assert L.ozimmu_split_cols(4, 4, fake, 4, 3, fake, fake, None, None) == 4
    assert L.ozimmu_split_cols(4, 4, fake, 4, 3, fake, fake, ctypes.c_void_p(12), None) == 5
    assert L.ozimmu_slice_gemm(4, 4, 256, fake, fake, 0, 1, 0, 128, fake, 4, None) == 3
    assert L.ozimmu_slice_gemm(4, 4, 256, fake, fake, 1, 1, 48, 128, fake, 4, None) == 1   # k0 not aligned
    assert L.ozimmu_slice_gemm(4, 4, 256, fake, fake, 1, 1, 0, 100, fake, 4, None) == 1    # ragged inside
    assert L.ozimmu_slice_gemm(4, 4, 256, fake, fake, 1, 1, 128, 256, fake, 4, None) == 1  # beyond k
    assert L.ozimmu_slice_gemm(4, 4, 1 << 18, fake, fake, 1, 1, 0, (1 << 17) + 128, fake, 4, None) == 1
    assert L.ozimmu_slice_gemm(4, 4, 256, fake, fake, 1, 1, 0, 128, fake, 3, None) == 2
    assert L.ozimmu_dgemm_stage(3, 4, 4, 4, fake, 4, fake, 4, fake, 4, 3, fake, 1 << 30, None) == 1


def test_launch_plan_host_logic():
    # the headline shape: 64 x 128 tiles, 8192 workgroups = 32 full rounds of the 256 CUs, one band, no k-blocking
    assert ozimmu.launch_plan(8192, 8192, 8192, 8) == {"tile_rows": 64, "tile_cols": 128, "workgroups": 8192,
                                                       "bands": 1, "int32_block_steps": 0}
    assert ozimmu.launch_plan(8192, 8192, 8192, 10)["bands"] == 2
    assert ozimmu.launch_plan(100, 100, 100, 16) == {"tile_rows": 64, "tile_cols": 64, "workgroups": 4,
                                                     "bands": 2, "int32_block_steps": 0}
    # k-blocking starts where the longest diagonal (s pairs) exceeds 2^17 products: steps of 32 positions
    assert ozimmu.launch_plan(4096, 4096, 131072, 8)["int32_block_steps"] == 512
    assert ozimmu.launch_plan(64, 64, 16384, 8)["int32_block_steps"] == 0
    assert ozimmu.launch_plan(64, 64, 16385, 8)["int32_block_steps"] == 512
    for s in range(1, 17):
        steps = ozimmu.launch_plan(1, 1, 1 << 22, s)["int32_block_steps"]
        assert steps * 32 * s <= ozimmu.INT32_BLOCK < (steps + 1) * 32 * s
    L = ozimmu.lib()
    plan = ozimmu.Plan()
    assert L.ozimmu_launch_plan(-1, 1, 1, 3, ctypes.byref(plan)) == 1
    assert L.ozimmu_launch_plan(1, 1, 1, 0, ctypes.byref(plan)) == 3
    assert L.ozimmu_launch_plan(1, 1, 1, 3, None) == 4


def test_blas_call_argument_errors():
    L = ozimmu.lib()
    fake = ctypes.c_void_p(256)
    f = L.ozimmu_dgemm_blas
    ok = [b"N", b"N", 4, 5, 6, 1.0, fake, 4, fake, 6, 0.0, fake, 4, 3, fake, 1 << 30, None]
    def call(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return f(*a)
    assert call(_0=b"X") == 1 and call(_1=b"?") == 1 and call(_2=-1) == 1
    assert call(_13=0) == 3 and call(_13=17) == 3
    assert call(_7=3) == 2            # lda < m for 'N'
    assert call(_0=b"T", _7=5) == 2   # lda < k for 'T'
    assert call(_9=5) == 2            # ldb < k for 'N'
    assert call(_1=b"T", _9=4) == 2   # ldb < n for 'T'
    assert call(_12=3) == 2           # ldc < m
    assert call(_11=None) == 4 and call(_6=None) == 4
    assert call(_14=None) == 5 and call(_15=16) == 5
    assert call(_2=0) == 0            # empty result: no-op


def test_auto_slice_count_argument_errors():
    L = ozimmu.lib()
    out = ctypes.c_size_t()
    assert L.ozimmu_auto_scratch_bytes(1000, ctypes.byref(out)) == 0 and out.value == 512 + 2 * 8 * 1024
    assert L.ozimmu_auto_scratch_bytes(-1, ctypes.byref(out)) == 1
    fake = ctypes.c_void_p(256)
    s = ctypes.c_int(-7)
    args = lambda **kw: [kw.get("m", 4), 4, 4, fake, kw.get("lda", 4), fake, 4, 0, kw.get("T", 1.0), kw.get("smax", 16),
                         kw.get("scratch", fake), kw.get("sb", 1 << 20), kw.get("out", ctypes.byref(s)), None, None]
    assert L.ozimmu_auto_num_slices(*args(m=-1)) == 1
    assert L.ozimmu_auto_num_slices(*args(lda=3)) == 2
    assert L.ozimmu_auto_num_slices(*args(smax=0)) == 3
    assert L.ozimmu_auto_num_slices(*args(smax=17)) == 3
    assert L.ozimmu_auto_num_slices(*args(T=-0.5)) == 3
    assert L.ozimmu_auto_num_slices(*args(T=float("nan"))) == 3
    assert L.ozimmu_auto_num_slices(*args(out=None)) == 4
    assert L.ozimmu_auto_num_slices(*args(scratch=None)) == 5
    assert L.ozimmu_auto_num_slices(*args(sb=100)) == 5
    assert s.value == -7   # untouched on error


def test_binding_raises_typed_error():
    with pytest.raises(ozimmu.OzimmuError) as e:
        ozimmu.workspace_bytes(1, 1, 1, 0)
    assert e.value.code == 3


def test_interposer_exports_the_vendor_gemm_symbols_and_blas_argument_errors():
    """libozimmu_preload.so must define exactly the vendor entry points it stands in for (so the dynamic
    loader binds a program's calls to it); host-side argument checks of the complex BLAS-style call."""
    pre = Path(ozimmu.__file__).resolve().parent / "libozimmu_preload.so"
    if not pre.exists():
        pytest.skip("libozimmu_preload.so has not been built (python -m paper_2306_11975_amd.build)")
    P = ctypes.CDLL(str(pre))
    for name in ("rocblas_dgemm", "rocblas_zgemm", "rocblas_dgemm_64", "rocblas_zgemm_64", "hipblasDgemm",
                 "hipblasZgemm", "hipblasDgemm_64", "hipblasZgemm_64", "rocblas_dgemm_strided_batched",
                 "rocblas_zgemm_strided_batched", "hipblasDgemmStridedBatched", "hipblasZgemmStridedBatched",
                 "rocblas_gemm_ex", "hipblasGemmEx"):
        assert getattr(P, name) is not None

    L = ozimmu.lib()
    two = (ctypes.c_double * 2)(1.0, 0.0)
    al, junk = ctypes.addressof(two), 4096   # junk: a non-null pointer that no check dereferences

    def z(ta, tb, m, n, k, lda, ldb, ldc, s=4, alpha=al, beta=al, C=junk, ws=None, ws_bytes=0):
        return L.ozimmu_zgemm_blas(ta, tb, m, n, k, alpha, junk, lda, junk, ldb, beta, C, ldc, s, ws, ws_bytes, None)

    assert z(b"X", b"N", 4, 4, 4, 4, 4, 4) == ozimmu.ERR_BAD_DIM
    assert z(b"N", b"N", -1, 4, 4, 4, 4, 4) == ozimmu.ERR_BAD_DIM
    assert z(b"N", b"N", 4, 4, 4, 4, 4, 4, s=0) == ozimmu.ERR_BAD_SLICES
    assert z(b"N", b"N", 5, 4, 3, 4, 3, 5) == ozimmu.ERR_BAD_LD        # lda < m
    assert z(b"C", b"N", 5, 4, 3, 2, 3, 5) == ozimmu.ERR_BAD_LD        # lda < k for a transposed A
    assert z(b"N", b"T", 5, 4, 3, 5, 3, 5) == ozimmu.ERR_BAD_LD        # ldb < n for a transposed B
    assert z(b"N", b"N", 5, 4, 3, 5, 3, 4) == ozimmu.ERR_BAD_LD        # ldc < m
    assert z(b"N", b"N", 5, 4, 3, 5, 3, 5, alpha=None) == ozimmu.ERR_NULL
    assert z(b"N", b"N", 5, 4, 3, 5, 3, 5, C=None) == ozimmu.ERR_NULL
    assert z(b"N", b"N", 0, 4, 3, 1, 3, 1, C=None) == ozimmu.OK        # empty result: nothing to do
    assert z(b"N", b"N", 5, 4, 3, 5, 3, 5) == ozimmu.ERR_WORKSPACE     # product needed, no workspace
    with_c = ozimmu.zgemm_blas_workspace_bytes(300, 200, 100, 8, False)
    without = ozimmu.zgemm_blas_workspace_bytes(300, 200, 100, 8, True)
    assert with_c - without >= 16 * 300 * 200 and without >= ozimmu.workspace_bytes(200, 300, 100, 8, True)


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 with no C++ or HIP types in it."""
    import shutil
    import subprocess

    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", str(HEADER)],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
