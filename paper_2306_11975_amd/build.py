"""Build libozimmu.so (HIP, gfx950) in-tree with hipcc. Run: python -m paper_2306_11975_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
OBJ = PKG / "_build"
LIB = PKG / "libozimmu.so"
EXAMPLE = PKG / "example_dgemm"       # stand-alone C++ user of the C ABI (csrc/example_dgemm.cpp)
PRELOAD = PKG / "libozimmu_preload.so"  # interposer for the vendor DGEMM/ZGEMM symbols (csrc/preload.cpp)
BLAS_CLIENT = PKG / "blas_client"     # plain rocBLAS/hipBLAS program the interposer is tried on (csrc/blas_client.cpp)

SOURCES = ["split.hip", "gemm.hip", "gemm_real.hip", "gemm_dd.hip", "gemm_complex.hip", "gate.hip", "probes.hip", "static_scratch.hip", "api.cpp"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Wall", f"-I{INCLUDE}", f"-I{CSRC}"]
# device code: gfx950 only; packed-FP32 instruction selection is switched off on the test machines
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


# translation units whose kernels write M0 in inline assembly (the LDS base of the direct loads)
USES_M0 = ("gemm_real.hip", "gemm_dd.hip", "gemm_complex.hip")


def _check_m0(src: str) -> None:
    """The direct global->LDS loads set M0 inside inline assembly, and the compiler does not accept M0 in
    a clobber list (reserved register). So the generated device assembly is checked instead: apart from
    those writes no instruction of these kernels may name M0."""
    import re

    stem = src.rsplit(".", 1)[0]
    listings = [p for p in OBJ.glob(f"{stem}-hip-amdgcn-amd-amdhsa-gfx950*.s")]
    if not listings:
        raise RuntimeError(f"no device assembly listing found for {src} in {OBJ}")
    ours = re.compile(r"^\s*s_mov_b32\s+m0,\s*(s\d+|vcc_lo|vcc_hi)\s*$")
    for listing in listings:
        for n, line in enumerate(listing.read_text().splitlines(), 1):
            code = line.split(";", 1)[0]
            if re.search(r"\bm0\b", code) and not ours.match(code):
                raise RuntimeError(f"{listing.name}:{n}: M0 is used outside the direct-load sequence: {line.strip()}")


def _compile(src: str) -> Path:
    obj = OBJ / (src + ".o")
    cmd = [hipcc(), *COMMON]
    if src.endswith(".hip"):
        cmd += DEVICE
    if src in USES_M0:
        cmd += ["-save-temps=obj"]       # leaves the device assembly next to the object
    cmd += ["-c", str(CSRC / src), "-o", str(obj)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    if src in USES_M0:
        _check_m0(src)
    return obj


def build(verbose: bool = True) -> Path:
    """Compile every translation unit and link the shared library (always recompiles)."""
    OBJ.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *map(str, objs), "-o", str(tmp)]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    # the stand-alone example links against the library it was just built next to
    tmp_ex = EXAMPLE.with_suffix(f".tmp{os.getpid()}")
    subprocess.run([hipcc(), "-O2", "-std=c++17", f"-I{INCLUDE}", str(CSRC / "example_dgemm.cpp"), f"-L{PKG}", "-lozimmu",
                    "-Wl,-rpath,$ORIGIN", "-o", str(tmp_ex)], check=True)
    os.replace(tmp_ex, EXAMPLE)
    # the interposer needs libozimmu and the HIP runtime only: the vendor BLAS is whatever the host program loads
    tmp_pre = PRELOAD.with_suffix(f".tmp{os.getpid()}.so")
    subprocess.run([hipcc(), *COMMON, "-shared", str(CSRC / "preload.cpp"), f"-L{PKG}", "-lozimmu", "-ldl",
                    "-Wl,-rpath,$ORIGIN", "-o", str(tmp_pre)], check=True)
    os.replace(tmp_pre, PRELOAD)
    tmp_cl = BLAS_CLIENT.with_suffix(f".tmp{os.getpid()}")
    subprocess.run([hipcc(), "-O2", "-std=c++17", str(CSRC / "blas_client.cpp"), "-lrocblas", "-lhipblas",
                    "-o", str(tmp_cl)], check=True)
    os.replace(tmp_cl, BLAS_CLIENT)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
