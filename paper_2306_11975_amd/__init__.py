"""MI355X-native Ozaki-scheme DGEMM on the INT8 matrix cores (gfx950).

``workloads`` holds the seeded synthetic inputs; ``ozimmu`` is the thin binding over the
C-ABI library built from ``csrc/`` (it raises if the HIP library has not been built: there is
no CPU fallback).
"""
__all__ = ["workloads", "ozimmu"]
