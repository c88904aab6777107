// ozimmu_dgemm_static: ozimmu_dgemm for callers that can neither allocate device memory nor pass a
// workspace (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// The workspace of the product (slice tensors, exponents, column maxima, integer sums that leave the
// registers) lives in a file-scope device array of OZIMMU_STATIC_SCRATCH_BYTES; every GPU the library
// runs on holds its own copy of the array until the process ends.
#include <atomic>

#include "ozimmu_internal.h"

namespace {

static __device__ __align__(256) unsigned char scratch[OZIMMU_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
// Device address of `scratch` on each device. In host code the array's name is only a handle for
// hipGetSymbolAddress; the address it returns is what kernels and every other call get.
std::atomic<void*> scratch_ptr[kMaxDevices];

hipError_t scratch_address(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {   // first call on this device (it is the current one); racing threads get the same answer
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

}  // namespace

extern "C" ozimmu_status_t ozimmu_dgemm_static(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                               const double* B, int64_t ldb, double* C, int64_t ldc,
                                               int num_slices, void* stream) {
    size_t need = 0;
    ozimmu_status_t rc = ozimmu_workspace_bytes(m, n, k, num_slices, 0, &need);
    if (rc != OZIMMU_OK) return rc;
    if (m == 0 || n == 0) return OZIMMU_OK;
    if (k > 0 && need > (size_t)OZIMMU_STATIC_SCRATCH_BYTES) return OZIMMU_ERR_TOO_LARGE;
    void* ws = nullptr;
    if (k > 0 && scratch_address(&ws) != hipSuccess) return OZIMMU_ERR_HIP;
    // Every byte of the workspace that the product reads is written first by the same call (the
    // splitters write the padding of the slice tensors as zeros, the column maxima are cleared by a
    // fill kernel), so what an earlier call left behind is never seen.
    return ozimmu_dgemm(m, n, k, A, lda, B, ldb, C, ldc, num_slices, ws, OZIMMU_STATIC_SCRATCH_BYTES, stream);
}
