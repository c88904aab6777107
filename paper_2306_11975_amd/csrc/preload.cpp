// libozimmu_preload.so: stands in for the vendor's double-precision GEMM entry points
// (Section 4.4, third extension: the vendor DGEMM/ZGEMM calls of an unmodified program are
// intercepted through the dynamic loader's preload list and computed by the Ozaki scheme with an
// automatically chosen number of slices).
//
//   LD_PRELOAD=/path/to/libozimmu_preload.so  program ...
//
// Intercepted: rocblas_dgemm, rocblas_zgemm, hipblasDgemm, hipblasZgemm, their _64 forms, their
// strided-batched forms (computed member by member) and the all-FP64 in-place case of rocblas_gemm_ex /
// hipblasGemmEx. A call
// is computed here when the handle is in host pointer mode (alpha and beta readable on the host) and
// the library accepts the arguments; every other call, and every call in vendor mode, goes on to the
// vendor's routine (found behind this library in the global scope, or in the loaded vendor library
// if the host keeps it in a local scope), which then also reports argument errors.
//
// Environment (read once, at the first intercepted call):
//   OZIMMU_MODE       "auto" (default): slice count chosen per call from the operands;
//                     "1" .. "16": that many slices; "vendor": pass everything through.
//   OZIMMU_THRESHOLD  admitted average mantissa loss in bits for "auto" (default 0: lossless split).
//   OZIMMU_MIN_WORK   calls with m*n*k below this go to the vendor (default 0: none do).
//   OZIMMU_VERBOSE    "1": one line per intercepted call on stderr.
//
// Unlike libozimmu itself this layer owns device memory: one workspace per device, grown on demand
// with hipMalloc (after a device synchronisation when an older, smaller one is replaced) and kept
// until the process ends. Calls are serialised by a lock while they are enqueued, and a call on a
// different stream than the previous one first waits (on the device) for that one's work, so the
// shared workspace is never used by two products at once. In "auto" mode each call waits for its
// stream once (the slice count comes back to the host).
#include <dlfcn.h>
#include <link.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include <hip/hip_runtime.h>
#include <hipblas/hipblas.h>
#include <rocblas/rocblas.h>

#include "ozimmu.h"

namespace {

struct Config {
    int slices = 0;          // 0: automatic; > 0: fixed; -1: vendor
    double threshold = 0.0;
    double min_work = 0.0;
    bool verbose = false;
};

const Config& config() {
    static Config cfg;
    static std::once_flag once;
    std::call_once(once, [] {
        if (const char* v = std::getenv("OZIMMU_MODE")) {
            if (!std::strcmp(v, "vendor")) cfg.slices = -1;
            else if (!std::strcmp(v, "auto") || !*v) cfg.slices = 0;
            else {
                char* end = nullptr;
                const long s = std::strtol(v, &end, 10);
                if (*end == 0 && s >= 1 && s <= OZIMMU_MAX_SLICES) cfg.slices = (int)s;
                else {
                    std::fprintf(stderr, "[ozimmu] OZIMMU_MODE=%s not understood (auto, vendor, 1..%d): using auto\n", v,
                                 OZIMMU_MAX_SLICES);
                }
            }
        }
        if (const char* v = std::getenv("OZIMMU_THRESHOLD")) {
            const double t = std::atof(v);
            if (t >= 0.0) cfg.threshold = t;
        }
        if (const char* v = std::getenv("OZIMMU_MIN_WORK")) cfg.min_work = std::atof(v);
        if (const char* v = std::getenv("OZIMMU_VERBOSE")) cfg.verbose = std::atoi(v) != 0;
    });
    return cfg;
}

// A symbol of the vendor library this interposer stands in front of. A program linked against the
// vendor library has it in the global scope behind this one (RTLD_NEXT finds it); a host that loaded
// it into a local scope (a Python extension module, a plugin) has not, so the loaded objects are
// searched for the library by name and the symbol is taken from that object. nullptr if absent.
struct FindObject {
    const char* part;
    void* handle;
};
int find_object(struct dl_phdr_info* info, size_t, void* data) {
    FindObject* f = static_cast<FindObject*>(data);
    if (info->dlpi_name && std::strstr(info->dlpi_name, f->part) && !std::strstr(info->dlpi_name, "ozimmu")) {
        f->handle = dlopen(info->dlpi_name, RTLD_NOLOAD | RTLD_LAZY);   // already loaded: only a handle to it
        return f->handle != nullptr;
    }
    return 0;
}
void* vendor_symbol(const char* library_part, const char* name) {
    if (void* f = dlsym(RTLD_NEXT, name)) return f;
    FindObject probe{library_part, nullptr};
    dl_iterate_phdr(find_object, &probe);
    return probe.handle ? dlsym(probe.handle, name) : nullptr;
}
template <class F>
F vendor(const char* library_part, const char* name) {
    F f = reinterpret_cast<F>(vendor_symbol(library_part, name));
    if (!f) std::fprintf(stderr, "[ozimmu] %s: no vendor library with this symbol is loaded\n", name);
    return f;
}

// ---- per-device workspace -------------------------------------------------------------------
constexpr int kMaxDevices = 64;
struct DeviceState {
    void* buffer = nullptr;
    size_t bytes = 0;
    hipEvent_t done = nullptr;
    hipStream_t last_stream = nullptr;
    bool used = false;
    int last_auto_slices[2] = {0, 0};   // what the last automatic choice of a plain product came to (real, complex): the next guess
};
DeviceState g_state[kMaxDevices];
std::mutex g_lock;

size_t align_up(size_t x) { return (x + OZIMMU_WORKSPACE_ALIGN - 1) / OZIMMU_WORKSPACE_ALIGN * OZIMMU_WORKSPACE_ALIGN; }

// At least `bytes` of device memory on the current device; earlier contents are not kept.
void* reserve(DeviceState& d, size_t bytes) {
    if (d.bytes >= bytes) return d.buffer;
    if (d.buffer) {
        if (hipDeviceSynchronize() != hipSuccess) return nullptr;
        (void)hipFree(d.buffer);
        d.buffer = nullptr;
        d.bytes = 0;
    }
    const size_t want = align_up(bytes + bytes / 8);
    if (hipMalloc(&d.buffer, want) != hipSuccess) {
        (void)hipGetLastError();
        d.buffer = nullptr;
        return nullptr;
    }
    d.bytes = want;
    return d.buffer;
}

struct Call {
    const char* name;
    bool cplx;
    char ta, tb;
    int64_t m, n, k;
    const double* alpha;   // host: 1 or 2 doubles
    const double* A;
    int64_t lda;
    const double* B;
    int64_t ldb;
    const double* beta;
    double* C;
    int64_t ldc;
};

// Computes the call with the Ozaki scheme; false if it has to go to the vendor instead.
bool compute(const Call& c, hipStream_t stream) {
    const Config& cfg = config();
    if (cfg.slices < 0 || !c.alpha || !c.beta) return false;
    if (c.m <= 0 || c.n <= 0 || c.k < 0) return false;   // empty or invalid: nothing to gain
    if ((double)c.m * (double)c.n * (double)c.k < cfg.min_work) return false;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;

    std::lock_guard<std::mutex> guard(g_lock);
    DeviceState& d = g_state[dev];
    if (!d.done && hipEventCreateWithFlags(&d.done, hipEventDisableTiming) != hipSuccess) return false;
    if (d.used && d.last_stream != stream && hipStreamWaitEvent(stream, d.done, 0) != hipSuccess) return false;

    const bool alpha_zero = c.alpha[0] == 0.0 && (!c.cplx || c.alpha[1] == 0.0);
    const bool beta_zero = c.beta[0] == 0.0 && (!c.cplx || c.beta[1] == 0.0);
    const bool product = c.k > 0 && !alpha_zero;
    int s = cfg.slices > 0 ? cfg.slices : 1;
    size_t scan_bytes = 0;
    // A product that overwrites C (beta 0) in automatic mode: count and product in one call, the count of the previous
    // such call as the guess; the splitters then count while they split (a small complex gate on a wide state is
    // formed in one pass over the state) and no operand is read just for the choice.
    if (product && cfg.slices == 0 && beta_zero) {
        size_t ws_bytes = 0;
        bool sized = ozimmu_auto_scratch_bytes(std::max(c.m, c.n), &scan_bytes) == OZIMMU_OK;
        scan_bytes = align_up(scan_bytes);
        for (int t = 1; sized && t <= OZIMMU_MAX_SLICES; ++t) {
            size_t need = 0;
            sized = (c.cplx ? ozimmu_zgemm_blas_workspace_bytes(c.m, c.n, c.k, t, 1, &need)
                            : ozimmu_workspace_bytes(c.n, c.m, c.k, t, 0, &need)) == OZIMMU_OK;
            ws_bytes = std::max(ws_bytes, need);
        }
        // the workspace of the largest slice count may not be available: then the two calls below, sized for the count chosen
        unsigned char* buf = sized ? static_cast<unsigned char*>(reserve(d, scan_bytes + ws_bytes)) : nullptr;
        int confirmed = 0;
        int& last = d.last_auto_slices[c.cplx ? 1 : 0];
        if (buf) {
            const ozimmu_status_t rc =
                c.cplx ? ozimmu_zgemm_blas_auto(c.ta, c.tb, c.m, c.n, c.k, c.alpha, c.A, c.lda, c.B, c.ldb, c.beta, c.C, c.ldc,
                                                cfg.threshold, OZIMMU_MAX_SLICES, last, buf + scan_bytes, ws_bytes, buf,
                                                scan_bytes, &s, &confirmed, stream)
                       : ozimmu_dgemm_blas_auto(c.ta, c.tb, c.m, c.n, c.k, c.alpha[0], c.A, c.lda, c.B, c.ldb, c.beta[0], c.C,
                                                c.ldc, cfg.threshold, OZIMMU_MAX_SLICES, last, buf + scan_bytes, ws_bytes,
                                                buf, scan_bytes, &s, &confirmed, stream);
            if (rc != OZIMMU_OK) return false;   // beta is 0: whatever C holds now, the vendor routine overwrites it
            last = s;
            d.used = true;
            d.last_stream = stream;
            (void)hipEventRecord(d.done, stream);
            if (cfg.verbose)
                std::fprintf(stderr, "[ozimmu] %s %c%c m=%lld n=%lld k=%lld slices=%d (auto) [one call%s]\n", c.name, c.ta,
                             c.tb, (long long)c.m, (long long)c.n, (long long)c.k, s, confirmed ? ", guess confirmed" : "");
            return true;
        }
    }
    if (product && cfg.slices == 0) {
        if (ozimmu_auto_scratch_bytes(std::max(c.m, c.n), &scan_bytes) != OZIMMU_OK) return false;
        scan_bytes = align_up(scan_bytes);
        void* scratch = reserve(d, scan_bytes);
        if (!scratch) return false;
        if (ozimmu_auto_num_slices_blas(c.ta, c.tb, c.m, c.n, c.k, c.A, c.lda, c.B, c.ldb, c.cplx, cfg.threshold,
                                        OZIMMU_MAX_SLICES, scratch, scan_bytes, &s, nullptr, stream) != OZIMMU_OK)
            return false;
    }
    size_t ws_bytes = 0;
    void* ws = nullptr;
    if (product) {
        const ozimmu_status_t rc = c.cplx ? ozimmu_zgemm_blas_workspace_bytes(c.m, c.n, c.k, s, beta_zero, &ws_bytes)
                                          : ozimmu_workspace_bytes(c.n, c.m, c.k, s, 0, &ws_bytes);
        if (rc != OZIMMU_OK) return false;
        ws = reserve(d, ws_bytes);
        if (!ws) return false;
    }
    ozimmu_status_t rc;
    if (c.cplx)
        rc = ozimmu_zgemm_blas(c.ta, c.tb, c.m, c.n, c.k, c.alpha, c.A, c.lda, c.B, c.ldb, c.beta, c.C, c.ldc, s, ws,
                               ws_bytes, stream);
    else
        rc = ozimmu_dgemm_blas(c.ta, c.tb, c.m, c.n, c.k, c.alpha[0], c.A, c.lda, c.B, c.ldb, c.beta[0], c.C, c.ldc, s, ws,
                               ws_bytes, stream);
    if (rc != OZIMMU_OK) return false;   // nothing has been written to C: the vendor routine redoes the call
    d.used = true;
    d.last_stream = stream;
    (void)hipEventRecord(d.done, stream);
    if (cfg.verbose)
        std::fprintf(stderr, "[ozimmu] %s %c%c m=%lld n=%lld k=%lld slices=%d%s\n", c.name, c.ta, c.tb, (long long)c.m,
                     (long long)c.n, (long long)c.k, s, cfg.slices == 0 && product ? " (auto)" : "");
    return true;
}

void note_passthrough(const char* name) {
    if (config().verbose) std::fprintf(stderr, "[ozimmu] %s -> vendor\n", name);
}

char op_letter(int op) { return op == 111 ? 'N' : op == 112 ? 'T' : op == 113 ? 'C' : '?'; }   // the BLAS operation codes both libraries use

// ---- rocBLAS ----------------------------------------------------------------------------------
bool rocblas_context(rocblas_handle handle, hipStream_t* stream) {
    using get_stream_t = rocblas_status (*)(rocblas_handle, hipStream_t*);
    using get_mode_t = rocblas_status (*)(rocblas_handle, rocblas_pointer_mode*);
    static const get_stream_t get_stream = reinterpret_cast<get_stream_t>(vendor_symbol("librocblas.so", "rocblas_get_stream"));
    static const get_mode_t get_mode = reinterpret_cast<get_mode_t>(vendor_symbol("librocblas.so", "rocblas_get_pointer_mode"));
    rocblas_pointer_mode mode;
    return handle && get_stream && get_mode && get_mode(handle, &mode) == rocblas_status_success &&
           mode == rocblas_pointer_mode_host && get_stream(handle, stream) == rocblas_status_success;
}

template <class Int, class T, class F>
rocblas_status rocblas_entry(const char* name, bool cplx, rocblas_handle handle, rocblas_operation ta, rocblas_operation tb,
                             Int m, Int n, Int k, const T* alpha, const T* A, Int lda, const T* B, Int ldb, const T* beta,
                             T* C, Int ldc) {
    hipStream_t stream = nullptr;
    if (config().slices >= 0 && rocblas_context(handle, &stream)) {
        const Call c{name, cplx, op_letter((int)ta), op_letter((int)tb), (int64_t)m, (int64_t)n, (int64_t)k,
                     reinterpret_cast<const double*>(alpha), reinterpret_cast<const double*>(A), (int64_t)lda,
                     reinterpret_cast<const double*>(B), (int64_t)ldb, reinterpret_cast<const double*>(beta),
                     reinterpret_cast<double*>(C), (int64_t)ldc};
        if (compute(c, stream)) return rocblas_status_success;
    }
    note_passthrough(name);
    static const F next = vendor<F>("librocblas.so", name);
    if (!next) return rocblas_status_internal_error;
    return next(handle, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc);
}

// ---- hipBLAS ----------------------------------------------------------------------------------
bool hipblas_context(hipblasHandle_t handle, hipStream_t* stream) {
    using get_stream_t = hipblasStatus_t (*)(hipblasHandle_t, hipStream_t*);
    using get_mode_t = hipblasStatus_t (*)(hipblasHandle_t, hipblasPointerMode_t*);
    static const get_stream_t get_stream = reinterpret_cast<get_stream_t>(vendor_symbol("libhipblas.so", "hipblasGetStream"));
    static const get_mode_t get_mode = reinterpret_cast<get_mode_t>(vendor_symbol("libhipblas.so", "hipblasGetPointerMode"));
    hipblasPointerMode_t mode;
    return handle && get_stream && get_mode && get_mode(handle, &mode) == HIPBLAS_STATUS_SUCCESS &&
           mode == HIPBLAS_POINTER_MODE_HOST && get_stream(handle, stream) == HIPBLAS_STATUS_SUCCESS;
}

template <class Int, class T, class F>
hipblasStatus_t hipblas_entry(const char* name, bool cplx, hipblasHandle_t handle, hipblasOperation_t ta,
                              hipblasOperation_t tb, Int m, Int n, Int k, const T* alpha, const T* A, Int lda, const T* B,
                              Int ldb, const T* beta, T* C, Int ldc) {
    hipStream_t stream = nullptr;
    if (config().slices >= 0 && hipblas_context(handle, &stream)) {
        const Call c{name, cplx, op_letter((int)ta), op_letter((int)tb), (int64_t)m, (int64_t)n, (int64_t)k,
                     reinterpret_cast<const double*>(alpha), reinterpret_cast<const double*>(A), (int64_t)lda,
                     reinterpret_cast<const double*>(B), (int64_t)ldb, reinterpret_cast<const double*>(beta),
                     reinterpret_cast<double*>(C), (int64_t)ldc};
        if (compute(c, stream)) return HIPBLAS_STATUS_SUCCESS;
    }
    note_passthrough(name);
    static const F next = vendor<F>("libhipblas.so", name);
    if (!next) return HIPBLAS_STATUS_INTERNAL_ERROR;
    return next(handle, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc);
}

// Strided-batched forms: the members are computed one after the other with the same workspace. If a
// member cannot be computed the whole call goes to the vendor; that is only safe while C is unchanged,
// i.e. at the first member or with beta == 0 (C is then overwritten anyway).
template <class Stride>
int compute_batched(Call c, hipStream_t stream, Stride sa, Stride sb, Stride sc, int64_t batch) {   // 1 done, 0 vendor, -1 error
    if (batch <= 0) return 0;
    const int w = c.cplx ? 2 : 1;
    const bool beta_zero = c.beta && c.beta[0] == 0.0 && (!c.cplx || c.beta[1] == 0.0);
    const double *A0 = c.A, *B0 = c.B;
    double* C0 = c.C;
    for (int64_t i = 0; i < batch; ++i) {
        c.A = A0 + (int64_t)sa * i * w;
        c.B = B0 + (int64_t)sb * i * w;
        c.C = C0 + (int64_t)sc * i * w;
        if (!compute(c, stream)) return (i == 0 || beta_zero) ? 0 : -1;
    }
    return 1;
}

template <class Int, class Stride, class T, class F>
rocblas_status rocblas_batched_entry(const char* name, bool cplx, rocblas_handle handle, rocblas_operation ta,
                                     rocblas_operation tb, Int m, Int n, Int k, const T* alpha, const T* A, Int lda,
                                     Stride sa, const T* B, Int ldb, Stride sb, const T* beta, T* C, Int ldc, Stride sc,
                                     Int batch) {
    hipStream_t stream = nullptr;
    if (config().slices >= 0 && rocblas_context(handle, &stream)) {
        const Call c{name, cplx, op_letter((int)ta), op_letter((int)tb), (int64_t)m, (int64_t)n, (int64_t)k,
                     reinterpret_cast<const double*>(alpha), reinterpret_cast<const double*>(A), (int64_t)lda,
                     reinterpret_cast<const double*>(B), (int64_t)ldb, reinterpret_cast<const double*>(beta),
                     reinterpret_cast<double*>(C), (int64_t)ldc};
        const int rc = compute_batched(c, stream, sa, sb, sc, (int64_t)batch);
        if (rc > 0) return rocblas_status_success;
        if (rc < 0) return rocblas_status_internal_error;
    }
    note_passthrough(name);
    static const F next = vendor<F>("librocblas.so", name);
    if (!next) return rocblas_status_internal_error;
    return next(handle, ta, tb, m, n, k, alpha, A, lda, sa, B, ldb, sb, beta, C, ldc, sc, batch);
}

template <class Int, class Stride, class T, class F>
hipblasStatus_t hipblas_batched_entry(const char* name, bool cplx, hipblasHandle_t handle, hipblasOperation_t ta,
                                      hipblasOperation_t tb, Int m, Int n, Int k, const T* alpha, const T* A, Int lda,
                                      Stride sa, const T* B, Int ldb, Stride sb, const T* beta, T* C, Int ldc, Stride sc,
                                      Int batch) {
    hipStream_t stream = nullptr;
    if (config().slices >= 0 && hipblas_context(handle, &stream)) {
        const Call c{name, cplx, op_letter((int)ta), op_letter((int)tb), (int64_t)m, (int64_t)n, (int64_t)k,
                     reinterpret_cast<const double*>(alpha), reinterpret_cast<const double*>(A), (int64_t)lda,
                     reinterpret_cast<const double*>(B), (int64_t)ldb, reinterpret_cast<const double*>(beta),
                     reinterpret_cast<double*>(C), (int64_t)ldc};
        const int rc = compute_batched(c, stream, sa, sb, sc, (int64_t)batch);
        if (rc > 0) return HIPBLAS_STATUS_SUCCESS;
        if (rc < 0) return HIPBLAS_STATUS_INTERNAL_ERROR;
    }
    note_passthrough(name);
    static const F next = vendor<F>("libhipblas.so", name);
    if (!next) return HIPBLAS_STATUS_INTERNAL_ERROR;
    return next(handle, ta, tb, m, n, k, alpha, A, lda, sa, B, ldb, sb, beta, C, ldc, sc, batch);
}

}  // namespace

extern "C" {

rocblas_status rocblas_dgemm(rocblas_handle handle, rocblas_operation transA, rocblas_operation transB, rocblas_int m,
                             rocblas_int n, rocblas_int k, const double* alpha, const double* A, rocblas_int lda,
                             const double* B, rocblas_int ldb, const double* beta, double* C, rocblas_int ldc) {
    return rocblas_entry<rocblas_int, double, decltype(&rocblas_dgemm)>("rocblas_dgemm", false, handle, transA, transB, m, n,
                                                                        k, alpha, A, lda, B, ldb, beta, C, ldc);
}

rocblas_status rocblas_dgemm_64(rocblas_handle handle, rocblas_operation transA, rocblas_operation transB, int64_t m,
                                int64_t n, int64_t k, const double* alpha, const double* A, int64_t lda, const double* B,
                                int64_t ldb, const double* beta, double* C, int64_t ldc) {
    return rocblas_entry<int64_t, double, decltype(&rocblas_dgemm_64)>("rocblas_dgemm_64", false, handle, transA, transB, m,
                                                                       n, k, alpha, A, lda, B, ldb, beta, C, ldc);
}

rocblas_status rocblas_zgemm(rocblas_handle handle, rocblas_operation transA, rocblas_operation transB, rocblas_int m,
                             rocblas_int n, rocblas_int k, const rocblas_double_complex* alpha,
                             const rocblas_double_complex* A, rocblas_int lda, const rocblas_double_complex* B,
                             rocblas_int ldb, const rocblas_double_complex* beta, rocblas_double_complex* C,
                             rocblas_int ldc) {
    return rocblas_entry<rocblas_int, rocblas_double_complex, decltype(&rocblas_zgemm)>(
        "rocblas_zgemm", true, handle, transA, transB, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc);
}

rocblas_status rocblas_zgemm_64(rocblas_handle handle, rocblas_operation transA, rocblas_operation transB, int64_t m,
                                int64_t n, int64_t k, const rocblas_double_complex* alpha, const rocblas_double_complex* A,
                                int64_t lda, const rocblas_double_complex* B, int64_t ldb,
                                const rocblas_double_complex* beta, rocblas_double_complex* C, int64_t ldc) {
    return rocblas_entry<int64_t, rocblas_double_complex, decltype(&rocblas_zgemm_64)>(
        "rocblas_zgemm_64", true, handle, transA, transB, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc);
}

hipblasStatus_t hipblasDgemm(hipblasHandle_t handle, hipblasOperation_t transA, hipblasOperation_t transB, int m, int n,
                             int k, const double* alpha, const double* AP, int lda, const double* BP, int ldb,
                             const double* beta, double* CP, int ldc) {
    return hipblas_entry<int, double, decltype(&hipblasDgemm)>("hipblasDgemm", false, handle, transA, transB, m, n, k, alpha,
                                                               AP, lda, BP, ldb, beta, CP, ldc);
}

hipblasStatus_t hipblasDgemm_64(hipblasHandle_t handle, hipblasOperation_t transA, hipblasOperation_t transB, int64_t m,
                                int64_t n, int64_t k, const double* alpha, const double* AP, int64_t lda, const double* BP,
                                int64_t ldb, const double* beta, double* CP, int64_t ldc) {
    return hipblas_entry<int64_t, double, decltype(&hipblasDgemm_64)>("hipblasDgemm_64", false, handle, transA, transB, m, n,
                                                                      k, alpha, AP, lda, BP, ldb, beta, CP, ldc);
}

hipblasStatus_t hipblasZgemm(hipblasHandle_t handle, hipblasOperation_t transA, hipblasOperation_t transB, int m, int n,
                             int k, const hipDoubleComplex* alpha, const hipDoubleComplex* AP, int lda,
                             const hipDoubleComplex* BP, int ldb, const hipDoubleComplex* beta, hipDoubleComplex* CP,
                             int ldc) {
    return hipblas_entry<int, hipDoubleComplex, decltype(&hipblasZgemm)>("hipblasZgemm", true, handle, transA, transB, m, n,
                                                                         k, alpha, AP, lda, BP, ldb, beta, CP, ldc);
}

hipblasStatus_t hipblasZgemm_64(hipblasHandle_t handle, hipblasOperation_t transA, hipblasOperation_t transB, int64_t m,
                                int64_t n, int64_t k, const hipDoubleComplex* alpha, const hipDoubleComplex* AP,
                                int64_t lda, const hipDoubleComplex* BP, int64_t ldb, const hipDoubleComplex* beta,
                                hipDoubleComplex* CP, int64_t ldc) {
    return hipblas_entry<int64_t, hipDoubleComplex, decltype(&hipblasZgemm_64)>(
        "hipblasZgemm_64", true, handle, transA, transB, m, n, k, alpha, AP, lda, BP, ldb, beta, CP, ldc);
}

rocblas_status rocblas_dgemm_strided_batched(rocblas_handle handle, rocblas_operation transA, rocblas_operation transB,
                                             rocblas_int m, rocblas_int n, rocblas_int k, const double* alpha,
                                             const double* A, rocblas_int lda, rocblas_stride stride_a, const double* B,
                                             rocblas_int ldb, rocblas_stride stride_b, const double* beta, double* C,
                                             rocblas_int ldc, rocblas_stride stride_c, rocblas_int batch_count) {
    return rocblas_batched_entry<rocblas_int, rocblas_stride, double, decltype(&rocblas_dgemm_strided_batched)>(
        "rocblas_dgemm_strided_batched", false, handle, transA, transB, m, n, k, alpha, A, lda, stride_a, B, ldb, stride_b,
        beta, C, ldc, stride_c, batch_count);
}

rocblas_status rocblas_zgemm_strided_batched(rocblas_handle handle, rocblas_operation transA, rocblas_operation transB,
                                             rocblas_int m, rocblas_int n, rocblas_int k,
                                             const rocblas_double_complex* alpha, const rocblas_double_complex* A,
                                             rocblas_int lda, rocblas_stride stride_a, const rocblas_double_complex* B,
                                             rocblas_int ldb, rocblas_stride stride_b, const rocblas_double_complex* beta,
                                             rocblas_double_complex* C, rocblas_int ldc, rocblas_stride stride_c,
                                             rocblas_int batch_count) {
    return rocblas_batched_entry<rocblas_int, rocblas_stride, rocblas_double_complex,
                                 decltype(&rocblas_zgemm_strided_batched)>(
        "rocblas_zgemm_strided_batched", true, handle, transA, transB, m, n, k, alpha, A, lda, stride_a, B, ldb, stride_b,
        beta, C, ldc, stride_c, batch_count);
}

hipblasStatus_t hipblasDgemmStridedBatched(hipblasHandle_t handle, hipblasOperation_t transA, hipblasOperation_t transB,
                                           int m, int n, int k, const double* alpha, const double* AP, int lda,
                                           long long strideA, const double* BP, int ldb, long long strideB,
                                           const double* beta, double* CP, int ldc, long long strideC, int batchCount) {
    return hipblas_batched_entry<int, long long, double, decltype(&hipblasDgemmStridedBatched)>(
        "hipblasDgemmStridedBatched", false, handle, transA, transB, m, n, k, alpha, AP, lda, strideA, BP, ldb, strideB,
        beta, CP, ldc, strideC, batchCount);
}

hipblasStatus_t hipblasZgemmStridedBatched(hipblasHandle_t handle, hipblasOperation_t transA, hipblasOperation_t transB,
                                           int m, int n, int k, const hipDoubleComplex* alpha, const hipDoubleComplex* AP,
                                           int lda, long long strideA, const hipDoubleComplex* BP, int ldb,
                                           long long strideB, const hipDoubleComplex* beta, hipDoubleComplex* CP, int ldc,
                                           long long strideC, int batchCount) {
    return hipblas_batched_entry<int, long long, hipDoubleComplex, decltype(&hipblasZgemmStridedBatched)>(
        "hipblasZgemmStridedBatched", true, handle, transA, transB, m, n, k, alpha, AP, lda, strideA, BP, ldb, strideB,
        beta, CP, ldc, strideC, batchCount);
}

rocblas_status rocblas_gemm_ex(rocblas_handle handle, rocblas_operation transA, rocblas_operation transB, rocblas_int m,
                               rocblas_int n, rocblas_int k, const void* alpha, const void* a, rocblas_datatype a_type,
                               rocblas_int lda, const void* b, rocblas_datatype b_type, rocblas_int ldb, const void* beta,
                               const void* c, rocblas_datatype c_type, rocblas_int ldc, void* d, rocblas_datatype d_type,
                               rocblas_int ldd, rocblas_datatype compute_type, rocblas_gemm_algo algo,
                               int32_t solution_index, uint32_t flags) {
    // only the all-FP64 (real or complex) in-place form is a DGEMM / ZGEMM; everything else is the vendor's
    const bool f64 = a_type == b_type && a_type == c_type && a_type == d_type && a_type == compute_type &&
                     (a_type == rocblas_datatype_f64_r || a_type == rocblas_datatype_f64_c) && c == d && ldc == ldd;
    hipStream_t stream = nullptr;
    if (f64 && config().slices >= 0 && rocblas_context(handle, &stream)) {
        const Call call{"rocblas_gemm_ex", a_type == rocblas_datatype_f64_c, op_letter((int)transA), op_letter((int)transB),
                        (int64_t)m, (int64_t)n, (int64_t)k, static_cast<const double*>(alpha), static_cast<const double*>(a),
                        (int64_t)lda, static_cast<const double*>(b), (int64_t)ldb, static_cast<const double*>(beta),
                        static_cast<double*>(d), (int64_t)ldd};
        if (compute(call, stream)) return rocblas_status_success;
    }
    note_passthrough("rocblas_gemm_ex");
    static const auto next = vendor<decltype(&rocblas_gemm_ex)>("librocblas.so", "rocblas_gemm_ex");
    if (!next) return rocblas_status_internal_error;
    return next(handle, transA, transB, m, n, k, alpha, a, a_type, lda, b, b_type, ldb, beta, c, c_type, ldc, d, d_type, ldd,
                compute_type, algo, solution_index, flags);
}

hipblasStatus_t hipblasGemmEx(hipblasHandle_t handle, hipblasOperation_t transA, hipblasOperation_t transB, int m, int n,
                              int k, const void* alpha, const void* A, hipDataType aType, int lda, const void* B,
                              hipDataType bType, int ldb, const void* beta, void* C, hipDataType cType, int ldc,
                              hipblasComputeType_t computeType, hipblasGemmAlgo_t algo) {
    const bool f64 = aType == bType && aType == cType && (aType == HIP_R_64F || aType == HIP_C_64F) &&
                     computeType == HIPBLAS_COMPUTE_64F;
    hipStream_t stream = nullptr;
    if (f64 && config().slices >= 0 && hipblas_context(handle, &stream)) {
        const Call call{"hipblasGemmEx", aType == HIP_C_64F, op_letter((int)transA), op_letter((int)transB), (int64_t)m,
                        (int64_t)n, (int64_t)k, static_cast<const double*>(alpha), static_cast<const double*>(A), (int64_t)lda,
                        static_cast<const double*>(B), (int64_t)ldb, static_cast<const double*>(beta),
                        static_cast<double*>(C), (int64_t)ldc};
        if (compute(call, stream)) return HIPBLAS_STATUS_SUCCESS;
    }
    note_passthrough("hipblasGemmEx");
    static const auto next = vendor<decltype(&hipblasGemmEx)>("libhipblas.so", "hipblasGemmEx");
    if (!next) return HIPBLAS_STATUS_INTERNAL_ERROR;
    return next(handle, transA, transB, m, n, k, alpha, A, aType, lda, B, bType, ldb, beta, C, cType, ldc, computeType, algo);
}

}  // extern "C"
