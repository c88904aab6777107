// A plain user of the vendor BLAS that knows nothing about ozimmu: reads one GEMM problem from a
// file, runs it through rocblas_{d,z}gemm, hipblas{D,Z}gemm or the gemm_ex forms on a stream of its own and writes C
// back. It exists to show (and test) that preloading libozimmu_preload.so redirects such a program.
//
//   blas_client <problem file> <result file>
//
// Problem file: nine int64 (api: 0 rocBLAS / 1 hipBLAS typed calls, 2 rocblas_gemm_ex / 3 hipblasGemmEx;
// complex 0/1; transa, transb as 0 N / 1 T / 2 C; m, n, k, repeats, streams), alpha and beta as two doubles each, then A, B, C column-major
// without padding (lda = rows of A as stored, ...). Complex data interleaved. The call is issued
// `repeats` times with the same arguments, round-robin over `streams` streams; with beta = 0 the result
// is that of one call. Result file: C, same layout.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include <hip/hip_runtime.h>
#include <hipblas/hipblas.h>
#include <rocblas/rocblas.h>

#define CHECK(cond)                                                            \
    do {                                                                       \
        if (!(cond)) {                                                         \
            std::fprintf(stderr, "blas_client: %s failed (line %d)\n", #cond, __LINE__); \
            return 1;                                                          \
        }                                                                      \
    } while (0)

int main(int argc, char** argv) {
    CHECK(argc == 3);
    std::FILE* in = std::fopen(argv[1], "rb");
    CHECK(in);
    int64_t h[9];
    double alpha[2], beta[2];
    CHECK(std::fread(h, sizeof(int64_t), 9, in) == 9);
    CHECK(std::fread(alpha, sizeof(double), 2, in) == 2 && std::fread(beta, sizeof(double), 2, in) == 2);
    const int64_t api = h[0], cplx = h[1], ta = h[2], tb = h[3], m = h[4], n = h[5], k = h[6], repeats = h[7], streams = h[8];
    CHECK(m > 0 && n > 0 && k > 0 && repeats >= 1 && streams >= 1 && streams <= 4);
    const int64_t w = cplx ? 2 : 1;
    const int64_t a_rows = ta ? k : m, a_cols = ta ? m : k, b_rows = tb ? n : k, b_cols = tb ? k : n;
    std::vector<double> A(w * a_rows * a_cols), B(w * b_rows * b_cols), C(w * m * n);
    CHECK(std::fread(A.data(), sizeof(double), A.size(), in) == A.size());
    CHECK(std::fread(B.data(), sizeof(double), B.size(), in) == B.size());
    CHECK(std::fread(C.data(), sizeof(double), C.size(), in) == C.size());
    std::fclose(in);

    double *dA, *dB, *dC;
    CHECK(hipMalloc(&dA, A.size() * 8) == hipSuccess && hipMalloc(&dB, B.size() * 8) == hipSuccess &&
          hipMalloc(&dC, C.size() * 8) == hipSuccess);
    CHECK(hipMemcpy(dA, A.data(), A.size() * 8, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(dB, B.data(), B.size() * 8, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(dC, C.data(), C.size() * 8, hipMemcpyHostToDevice) == hipSuccess);
    hipStream_t st[4];
    for (int i = 0; i < streams; ++i) CHECK(hipStreamCreate(&st[i]) == hipSuccess);

    if (api == 0 || api == 2) {
        rocblas_handle handle;
        CHECK(rocblas_create_handle(&handle) == rocblas_status_success);
        const rocblas_operation ops[3] = {rocblas_operation_none, rocblas_operation_transpose,
                                          rocblas_operation_conjugate_transpose};
        for (int64_t r = 0; r < repeats; ++r) {
            CHECK(rocblas_set_stream(handle, st[r % streams]) == rocblas_status_success);
            rocblas_status rc;
            if (api == 2) {
                const rocblas_datatype ty = cplx ? rocblas_datatype_f64_c : rocblas_datatype_f64_r;
                rc = rocblas_gemm_ex(handle, ops[ta], ops[tb], (rocblas_int)m, (rocblas_int)n, (rocblas_int)k, alpha, dA, ty,
                                     (rocblas_int)a_rows, dB, ty, (rocblas_int)b_rows, beta, dC, ty, (rocblas_int)m, dC, ty,
                                     (rocblas_int)m, ty, rocblas_gemm_algo_standard, 0, 0);
            } else if (cplx)
                rc = rocblas_zgemm(handle, ops[ta], ops[tb], (rocblas_int)m, (rocblas_int)n, (rocblas_int)k,
                                   reinterpret_cast<const rocblas_double_complex*>(alpha),
                                   reinterpret_cast<const rocblas_double_complex*>(dA), (rocblas_int)a_rows,
                                   reinterpret_cast<const rocblas_double_complex*>(dB), (rocblas_int)b_rows,
                                   reinterpret_cast<const rocblas_double_complex*>(beta),
                                   reinterpret_cast<rocblas_double_complex*>(dC), (rocblas_int)m);
            else
                rc = rocblas_dgemm(handle, ops[ta], ops[tb], (rocblas_int)m, (rocblas_int)n, (rocblas_int)k, alpha, dA,
                                   (rocblas_int)a_rows, dB, (rocblas_int)b_rows, beta, dC, (rocblas_int)m);
            CHECK(rc == rocblas_status_success);
        }
        CHECK(hipDeviceSynchronize() == hipSuccess);
        CHECK(rocblas_destroy_handle(handle) == rocblas_status_success);
    } else {
        hipblasHandle_t handle;
        CHECK(hipblasCreate(&handle) == HIPBLAS_STATUS_SUCCESS);
        const hipblasOperation_t ops[3] = {HIPBLAS_OP_N, HIPBLAS_OP_T, HIPBLAS_OP_C};
        for (int64_t r = 0; r < repeats; ++r) {
            CHECK(hipblasSetStream(handle, st[r % streams]) == HIPBLAS_STATUS_SUCCESS);
            hipblasStatus_t rc;
            if (api == 3) {
                const hipDataType ty = cplx ? HIP_C_64F : HIP_R_64F;
                rc = hipblasGemmEx(handle, ops[ta], ops[tb], (int)m, (int)n, (int)k, alpha, dA, ty, (int)a_rows, dB, ty,
                                   (int)b_rows, beta, dC, ty, (int)m, HIPBLAS_COMPUTE_64F, HIPBLAS_GEMM_DEFAULT);
            } else if (cplx)
                rc = hipblasZgemm(handle, ops[ta], ops[tb], (int)m, (int)n, (int)k,
                                  reinterpret_cast<const hipDoubleComplex*>(alpha),
                                  reinterpret_cast<const hipDoubleComplex*>(dA), (int)a_rows,
                                  reinterpret_cast<const hipDoubleComplex*>(dB), (int)b_rows,
                                  reinterpret_cast<const hipDoubleComplex*>(beta), reinterpret_cast<hipDoubleComplex*>(dC),
                                  (int)m);
            else
                rc = hipblasDgemm(handle, ops[ta], ops[tb], (int)m, (int)n, (int)k, alpha, dA, (int)a_rows, dB, (int)b_rows,
                                  beta, dC, (int)m);
            CHECK(rc == HIPBLAS_STATUS_SUCCESS);
        }
        CHECK(hipDeviceSynchronize() == hipSuccess);
        CHECK(hipblasDestroy(handle) == HIPBLAS_STATUS_SUCCESS);
    }

    CHECK(hipMemcpy(C.data(), dC, C.size() * 8, hipMemcpyDeviceToHost) == hipSuccess);
    std::FILE* out = std::fopen(argv[2], "wb");
    CHECK(out);
    CHECK(std::fwrite(C.data(), sizeof(double), C.size(), out) == C.size());
    std::fclose(out);
    return 0;
}
