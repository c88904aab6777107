// Stand-alone use of the C ABI (no Python, no framework): allocate with HIP, ask for the number
// of slices that splits the inputs without loss, multiply, and compare with a plain FP64 loop.
//   hipcc -Iinclude example_dgemm.cpp -L. -lozimmu
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <random>
#include <vector>

#include "ozimmu.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 2; } } while (0)
#define CHECK_OZ(x) do { ozimmu_status_t s_ = (x); if (s_ != OZIMMU_OK) { std::printf("ozimmu error: %s at %s:%d\n", ozimmu_status_string(s_), __FILE__, __LINE__); return 3; } } while (0)

int main() {
    const int64_t m = 300, n = 200, k = 1500;
    std::mt19937_64 rng(1);
    std::uniform_real_distribution<double> uni(-0.5, 0.5);
    std::normal_distribution<double> nor(0.0, 1.0);
    std::vector<double> A(m * k), B(k * n), C(m * n);
    for (auto& x : A) x = uni(rng) * std::exp(nor(rng));
    for (auto& x : B) x = uni(rng) * std::exp(nor(rng));

    double *dA, *dB, *dC;
    CHECK_HIP(hipMalloc(&dA, sizeof(double) * A.size()));
    CHECK_HIP(hipMalloc(&dB, sizeof(double) * B.size()));
    CHECK_HIP(hipMalloc(&dC, sizeof(double) * C.size()));
    CHECK_HIP(hipMemcpy(dA, A.data(), sizeof(double) * A.size(), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dB, B.data(), sizeof(double) * B.size(), hipMemcpyHostToDevice));

    size_t scratch_bytes = 0, ws_bytes = 0;
    CHECK_OZ(ozimmu_auto_scratch_bytes(n, &scratch_bytes));
    void* scratch;
    CHECK_HIP(hipMalloc(&scratch, scratch_bytes));
    int slices = 0;
    CHECK_OZ(ozimmu_auto_num_slices(m, n, k, dA, k, dB, n, 0, /*threshold=*/0.0, OZIMMU_MAX_SLICES, scratch,
                                    scratch_bytes, &slices, nullptr, nullptr));
    CHECK_OZ(ozimmu_workspace_bytes(m, n, k, slices, 0, &ws_bytes));
    void* ws;
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    CHECK_OZ(ozimmu_dgemm(m, n, k, dA, k, dB, n, dC, n, slices, ws, ws_bytes, nullptr));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(C.data(), dC, sizeof(double) * C.size(), hipMemcpyDeviceToHost));

    double worst = 0.0;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double ref = 0.0, mag = 0.0;
            for (int64_t l = 0; l < k; ++l) {
                ref += A[i * k + l] * B[l * n + j];
                mag += std::fabs(A[i * k + l] * B[l * n + j]);
            }
            worst = std::fmax(worst, std::fabs(C[i * n + j] - ref) / mag);
        }
    std::printf("ozimmu_dgemm %lldx%lldx%lld with %d slices (lossless split): max |C - C_fp64| / (|A||B|) = %.3g\n",
                (long long)m, (long long)n, (long long)k, slices, worst);
    (void)hipFree(dA); (void)hipFree(dB); (void)hipFree(dC); (void)hipFree(scratch); (void)hipFree(ws);
    return worst < 1e-13 ? 0 : 1;   // both are FP64-accurate: they differ by a few rounding errors of the plain loop
}
