// Device characterisation probe (not part of the DGEMM path): the sustained INT8 MFMA issue rate
// of the chip for a given operand bit pattern and MFMA shape. The benchmark reports it next to the
// kernel's roofline fraction: on MI355X the matrix-core clock under load depends on how many operand
// bits toggle, so the published peak (measured at the boost clock) is not reachable with random
// 7-bit slices.
#include "ozimmu_internal.h"
#include "ozimmu_probe.h"

namespace ozimmu {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ unsigned mix(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// Four operand pairs of a lane for the given pattern.
__device__ __forceinline__ void probe_operands(int pattern, v4i (&a)[4], v4i (&b)[4]) {
    for (int i = 0; i < 4; ++i)
        for (int c = 0; c < 4; ++c) {
            unsigned ha = mix(threadIdx.x * 64 + i * 8 + c + blockIdx.x * 7919), hb = mix(ha + 12345);
            if (pattern == 0) ha = hb = 0;
            if (pattern >= 2) {
                // bytes as sign-magnitude values: `bits` magnitude bits, sign from bit 7 unless unsigned
                const int bits = pattern == 3 ? 3 : 7;
                const bool with_sign = pattern != 4;
                unsigned va = 0, vb = 0;
                for (int k = 0; k < 4; ++k) {
                    int xa = (int)((ha >> (8 * k)) & ((1u << bits) - 1u)), xb = (int)((hb >> (8 * k)) & ((1u << bits) - 1u));
                    if (with_sign && ((ha >> (8 * k + 7)) & 1)) xa = -xa;
                    if (with_sign && ((hb >> (8 * k + 7)) & 1)) xb = -xb;
                    va |= ((unsigned)xa & 255u) << (8 * k);
                    vb |= ((unsigned)xb & 255u) << (8 * k);
                }
                ha = va;
                hb = pattern == 5 ? 0x01010101u : pattern == 6 ? 0u : vb;
            }
            a[i][c] = (int)ha;
            b[i][c] = (int)hb;
        }
}

// The small shape with four wavefronts per SIMD (a workgroup of sixteen wavefronts per CU, at most 128 registers): 16
// independent v_mfma_i32_16x16x64_i8 per iteration, 4 result registers each.
__global__ __launch_bounds__(1024) void mfma_rate_small_kernel(int pattern, int iters, int* sink, long long* clocks) {
    const long long c0 = clock64(), w0 = wall_clock64();
    v4i acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = v4i{0, 0, 0, 0};
    v4i a[4], b[4];
    probe_operands(pattern, a, b);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i * 4 + j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 0x12345678) sink[threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clocks[0] = clock64() - c0;
        clocks[1] = wall_clock64() - w0;
    }
}

// Register-only issue loop: 16 independent INT8 MFMAs per iteration (SHAPE 0: 32x32x32, 16 result
// registers each, 32768 multiply-adds; SHAPE 2: the older 16x16x32, 64 instructions of 8192 multiply-adds
// per iteration), one workgroup of four wavefronts per CU (one wavefront per SIMD).
// pattern 0: all-zero operands, 1: random bytes, 2: random 7-bit magnitudes with random sign
// (sign-magnitude values in [-127, 127], the value distribution of Ozaki slices beyond the first),
// 3: random signed 3-bit magnitudes, 4: random 7-bit magnitudes without sign, 5: A as 2 and every
// byte of B equal to 1, 6: A as 2 and B zero.
template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int pattern, int iters, int* sink, long long* clocks) {
    const long long c0 = clock64(), w0 = wall_clock64();
    v16i acc[16];
    v4i acc4[32];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc4[i][r] = 0;
    v4i a[4], b[4];
    probe_operands(pattern, a, b);
    for (int it = 0; it < iters; ++it) {
        if (SHAPE == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i * 4 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
        } else if (SHAPE == 2) {   // 64 instructions of a quarter of the size, 8 operand bytes per lane
#pragma unroll
            for (int h = 0; h < 4; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const long a8 = (long)(((unsigned long)(unsigned)a[i][1] << 32) | (unsigned)a[i][0]);
                        const long b8 = (long)(((unsigned long)(unsigned)b[j][1] << 32) | (unsigned)b[j][0]);
                        acc4[(h & 1) * 16 + i * 4 + j] = __builtin_amdgcn_mfma_i32_16x16x32_i8(a8, b8, acc4[(h & 1) * 16 + i * 4 + j], 0, 0, 0);
                    }
        }
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
#pragma unroll
    for (int i = 0; i < 32; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) s += acc4[i][r];
    if (s == 0x12345678) sink[threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clocks[0] = clock64() - c0;
        clocks[1] = wall_clock64() - w0;
    }
}

}  // namespace
}  // namespace ozimmu

using namespace ozimmu;

extern "C" {

// Allocates a few KiB of device and pinned host memory for the duration of the call and
// synchronises the device: a measurement utility, not a building block.
ozimmu_status_t ozimmu_probe_int8_mfma(int pattern, int shape, int iters, double* tera_ops_per_s, double* shader_mhz) {
    if (pattern < 0 || pattern > 6 || shape < 0 || shape > 2 || iters < 1) return OZIMMU_ERR_BAD_DIM;
    if (!tera_ops_per_s || !shader_mhz) return OZIMMU_ERR_NULL;
    int cus = 0, dev = 0;
    int* sink = nullptr;
    long long* clocks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok = hipGetDevice(&dev) == hipSuccess &&
              hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
              hipMalloc(&sink, 4096) == hipSuccess && hipHostMalloc(&clocks, 64) == hipSuccess &&
              hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
    float ms = 0.f;
    const int waves = shape == 1 ? 16 : 4;   // per CU
    auto launch = [&](int n) {
        if (shape == 0) mfma_rate_kernel<0><<<dim3(cus), dim3(256)>>>(pattern, n, sink, clocks);
        else if (shape == 1) mfma_rate_small_kernel<<<dim3(cus), dim3(1024)>>>(pattern, n, sink, clocks);
        else mfma_rate_kernel<2><<<dim3(cus), dim3(256)>>>(pattern, n, sink, clocks);
    };
    if (ok) {
        launch(64);  // warm-up
        ok = hipEventRecord(e0) == hipSuccess;
        launch(iters);
        ok = ok && hipEventRecord(e1) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
             hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    }
    if (ok && ms > 0.f) {
        const double ops_per_iteration = shape == 1 ? 16.0 * 32768.0 : 16.0 * 65536.0;   // per wavefront
        *tera_ops_per_s = (double)cus * waves * iters * ops_per_iteration / (ms * 1e-3) / 1e12;
        *shader_mhz = clocks[1] > 0 ? (double)clocks[0] / (double)clocks[1] * 100.0 : 0.0;  // wall clock: 100 MHz
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (clocks) (void)hipHostFree(clocks);
    return ok ? OZIMMU_OK : OZIMMU_ERR_HIP;
}

}  // extern "C"
