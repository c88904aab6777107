// Device characterisation probes (not part of the DGEMM path): the sustained INT8 MFMA issue rate
// of the chip for a given operand bit pattern, and the LDS ds_read_b128 throughput for a given
// address pattern. The benchmark reports the first next to the kernel's roofline fraction: on
// MI355X the matrix-core clock under load depends on how many operand bits toggle, so the
// published peak (measured at the boost clock) is not reachable with random 7-bit slices.
#include "ozimmu_internal.h"

namespace ozimmu {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ unsigned mix(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// Register-only issue loop: 16 independent 32x32x32 INT8 MFMAs per iteration, 4 waves per CU.
// pattern 0: all-zero operands, 1: random bytes, 2: random 7-bit magnitudes with random sign
// (sign-magnitude values in [-127, 127], the value distribution of Ozaki slices beyond the first),
// 3: random signed 3-bit magnitudes, 4: random 7-bit magnitudes without sign, 5: A as 2 and every
// byte of B equal to 1, 6: A as 2 and B zero.
__global__ __launch_bounds__(256) void mfma_rate_kernel(int pattern, int iters, int* sink, long long* clocks) {
    const long long c0 = clock64(), w0 = wall_clock64();
    v16i acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    v4i a[4], b[4];
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
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 0x12345678) sink[threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clocks[0] = clock64() - c0;
        clocks[1] = wall_clock64() - w0;
    }
}

// 16 waves per CU, 8 independent wave-wide 16-byte LDS reads per iteration.
// pattern 0: lane i reads bytes [16 i, 16 i + 16) (trivially conflict free);
// 1: row (lane % 32) of 64-byte rows, 16-byte column lane / 32, no swizzle;
// 2: the same with the column XOR-ed with bits 2..3 of the row (the slice-tensor block layout).
__global__ __launch_bounds__(1024) void lds_read_kernel(int pattern, int iters, int* sink) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 65536 / 4; i += 1024) reinterpret_cast<int*>(lds)[i] = i;
    __syncthreads();
    const int row = lane & 31, half = lane >> 5;
    unsigned off[4];
    for (int kk = 0; kk < 4; ++kk) {
        const int c = (kk * 2 + half) & 3;
        off[kk] = pattern == 0 ? (unsigned)(lane * 16 + kk * 1024)
                : pattern == 1 ? (unsigned)(row * 64 + (c << 4) + (kk >> 1) * 2048)
                               : (unsigned)(row * 64 + ((c ^ ((row >> 2) & 3)) << 4) + (kk >> 1) * 2048);
    }
    const unsigned base = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char*)lds + (wave & 3) * 8192;
    const unsigned a0 = base + off[0], a1 = base + off[1], a2 = base + off[2], a3 = base + off[3];
    v4i x0, x1, x2, x3, x4, x5, x6, x7;
    for (int it = 0; it < iters; ++it) {
        asm volatile(
            "ds_read_b128 %0, %8\n\t"
            "ds_read_b128 %1, %9\n\t"
            "ds_read_b128 %2, %10\n\t"
            "ds_read_b128 %3, %11\n\t"
            "ds_read_b128 %4, %8 offset:4096\n\t"
            "ds_read_b128 %5, %9 offset:4096\n\t"
            "ds_read_b128 %6, %10 offset:4096\n\t"
            "ds_read_b128 %7, %11 offset:4096\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3), "=&v"(x4), "=&v"(x5), "=&v"(x6), "=&v"(x7)
            : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
            : "memory");
    }
    v4i acc = x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7;
    if (acc[0] == 0x12345678) sink[tid] = acc[1] + acc[2] + acc[3];
}

}  // namespace
}  // namespace ozimmu

using namespace ozimmu;

extern "C" {

// Allocates a few KiB of device and pinned host memory for the duration of the call and
// synchronises the device: a measurement utility, not a building block.
ozimmu_status_t ozimmu_probe_int8_mfma(int pattern, int iters, double* tera_ops_per_s, double* shader_mhz) {
    if (pattern < 0 || pattern > 6 || iters < 1) return OZIMMU_ERR_BAD_DIM;
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
    if (ok) {
        mfma_rate_kernel<<<dim3(cus), dim3(256)>>>(pattern, 64, sink, clocks);  // warm-up
        ok = hipEventRecord(e0) == hipSuccess;
        mfma_rate_kernel<<<dim3(cus), dim3(256)>>>(pattern, iters, sink, clocks);
        ok = ok && hipEventRecord(e1) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
             hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    }
    if (ok && ms > 0.f) {
        *tera_ops_per_s = (double)cus * 4.0 * iters * 16.0 * 65536.0 / (ms * 1e-3) / 1e12;
        *shader_mhz = clocks[1] > 0 ? (double)clocks[0] / (double)clocks[1] * 100.0 : 0.0;  // wall clock: 100 MHz
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (clocks) (void)hipHostFree(clocks);
    return ok ? OZIMMU_OK : OZIMMU_ERR_HIP;
}

ozimmu_status_t ozimmu_probe_lds_read(int pattern, int iters, double* bytes_per_ns_per_cu) {
    if (pattern < 0 || pattern > 2 || iters < 1) return OZIMMU_ERR_BAD_DIM;
    if (!bytes_per_ns_per_cu) return OZIMMU_ERR_NULL;
    int cus = 0, dev = 0;
    int* sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok = hipGetDevice(&dev) == hipSuccess &&
              hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
              hipMalloc(&sink, 8192) == hipSuccess && hipEventCreate(&e0) == hipSuccess &&
              hipEventCreate(&e1) == hipSuccess &&
              hipFuncSetAttribute(reinterpret_cast<const void*>(&lds_read_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 65536) == hipSuccess;
    float ms = 0.f;
    if (ok) {
        lds_read_kernel<<<dim3(cus), dim3(1024), 65536>>>(pattern, 64, sink);
        ok = hipEventRecord(e0) == hipSuccess;
        lds_read_kernel<<<dim3(cus), dim3(1024), 65536>>>(pattern, iters, sink);
        ok = ok && hipEventRecord(e1) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
             hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    }
    if (ok && ms > 0.f) *bytes_per_ns_per_cu = (double)iters * 8.0 * 16.0 * 1024.0 / (ms * 1e6);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    return ok ? OZIMMU_OK : OZIMMU_ERR_HIP;
}

}  // extern "C"
