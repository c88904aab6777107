// Device helpers shared by the slice-product kernels (gfx950 only).
#pragma once

#include <type_traits>

#include "ozimmu_internal.h"

namespace ozimmu {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef long long v2l __attribute__((ext_vector_type(2)));

// Workgroup -> tile. Hardware deals workgroups round-robin over the 8 XCDs (each with its own
// L2); give every XCD a contiguous run of tiles, ordered in column panels 8 tiles tall so that
// the 32 workgroups resident on an XCD (8 x 4 tiles) share A and B panels through that L2.
__device__ __forceinline__ void tile_of_logical(int logical, int tiles_m, int tiles_n, int& tm, int& tn) {
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = logical / per_group;
    const int first_m = group * GM;
    const int rows = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
    const int in_group = logical - group * per_group;
    tm = first_m + in_group % rows;
    tn = in_group / rows;
}
// XCD x owns the logical tiles [first, first + count): the total is dealt out in eight nearly equal runs.
__device__ __forceinline__ void xcd_tile_range(int xcd, int total, int& first, int& count) {
    const int q = total >> 3, r = total & 7;
    first = xcd * q + (xcd < r ? xcd : r);
    count = q + (xcd < r ? 1 : 0);
}
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
    int first, count;
    xcd_tile_range(bid & 7, tiles_m * tiles_n, first, count);
    tile_of_logical(first + (bid >> 3), tiles_m, tiles_n, tm, tn);
}

// A zero the optimiser cannot see through. Address arithmetic of the code that runs after the
// k-walk is made to depend on it, so that it is computed there and not hoisted above the walk,
// where it would occupy registers the matrix-core loop needs.
__device__ __forceinline__ unsigned opaque_zero() {
    unsigned z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

// The same in a scalar register, for wave-uniform values that are to be formed after the k-walk.
__device__ __forceinline__ int opaque_scalar_zero() {
    int z;
    asm volatile("s_mov_b32 %0, 0" : "=s"(z));
    return z;
}

// The lane number, formed where it is asked for (not once ahead of the k-walk, where the value would have to
// be kept, or spilled, across it).
__device__ __forceinline__ int lane_here() {
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=&v"(l));
    return l;
}

// The accumulators live in the accumulation half of the register file for the whole k-walk.
// Initialising and reading them through these two helpers pins that choice, so that no copies
// between the two halves of the file are made around the loop.
__device__ __forceinline__ int acc_zero() {
    int a;
    asm("v_accvgpr_write_b32 %0, 0" : "=a"(a));
    return a;
}
__device__ __forceinline__ int acc_read(int a) {
    int v;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// To be called between the last MFMA and the first acc_read of its results. The reads sit in inline assembly,
// where the compiler does not see them: it neither inserts the wait states that a read of a matrix-core result
// needs (up to 19 after the issue of an MFMA of sixteen passes) nor keeps other instructions from moving in
// between. Everything issued so far stays ahead of this point and 32 wait states pass before anything after it.
__device__ __forceinline__ void mfma_results_ready() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// One wavefront-wide direct load: lane i fetches 16 bytes from gbase + voff_i and the hardware
// writes them to LDS at lds_addr + 16 i (M0 carries the LDS base). Issued as inline assembly so
// that its completion is awaited only by the explicit vmcnt before the step barrier and not
// before every LDS read in between.
__device__ __forceinline__ void dma_load16(const void* gbase, unsigned voff, unsigned lds_addr) {
    // both are wave-uniform by construction; should the register allocator have parked one of them in a
    // vector register, this brings it back into a scalar one (it costs nothing otherwise)
    const unsigned long long gb = (unsigned long long)gbase;
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)gb);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(gb >> 32));
    const void* gs = (const void*)(((unsigned long long)hi << 32) | lo);
    const unsigned la = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr);
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %0"
        :
        : "s"(gs), "v"(voff), "s"(la)
        : "memory");  // M0 is written here (the compiler refuses it as a clobber: reserved register); the build
                      // checks the generated assembly for any other use of M0 in the kernels
}

// Wait until at most N of this wave's direct loads are outstanding (they return in order, so
// everything older has landed) and until its own LDS reads are done, then meet the other waves.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(N) : "memory");
}

// Compile-time loop: f(integral_constant<int, I>) for I = BEGIN .. END - 1.
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}

__device__ __forceinline__ v16i mfma(const v4i& a, const v4i& b, const v16i& c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

// acc = RN(acc + S_e 2^(-7 (e + 2))) for the diagonals of a band, least significant first. The
// product of an integer below 2^31 and a power of two is exact, so the fused operation rounds
// exactly like the sum it stands for.
template <int SB>
__device__ __forceinline__ void fold_band(double (&sum)[16], const v16i (&acc)[kBand]) {
    constexpr int ND = SB < kBand ? SB : kBand, E0 = SB - ND;
    mfma_results_ready();
#pragma unroll
    for (int e = SB - 1; e >= E0; --e) {
        const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * (e + 2)) << 52);
#pragma unroll
        for (int u = 0; u < 16; ++u) sum[u] = fma((double)acc_read(acc[e - E0][u]), sc, sum[u]);
        __builtin_amdgcn_sched_barrier(0);   // one diagonal's temporaries at a time
    }
}

// Raise a kernel's dynamic LDS limit once per device instead of before every launch (the call
// is a host-side driver round trip, and it keeps the launch path free of anything but the launch).
// One instantiation, hence one set of flags, per kernel. Two host threads racing here both make
// the (idempotent) driver call.
template <auto kernel>
inline hipError_t allow_dynamic_lds(int bytes) {
    static bool done[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && done[dev]) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 64) done[dev] = true;
    return e;
}

}  // namespace
}  // namespace ozimmu
