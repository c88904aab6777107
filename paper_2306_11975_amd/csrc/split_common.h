// Bit-level pieces of SplitInt (Section 3.1; cut by bit operations, Section 4.1) shared by the splitter
// kernels and by the kernel that splits the rows of a state vector on the fly: the exponent of a row
// maximum, an element as a fixed-point fraction under that exponent, and its signed 7-bit slices.
#pragma once

#include "ozimmu_internal.h"

namespace ozimmu {
namespace {

constexpr unsigned long long kAbsMask = 0x7fffffffffffffffull;
constexpr unsigned long long kMantMask = 0x000fffffffffffffull;

// Exponent E with maxabs < 2^E and maxabs >= 2^(E-1); 0 for a zero row.
__device__ __forceinline__ int exponent_of_max(unsigned long long maxbits) {
    if (maxbits == 0) return 0;
    int e = (int)(maxbits >> 52);
    if (e != 0) return e - 1022;
    return (64 - __clzll((long long)maxbits)) - 1074;  // subnormal maximum
}

// |x| 2^(-E) < 1 as a binary fraction of up to 128 bits: bit 63 of hi has weight 1/2. Slice p is
// the p-th group of 7 bits after the binary point (truncation: the bits are simply cut), so once
// the significand sits at its place every slice is a bit field at a fixed position. The one
// shift whose amount varies from element to element is paid once, not once per slice.
struct Fixed {
    unsigned long long hi, lo;
};

template <bool WIDE>   // WIDE: more than 9 slices, i.e. more than the 63 bits the upper half can serve
__device__ __forceinline__ Fixed to_fixed(unsigned long long bits, int E) {
    const unsigned e = (unsigned)(bits >> 52) & 0x7ffu;
    const unsigned long long mant = bits & kMantMask;
    // significand with its leading bit at bit 63 (subnormal: no implicit bit, exponent field 1)
    const unsigned long long T = (e ? (mant | (1ull << 52)) : mant) << 11;
    // right shift that puts the binary point of |x| 2^(-E) just above bit 63. Never negative for
    // normal numbers (|x| < 2^E); in a subnormal row the significands have leading zeros of
    // their own and the shift of the largest ones goes the other way (by at most 52).
    const int z = E + 1022 - (int)(e ? e : 1u);
    Fixed f;
    f.hi = z < 0 ? T << (-z) : z < 64 ? T >> z : 0ull;
    f.lo = 0ull;
    if (WIDE) f.lo = z <= 0 ? 0ull : z < 64 ? T << (64 - z) : z < 128 ? T >> (z - 64) : 0ull;
    return f;
}

// Magnitude of slice p (1-based). With p a constant after unrolling this is one bit-field
// extract of a 32-bit half, or a funnel shift when the field straddles two words.
__device__ __forceinline__ unsigned field(const Fixed& f, int p) {
    const int o = OZIMMU_SLICE_BITS * (p - 1);   // bits of the fraction ahead of the field
    if (o + OZIMMU_SLICE_BITS <= 64) return (unsigned)(f.hi >> (64 - OZIMMU_SLICE_BITS - o)) & 127u;
    if (o >= 64) return (unsigned)(f.lo >> (128 - OZIMMU_SLICE_BITS - o)) & 127u;
    return ((unsigned)(f.hi << (o + OZIMMU_SLICE_BITS - 64)) & 127u) | (unsigned)(f.lo >> (128 - OZIMMU_SLICE_BITS - o));
}

// Signs of four consecutive elements as byte masks, and the byte-wise negation of the packed
// magnitudes c (each 0..127) where the sign is set: per byte (c ^ 0xff) + 1 without a carry into
// the next byte, i.e. the low seven bits are added on their own and the top bit is put back.
struct SignMask {
    uint32_t m7, m1, m80;
};
__device__ __forceinline__ SignMask sign_mask(unsigned long long b0, unsigned long long b1,
                                              unsigned long long b2, unsigned long long b3) {
    const uint32_t m = ((uint32_t)(b0 >> 63) * 0xffu) | ((uint32_t)(b1 >> 63) * 0xff00u) |
                       ((uint32_t)(b2 >> 63) * 0xff0000u) | ((uint32_t)(b3 >> 63) * 0xff000000u);
    return {m & 0x7f7f7f7fu, m & 0x01010101u, m & 0x80808080u};
}
__device__ __forceinline__ uint32_t apply_sign(uint32_t packed, const SignMask& sm) {
    return ((packed ^ sm.m7) + sm.m1) ^ sm.m80;
}
template <bool WIDE>
__device__ __forceinline__ uint32_t packed_slice(const Fixed (&x)[4], const SignMask& sm, int p) {
    const uint32_t c = field(x[0], p) | (field(x[1], p) << 8) | (field(x[2], p) << 16) | (field(x[3], p) << 24);
    return apply_sign(c, sm);
}

// max(x, x of the lane N further round the row of 16 lanes): four of them (N = 8, 4, 2, 1) leave the row's maximum in every lane
template <int N>
__device__ __forceinline__ unsigned row_max_step(unsigned x) {
    const unsigned o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x120 + N, 0xf, 0xf, false);
    return o > x ? o : x;
}

// Slice-count scan (Section 4.4, automatic choice of the number of slices): with the row or column exponent E, z is the
// distance of an element's leading bit below the binary point (clamped to 7 x 16) and L the number of bits it stores;
// s slices lose max(0, z + L - 7 s) - max(0, z - 7 s) of them.
// z (clamped) and L of one element; both 0 for a zero.
__device__ __forceinline__ void loss_position(unsigned long long bits, int E, uint32_t& z, uint32_t& L) {
    const unsigned long long mag = bits & kAbsMask;
    const int e = (int)(mag >> 52);
    int zz = E + 1022 - e, LL = 53;
    if (e == 0) {                       // zero, or subnormal with leading bit b of the stored field
        if (mag == 0) {
            zz = 0;
            LL = 0;
        } else {
            const int b = 63 - __clzll((long long)mag);
            LL = b + 1;
            zz = E + 1073 - b;
        }
    }
    z = (uint32_t)(zz < 0 ? 0 : zz > OZIMMU_SLICE_BITS * OZIMMU_MAX_SLICES ? OZIMMU_SLICE_BITS * OZIMMU_MAX_SLICES : zz);
    L = (uint32_t)LL;
}

// What the check of a guessed slice count g needs of a plane: sums of |v - 7 g|, |z - 7 g|, the same for g - 1, and of
// the stored bits L (v = z + L); the bits lost with s slices are (sum |v - 7 s| - sum |z - 7 s| + sum L) / 2.
constexpr int kScanCounters = 5;
struct ScanCount {
    uint32_t sv_g, sz_g, sv_h, sz_h, bits;
};
// A kernel that counts while it splits: per plane five 64-bit counters in one of kScanSlots slots (a workgroup adds
// into slot blockIdx.x % kScanSlots: few workgroups meet on an address), nc counters to a slot.
constexpr int kScanSlots = 2048;
struct ScanTarget {
    unsigned long long* slots;   // null: no counting; else zeroed [kScanSlots][nc], this plane's five at + 0 .. 4
    int nc;                      // counters per slot (5 per plane of the operand)
    uint32_t edge_g, edge_h;     // 7 g and 7 (g - 1) in every byte
};
__device__ __forceinline__ void scan_count4(ScanCount& a, const unsigned long long (&b)[4], int E, uint32_t edge_g, uint32_t edge_h) {
    uint32_t pz = 0, pl = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        uint32_t z, L;
        loss_position(b[u], E, z, L);
        pz |= z << (8 * u);
        pl |= L << (8 * u);
    }
    const uint32_t pv = pz + pl;   // bytewise: no byte exceeds 165
    a.bits = __builtin_amdgcn_sad_u8(pl, 0u, a.bits);
    a.sv_g = __builtin_amdgcn_sad_u8(pv, edge_g, a.sv_g);
    a.sz_g = __builtin_amdgcn_sad_u8(pz, edge_g, a.sz_g);
    a.sv_h = __builtin_amdgcn_sad_u8(pv, edge_h, a.sv_h);
    a.sz_h = __builtin_amdgcn_sad_u8(pz, edge_h, a.sz_h);
}
// The workgroup's counters -> its slot. lds: five zeroed words; every thread of the workgroup calls this.
__device__ __forceinline__ void scan_flush(const ScanCount& a, unsigned* lds, const ScanTarget& t) {
    unsigned c[kScanCounters] = {a.sv_g, a.sz_g, a.sv_h, a.sz_h, a.bits};
#pragma unroll
    for (int i = 0; i < kScanCounters; ++i) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) c[i] += __shfl_xor(c[i], off, 64);
        if ((threadIdx.x & 63) == 0 && c[i]) atomicAdd(&lds[i], c[i]);
    }
    __syncthreads();
    if (threadIdx.x < kScanCounters && lds[threadIdx.x])
        atomicAdd(&t.slots[(size_t)(blockIdx.x % kScanSlots) * t.nc + threadIdx.x], (unsigned long long)lds[threadIdx.x]);
}

// sum over the row of 16 lanes, left in every lane of it (rotations by 8, 4, 2, 1)
template <int N>
__device__ __forceinline__ unsigned row_sum_step(unsigned x) {
    return x + (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x120 + N, 0xf, 0xf, false);
}

}  // namespace
}  // namespace ozimmu
