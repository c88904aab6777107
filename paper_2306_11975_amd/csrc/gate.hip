// A gate on a state vector (Section 4.4): the complex product of a tall operand Z (m x k, the reshaped state,
// interleaved re/im) with a small one (B: k x n, the gate), k and n at most 128 (256 with up to eight slices), in ONE kernel
// that reads Z once and writes the result once.
//
// With so short an inner dimension the product is bound by the memory traffic of the state and by the vector
// work around the matrix cores (cutting the state into slices, folding the diagonals in FP64), and splitting the
// state in a kernel of its own doubles that traffic (slices written, slices read back). Here a workgroup of four
// wavefronts (eight when k or n exceeds 64, sixteen beyond 128) takes 32 rows of Z: it finds the exponents of their
// real and imaginary parts and cuts both planes into
// slices (SplitInt, Section 3.1; the same bit operations as the splitter kernels) straight into LDS, as operand
// fragments of v_mfma_i32_16x16x64_i8 (16 rows x 64 positions of k).
//
// The gate is split beforehand (gate_split_kernel) into two slice tensors whose 16-row fragments interleave its
// planes: fragment f of T1 holds columns 8 f .. 8 f + 7 of Br in rows 0..7 and the same columns of Bi in rows
// 8..15, T2 the other way round. A wavefront owns 16 rows and 8 complex columns at a time: Ar times a T1 fragment
// gives G(Ar,Br) in lanes 0..7 (of every 16) and G(Ar,Bi) in lanes 8..15, Ai times the T2 fragment gives G(Ai,Bi)
// and G(Ai,Br) in the same lanes, so that one rounded FP64 operation per lane forms re = G(Ar,Br) - G(Ai,Bi) or
// im = G(Ar,Bi) + G(Ai,Br); lanes 8 apart exchange half of their values and every lane stores whole (re, im) pairs.
// All anti-diagonals of a product are resident in registers (four per diagonal), every product is folded in FP64
// in the fixed order, least significant first, and scaled by 2^(EA_i + EB_j) (the summing-up step of the algorithm,
// Section 3.1).
//
// Why the small MFMA shape: a wavefront issues vector instructions at half the rate its SIMD can take them, and
// with the 32 x 32 shape the eight resident diagonals of a patch cost 128 registers, which leaves room for two
// wavefronts per SIMD only: whenever one of them waited for memory or for the matrix core, the vector pipeline ran
// at half speed. With 16 x 16 patches (32 registers for the diagonals) four wavefronts fit a SIMD; beyond eight
// slices (up to 64 registers for the diagonals and as many again for the fragments) two.
// Register allocation is left to the compiler: without accumulation-register operands in inline assembly the MFMA
// results land in ordinary vector registers, where the FP64 fold reads them directly, and a product's first MFMA
// per diagonal takes the constant 0 as its addend instead of cleared registers.
#include "mfma_common.h"
#include "split_common.h"

namespace ozimmu {
namespace {

constexpr int kGateMax = 128;    // largest k and n with more than eight slices
constexpr int kGateMaxFew = 256; // largest k and n with up to eight slices
constexpr int kGateRows = 32;    // rows of Z per workgroup: two fragments of 16
constexpr int kGateStep = 64;    // positions of k per MFMA

// A fragment: 16 rows x 64 positions, 1 KiB. Lane l of the MFMA operand holds row l % 16, positions 16 (l / 16) .. + 15
// (both operands alike, which is all a sum over k needs); its 16 bytes sit at byte 16 l.
__device__ __forceinline__ int frag_offset(int row, int pos) { return ((pos >> 4) * 16 + row) * 16 + (pos & 15); }

// to_fixed for a row whose maximum is a normal number (the shift is then never negative) when only the upper 56 bits
// of the fraction are wanted (eight slices at most): a shift of 64 or more is cut to 63, which leaves nothing there.
__device__ __forceinline__ Fixed to_fixed_upper(unsigned long long bits, int E) {
    const unsigned e = (unsigned)(bits >> 52) & 0x7ffu;
    const unsigned long long mant = bits & kMantMask;
    const unsigned long long T = (e ? (mant | (1ull << 52)) : mant) << 11;
    const unsigned z = (unsigned)(E + 1022) - (e ? e : 1u);
    Fixed f;
    f.hi = T >> (z < 63u ? z : 63u);
    f.lo = 0ull;
    return f;
}

// scan_count4 with the edges of a compile-time slice count (no counters for S - 1 = 0 slices)
template <int S>
__device__ __forceinline__ void scan_count4(ScanCount& a, const unsigned long long (&b)[4], int E) {
    scan_count4(a, b, E, 0x01010101u * (uint32_t)(OZIMMU_SLICE_BITS * S), 0x01010101u * (uint32_t)(OZIMMU_SLICE_BITS * (S > 1 ? S - 1 : 1)));
}

// bits an element at (z, L) loses with s slices
__device__ __forceinline__ unsigned lost_bits(uint32_t z, uint32_t L, int s) {
    const int edge = OZIMMU_SLICE_BITS * s, below = (int)(z + L) - edge, above = (int)z - edge;
    return (unsigned)((below > 0 ? below : 0) - (above > 0 ? above : 0));
}

typedef int v4acc __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4acc mfma16(const v4i& a, const v4i& b, const v4acc& c) {
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------- the gate -> T1, T2, exponents
// One workgroup per fragment f (8 columns of B). Thread (c, w) = (tid % 8, tid / 8) owns column 8 f + c and the four
// positions 4 w .. 4 w + 3 of k. T: tensor t at t * s * nfr * ks KiB, slice q at q * nfr * ks KiB, fragment (f, step)
// at (f ks + step) KiB. E: [t][f][16] exponents of the fragments' rows.
template <bool WIDE>   // more than nine slices: the fraction takes both words of the fixed-point value
__global__ __launch_bounds__(512) void gate_split_kernel(const double* __restrict__ B, int64_t ldb, int k, int n, int s,
                                                         int ks, int nfr, int8_t* __restrict__ T, int32_t* __restrict__ E,
                                                         unsigned* __restrict__ scan) {
    const int tid = threadIdx.x, r8 = tid & 7, w = tid >> 3, f = blockIdx.x, c = f * 8 + r8;
    const ulonglong2* src = reinterpret_cast<const ulonglong2*>(B);
    ulonglong2 v[4];
    unsigned long long mx_re = 0, mx_im = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int l = 4 * w + u;
        v[u] = ulonglong2{0ull, 0ull};
        if (l < k && c < n) v[u] = src[(int64_t)l * ldb + c];
        const unsigned long long a = v[u].x & kAbsMask, b = v[u].y & kAbsMask;
        mx_re = a > mx_re ? a : mx_re;
        mx_im = b > mx_im ? b : mx_im;
    }
    __shared__ unsigned long long colmax[64][8][2];
    __shared__ unsigned lost_lds[4];
    if (scan && tid < 4) lost_lds[tid] = 0u;
    const int words = blockDim.x >> 3;   // 32 (k <= 128) or 64
    colmax[w][r8][0] = mx_re;
    colmax[w][r8][1] = mx_im;
    __syncthreads();
    for (int i = 0; i < words; ++i) {
        mx_re = colmax[i][r8][0] > mx_re ? colmax[i][r8][0] : mx_re;
        mx_im = colmax[i][r8][1] > mx_im ? colmax[i][r8][1] : mx_im;
    }
    const int e_re = exponent_of_max(mx_re), e_im = exponent_of_max(mx_im);
    if (w == 0) {
        E[f * 16 + r8] = e_re;
        E[f * 16 + 8 + r8] = e_im;
        E[nfr * 16 + f * 16 + r8] = e_im;
        E[nfr * 16 + f * 16 + 8 + r8] = e_re;
    }
    if (scan) {
        // the bits the fragment's columns lose with s and with s - 1 slices (Section 4.4): [re s, re s - 1, im s, im s - 1][nfr]
        unsigned lost[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint32_t z, L;
            loss_position(v[u].x, e_re, z, L);
            lost[0] += lost_bits(z, L, s);
            lost[1] += lost_bits(z, L, s - 1);
            loss_position(v[u].y, e_im, z, L);
            lost[2] += lost_bits(z, L, s);
            lost[3] += lost_bits(z, L, s - 1);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) lost[i] += __shfl_xor(lost[i], off, 64);
            if ((tid & 63) == 0 && lost[i]) atomicAdd(&lost_lds[i], lost[i]);
        }
        __syncthreads();
        if (tid < 4) scan[tid * nfr + f] = lost_lds[tid];
    }
    if (4 * w >= kGateStep * ks) return;
    const int64_t slice = (int64_t)nfr * ks * kFragBytes, tensor = (int64_t)s * slice;
    Fixed xr[4], xi[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        xr[u] = to_fixed<WIDE>(v[u].x, e_re);
        xi[u] = to_fixed<WIDE>(v[u].y, e_im);
    }
    const SignMask sr = sign_mask(v[0].x, v[1].x, v[2].x, v[3].x);
    const SignMask si = sign_mask(v[0].y, v[1].y, v[2].y, v[3].y);
    const int l0 = 4 * w, step = l0 / kGateStep, ll = l0 % kGateStep;
    const int64_t lo = (int64_t)(f * ks + step) * kFragBytes + frag_offset(r8, ll);       // first plane of the fragment
    const int64_t hi = (int64_t)(f * ks + step) * kFragBytes + frag_offset(8 + r8, ll);   // second plane
#pragma unroll
    for (int p = 1; p <= (WIDE ? OZIMMU_MAX_SLICES : 9); ++p) {
        if (p <= s) {
            const uint32_t pr = packed_slice<WIDE>(xr, sr, p), pi = packed_slice<WIDE>(xi, si, p);
            int8_t* d = T + (p - 1) * slice;
            *reinterpret_cast<uint32_t*>(d + lo) = pr;
            *reinterpret_cast<uint32_t*>(d + hi) = pi;
            *reinterpret_cast<uint32_t*>(d + tensor + lo) = pi;
            *reinterpret_cast<uint32_t*>(d + tensor + hi) = pr;
        }
    }
}

// ---------------------------------------------------------------------------- the product
// S slices; CLS, the size class of k and n: 0 up to 64 (one step of 64 positions, eight fragments of B, four wavefronts),
// 1 up to 128 (two steps, sixteen fragments), 2 up to 256 (four steps, 32 fragments, sixteen wavefronts; up to eight slices).
// SCAN: the kernel also counts, for the two planes of Z, what the slice-count choice needs to know about S and S - 1
// slices (Section 4.4; five counters per plane and tile, added up by gate_scan_reduce_kernel), so that a caller who
// guessed S can have the guess checked without another pass over Z.
// WAVES: wavefronts of the workgroup: 8 for CLS 1, 16 for CLS 2, 4 for CLS 0 (a gate of at most 32 x 32 has work for no
// more per tile; up to 64 x 64 a lane takes two words of its row and a wavefront four patches): four such workgroups
// then share a compute unit up to eight slices, and the latency of a tile's loads and its barrier hide behind three
// other tiles instead of one.
constexpr int gate_waves(int cls, int few) { return cls == 2 ? 16 : few ? 4 : 8; }
template <int S, int CLS, bool SCAN, int FEW = 0>   // FEW: 1 = four wavefronts, k <= 32; 2 = four wavefronts, two words to a lane
__global__ __launch_bounds__(64 * gate_waves(CLS, FEW)) __attribute__((amdgpu_waves_per_eu(S <= kBand ? 4 : 2, S <= kBand ? 4 : 2)))
void gate_kernel(const GateArgs g) {
    static_assert(!FEW || CLS == 0, "four wavefronts: the smallest class only");
    constexpr bool WIDE = S > 9;   // the slices beyond the ninth come from the lower word of the fixed-point fraction
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int KS = 1 << CLS, NFR = 8 << CLS, WAVES = gate_waves(CLS, FEW), NT = 64 * WAVES;
    constexpr int SLICE = KS * 2 * kFragBytes;   // one slice of one plane of the tile's rows: [step][row fragment]
    constexpr int PLANE = S * SLICE;
    // behind the two planes: exponents of the tile's rows, [plane][32], then those of the gate's fragments, [tensor][NFR][16]
    int* ex = reinterpret_cast<int*>(lds + 2 * PLANE);
    int* ex_gate = ex + 2 * kGateRows;
    unsigned* scan_lds = reinterpret_cast<unsigned*>(ex_gate + 2 * NFR * 16);   // SCAN: [wavefront][plane][5] counters
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row_tile = (int64_t)blockIdx.x * kGateRows;

    // ---- this wavefront's patches: rows 16 rf .. + 15 of the tile, complex columns 8 f .. 8 f + 7 for f = cg, cg + WAVES / 2, ...
    const int rf = wave & 1, cg = wave >> 1;
    const unsigned char* a_rd = lds + rf * kFragBytes + 16 * lane;
    constexpr int BSLICE = NFR * KS * kFragBytes, TENSOR = S * BSLICE;
    auto read_a = [&](int plane, int p, int step) __attribute__((always_inline)) -> v4i {
        return *reinterpret_cast<const v4i*>(a_rd + plane * PLANE + p * SLICE + step * 2 * kFragBytes);
    };
    // fragments of the gate: a wave-uniform byte offset (tensor, fragment) plus the lane's 16 bytes, unsigned, so that the
    // loads take the tensor's address as their scalar base and a 32-bit register as offset
    const unsigned b_lane = 16u * (unsigned)lane;
    auto b_base = [&](int t, int f) __attribute__((always_inline)) -> unsigned {
        return (unsigned)__builtin_amdgcn_readfirstlane(t * TENSOR + f * KS * kFragBytes);
    };
    auto load_b = [&](unsigned base, int q, int step) __attribute__((always_inline)) -> v4i {
        return *reinterpret_cast<const v4i*>(g.T + (base + (unsigned)(q * BSLICE + step * kFragBytes) + b_lane));
    };
    // the gate's fragments of the first walk are requested before anything else: they are on their way while Z is split
    v4i b[S];
    {
        const unsigned first = b_base(0, cg);
        static_for<0, S>([&](auto pc) __attribute__((always_inline)) { b[decltype(pc)::value] = load_b(first, decltype(pc)::value, 0); });
    }

    // ---- the rows of Z -> exponents and slices in LDS. LPR lanes work on a row (16, or 32 with sixteen wavefronts); a
    // lane owns W words of four consecutive complex elements of it (words cl, LPR + cl, ...). A narrow gate (k <= 32,
    // k <= 16) has its rows' live words in 8 or 4 lanes: then half or a quarter of the wavefronts split all 32 rows and
    // the others skip this part. The positions of a step beyond those words are never written: the gate's fragments
    // hold zeros there (gate_split_kernel), and an integer times zero is zero whatever the LDS holds.
    for (int i = tid; i < 2 * NFR * 16; i += NT) ex_gate[i] = g.E[i];
    constexpr int LPR = FEW == 1 ? 16 : NT / kGateRows, W = KS * 16 / LPR;   // (FEW 1: k <= 32, never 16 lanes to a row)
    const int lshift = FEW == 2 ? 3 : CLS == 0 ? (g.k <= 16 ? 2 : g.k <= 32 ? 3 : 4) : (LPR == 32 ? 5 : 4);   // log2 of the lanes per row
    if (tid < (kGateRows << lshift)) {   // whole wavefronts
        const int lrow = tid >> lshift, cl = tid & ((1 << lshift) - 1);
        const int64_t row = row_tile + lrow;
        const bool live = row < g.m;
        const ulonglong2* src = reinterpret_cast<const ulonglong2*>(g.Z) + (live ? row : 0) * g.ldz;
        ulonglong2 v[W][4];
#pragma unroll
        for (int j = 0; j < W; ++j)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int l = (cl + LPR * j) * 4 + u;
                v[j][u] = ulonglong2{0ull, 0ull};
                if (live && l < g.k) v[j][u] = src[l];
            }
        // Exponents of the row's two planes. The high words of the |x| bit patterns decide unless the row's maximum is
        // zero or subnormal: maxima of those over the row's 16 lanes with rotations inside the row, one instruction each.
        unsigned hw_re = 0, hw_im = 0;
#pragma unroll
        for (int j = 0; j < W; ++j)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned a = (unsigned)(v[j][u].x >> 32) & 0x7fffffffu, b2 = (unsigned)(v[j][u].y >> 32) & 0x7fffffffu;
                hw_re = a > hw_re ? a : hw_re;
                hw_im = b2 > hw_im ? b2 : hw_im;
            }
        if (CLS != 0 || lshift == 4) {
            hw_re = row_max_step<1>(row_max_step<2>(row_max_step<4>(row_max_step<8>(hw_re))));
            hw_im = row_max_step<1>(row_max_step<2>(row_max_step<4>(row_max_step<8>(hw_im))));
            if constexpr (LPR == 32) {   // the row's other sixteen lanes
                const unsigned o = __shfl_xor(hw_re, 16, 64), q = __shfl_xor(hw_im, 16, 64);
                hw_re = o > hw_re ? o : hw_re;
                hw_im = q > hw_im ? q : hw_im;
            }
        } else {   // rows of 4 or 8 lanes
            for (int off = 1 << (lshift - 1); off >= 1; off >>= 1) {
                const unsigned o = __shfl_xor(hw_re, off, 64), q = __shfl_xor(hw_im, off, 64);
                hw_re = o > hw_re ? o : hw_re;
                hw_im = q > hw_im ? q : hw_im;
            }
        }
        int e_re = (int)(hw_re >> 20) - 1022, e_im = (int)(hw_im >> 20) - 1022;   // as exponent_of_max for a normal maximum
        const bool normal = __all(hw_re >= 0x00100000u && hw_im >= 0x00100000u);
        if (!normal) {
            // some row of this wavefront has a zero or subnormal maximum (rows past the end of Z among them): full 64-bit maxima
            unsigned long long mx_re = 0, mx_im = 0;
#pragma unroll
            for (int j = 0; j < W; ++j)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned long long a = v[j][u].x & kAbsMask, b2 = v[j][u].y & kAbsMask;
                    mx_re = a > mx_re ? a : mx_re;
                    mx_im = b2 > mx_im ? b2 : mx_im;
                }
            for (int off = 1 << (lshift - 1); off >= 1; off >>= 1) {
                const unsigned long long o = __shfl_xor(mx_re, off, 64), q = __shfl_xor(mx_im, off, 64);
                mx_re = o > mx_re ? o : mx_re;
                mx_im = q > mx_im ? q : mx_im;
            }
            e_re = exponent_of_max(mx_re);
            e_im = exponent_of_max(mx_im);
        }
        if (cl == 0) {
            ex[lrow] = e_re;
            ex[kGateRows + lrow] = e_im;
        }
        ScanCount cnt_re = {}, cnt_im = {};
        auto emit = [&](auto normal_tag) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < W; ++j) {
                Fixed xr[4], xi[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if constexpr (decltype(normal_tag)::value && S <= kBand) {
                        xr[u] = to_fixed_upper(v[j][u].x, e_re);
                        xi[u] = to_fixed_upper(v[j][u].y, e_im);
                    } else {
                        xr[u] = to_fixed<WIDE>(v[j][u].x, e_re);
                        xi[u] = to_fixed<WIDE>(v[j][u].y, e_im);
                    }
                }
                const SignMask sr = sign_mask(v[j][0].x, v[j][1].x, v[j][2].x, v[j][3].x);
                const SignMask si = sign_mask(v[j][0].y, v[j][1].y, v[j][2].y, v[j][3].y);
                if constexpr (SCAN) {
                    const unsigned long long re4[4] = {v[j][0].x, v[j][1].x, v[j][2].x, v[j][3].x};
                    const unsigned long long im4[4] = {v[j][0].y, v[j][1].y, v[j][2].y, v[j][3].y};
                    scan_count4<S>(cnt_re, re4, e_re);
                    scan_count4<S>(cnt_im, im4, e_im);
                }
                const int word = cl + LPR * j;   // sixteen words to a step
                unsigned char* dst = lds + ((word >> 4) * 2 + (lrow >> 4)) * kFragBytes + frag_offset(lrow & 15, (word & 15) * 4);
                static_for<1, S + 1>([&](auto pc) __attribute__((always_inline)) {
                    constexpr int p = decltype(pc)::value;
                    *reinterpret_cast<uint32_t*>(dst + (p - 1) * SLICE) = packed_slice<WIDE>(xr, sr, p);
                    *reinterpret_cast<uint32_t*>(dst + PLANE + (p - 1) * SLICE) = packed_slice<WIDE>(xi, si, p);
                });
                __builtin_amdgcn_sched_barrier(0);   // one word's temporaries at a time
            }
        };
        if (normal) emit(std::true_type{});
        else emit(std::false_type{});
        if constexpr (SCAN) {
            // sums over the wavefront (rotations inside the rows of 16 lanes, then the four rows through scalar registers),
            // one LDS word per wavefront and counter: no atomics, which a tile of few elements would feel
            unsigned c[2 * kScanCounters] = {cnt_re.sv_g, cnt_re.sz_g, cnt_re.sv_h, cnt_re.sz_h, cnt_re.bits,
                                             cnt_im.sv_g, cnt_im.sz_g, cnt_im.sv_h, cnt_im.sz_h, cnt_im.bits};
            unsigned mine = 0;
#pragma unroll
            for (int i = 0; i < 2 * kScanCounters; ++i) {
                const unsigned r = row_sum_step<1>(row_sum_step<2>(row_sum_step<4>(row_sum_step<8>(c[i]))));
                const unsigned total = (unsigned)__builtin_amdgcn_readlane((int)r, 0) + (unsigned)__builtin_amdgcn_readlane((int)r, 16) +
                                       (unsigned)__builtin_amdgcn_readlane((int)r, 32) + (unsigned)__builtin_amdgcn_readlane((int)r, 48);
                mine = lane == i ? total : mine;
            }
            if (lane < 2 * kScanCounters) scan_lds[wave * (2 * kScanCounters) + lane] = mine;
        }
    } else if constexpr (SCAN) {
        if (lane < 2 * kScanCounters) scan_lds[wave * (2 * kScanCounters) + lane] = 0u;
    }
    __syncthreads();
    if constexpr (SCAN) {
        if (tid < 2 * kScanCounters) {
            unsigned total = 0;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) total += scan_lds[w * (2 * kScanCounters) + tid];
            g.scan[(int64_t)tid * gridDim.x + blockIdx.x] = total;   // [counter][tile]
        }
    }

    // ---- the products
    // accumulator layout of the 16x16 MFMA: lane holds column (lane % 16); register u holds row 4 (lane / 16) + u
    const int lrow0 = rf * 16 + 4 * (lane >> 4), c8 = lane & 7;
    const bool is_im = (lane & 8) != 0;
    // patches of this wavefront that hold a column of C at all (wave-uniform)
    constexpr int CGS = WAVES / 2;   // wavefronts side by side over the fragments of B
    const int np = g.n > 8 * cg ? (g.n - 8 * cg - 1) / (8 * CGS) + 1 : 0;
    if (np == 0) return;

    v4acc acc[S];
    v4i a[S];
    double part[4];
    // iteration it: patch it / 2, pass it % 2 (0: Ar with T1, 1: Ai with T2)
    for (int it = 0; it < 2 * np; ++it) {
        const int pass = it & 1, f = cg + CGS * (it >> 1);
        const int nit = it + 1 < 2 * np ? it + 1 : 0;   // (after the last one the first one's fragments again, unused)
        const unsigned b_this = b_base(pass, f), b_next = b_base(nit & 1, cg + CGS * (nit >> 1));
        static_for<0, S>([&](auto pc) __attribute__((always_inline)) { a[decltype(pc)::value] = read_a(pass, decltype(pc)::value, 0); });
        __builtin_amdgcn_sched_barrier(0);
        // Group q of a step = the MFMAs of B fragment q with the A fragments S - 1 - q .. 0, each into the sum of
        // its anti-diagonal p + q: b[q] and a[S - 1 - q] have their last use of the step there and are fetched again,
        // in place, for the next step. Across the end of a walk only the B fragments are (they come from memory); the
        // A fragments are read from LDS after the fold, which needs their registers.
        static_for<0, KS>([&](auto sc) __attribute__((always_inline)) {
            constexpr int step = decltype(sc)::value;
            constexpr bool last_step = step == KS - 1;
            static_for<0, S>([&](auto qc) __attribute__((always_inline)) {
                constexpr int q = decltype(qc)::value, pmax = S - 1 - q;
                static_for<0, pmax + 1>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int p = pmax - decltype(ic)::value;
                    if constexpr (step == 0 && q == 0) acc[p] = mfma16(a[p], b[0], v4acc{0, 0, 0, 0});
                    else acc[p + q] = mfma16(a[p], b[q], acc[p + q]);
                });
                if constexpr (last_step) {
                    b[q] = load_b(b_next, q, 0);
                } else {
                    b[q] = load_b(b_this, q, step + 1);
                    a[pmax] = read_a(pass, pmax, step + 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        // G = the diagonals, least significant first: acc = RN(acc + S_e 2^(-7 (e + 2))) (the product of an integer
        // below 2^31 and a power of two is exact, so the fused operation rounds like the sum it stands for) ...
        // (the first term as a plain product: RN(0 + t) = t, and t is exact)
        // The four least significant diagonals, two at a time as one integer 2^7 S_(e-1) + S_e: diagonal e sums e + 1 slice
        // products of at most 64 KS positions and 127^2 each, so while ((S - 1) 2^7 + S) 64 KS 127^2 < 2^31 that integer
        // fits 32 bits; and the partial sums of those four terms are integers of less than 2^53 units of 2^(-7 (S + 1)),
        // so no rounding happens among them and any grouping gives the value the one-by-one sequence gives.
        constexpr bool MERGE = S >= 4 && ((long long)(S - 1) * 128 + S) * (64 * KS) * (127 * 127) < (1ll << 31);
        constexpr int E_FIRST = MERGE ? S - 5 : S - 2;   // the diagonals from here down are added one by one
        auto scale_of = [](int e) __attribute__((always_inline)) {
            return __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * (e + 2)) << 52);
        };
        double sum[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (MERGE) {
                const int low = acc[S - 2][u] * (1 << OZIMMU_SLICE_BITS) + acc[S - 1][u];
                const int next = acc[S - 4][u] * (1 << OZIMMU_SLICE_BITS) + acc[S - 3][u];
                sum[u] = fma((double)next, scale_of(S - 3), (double)low * scale_of(S - 1));
            } else {
                sum[u] = (double)acc[S - 1][u] * scale_of(S - 1);
            }
        }
#pragma unroll
        for (int e = E_FIRST; e >= 0; --e) {
            const double sc = scale_of(e);
#pragma unroll
            for (int u = 0; u < 4; ++u) sum[u] = fma((double)acc[e][u], sc, sum[u]);
        }
        // ... times 2^(EA_i + EB_j)
        const v4i ea = *reinterpret_cast<const v4i*>(ex + pass * kGateRows + lrow0);   // four consecutive rows
        const int eb = ex_gate[pass * (NFR * 16) + f * 16 + (lane & 15)];
#pragma unroll
        for (int u = 0; u < 4; ++u) sum[u] = ldexp(sum[u], ea[u] + eb);
        if (pass == 0) {
#pragma unroll
            for (int u = 0; u < 4; ++u) part[u] = sum[u];
        } else {
            // lanes 0..7 of every 16: re = G(Ar,Br) - G(Ai,Bi); lanes 8..15: im = G(Ar,Bi) + G(Ai,Br)
            // (the subtraction as the addition of the negated term: one flipped sign bit, no selection)
            const long long flip = is_im ? 0ll : (long long)(1ull << 63);
            double other[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                sum[u] = part[u] + __longlong_as_double(__double_as_longlong(sum[u]) ^ flip);
                // the other part of the same element, from the lane 8 further (rotation of the row of 16 lanes by 8)
                const unsigned long long x = (unsigned long long)__double_as_longlong(sum[u]);
                const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)x, 0x128, 0xf, 0xf, false);
                const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(x >> 32), 0x128, 0xf, 0xf, false);
                other[u] = __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
            }
            // the lane with the real parts stores rows 0 and 1 of its four, the one with the imaginary parts rows 2 and 3
            const int col = f * 8 + c8;
            const int64_t row0 = row_tile + lrow0 + (is_im ? 2 : 0);
            double* c = g.Cz + 2 * (row0 * g.ldcz + col);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                double2 z;
                z.x = is_im ? other[u + 2] : sum[u];
                z.y = is_im ? sum[u + 2] : other[u];
                if (row0 + u < g.m && col < g.n) *reinterpret_cast<double2*>(c + 2 * (int64_t)u * g.ldcz) = z;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The counters of all tiles ([counter][tile]) and of the gate's fragments (behind them, [4][nfr]) -> the bits the two
// planes of Z (planes 0, 1) and of B (planes 2, 3) lose with s and with s - 1 slices: out[plane * 16 + s - 1] and
// out[plane * 16 + s - 2], the layout of the slice-count sums. `out` may be mapped host memory. One workgroup.
__global__ __launch_bounds__(1024) void gate_scan_reduce_kernel(const unsigned* __restrict__ partials, int64_t tiles, int nfr,
                                                                int s, unsigned long long* __restrict__ out) {
    __shared__ unsigned long long sums[2 * kScanCounters + 4];
    if (threadIdx.x < 2 * kScanCounters + 4) sums[threadIdx.x] = 0ull;
    __syncthreads();
    // eighty loads in flight per thread (the words come from beyond the L2, written by other XCDs); a tile index past
    // the end reads the last tile and adds nothing
    unsigned long long mine[2 * kScanCounters] = {};
    constexpr int U = 8;
    for (int64_t base = threadIdx.x; base < tiles; base += 1024 * U) {
        unsigned v[U][2 * kScanCounters];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t t = base + 1024 * u, tc = t < tiles ? t : tiles - 1;
#pragma unroll
            for (int i = 0; i < 2 * kScanCounters; ++i) v[u][i] = partials[i * tiles + tc];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool in = base + 1024 * u < tiles;
#pragma unroll
            for (int i = 0; i < 2 * kScanCounters; ++i) mine[i] += in ? v[u][i] : 0u;
        }
    }
#pragma unroll
    for (int i = 0; i < 2 * kScanCounters; ++i) {
        unsigned long long v = mine[i];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
        if ((threadIdx.x & 63) == 0 && v) atomicAdd(&sums[i], v);
    }
    const unsigned* of_gate = partials + 2 * kScanCounters * tiles;
    if ((int)threadIdx.x < 4 * nfr) atomicAdd(&sums[2 * kScanCounters + threadIdx.x / nfr], (unsigned long long)of_gate[threadIdx.x]);
    __syncthreads();
    if (threadIdx.x < 2) {
        const unsigned long long* c = sums + threadIdx.x * kScanCounters;
        out[threadIdx.x * OZIMMU_MAX_SLICES + s - 1] = (c[0] - c[1] + c[4]) >> 1;
        if (s > 1) out[threadIdx.x * OZIMMU_MAX_SLICES + s - 2] = (c[2] - c[3] + c[4]) >> 1;
    } else if (threadIdx.x < 4) {
        const unsigned long long* c = sums + 2 * kScanCounters + 2 * (threadIdx.x - 2);
        out[threadIdx.x * OZIMMU_MAX_SLICES + s - 1] = c[0];
        if (s > 1) out[threadIdx.x * OZIMMU_MAX_SLICES + s - 2] = c[1];
    }
}

template <int S, int CLS, bool SCAN, int FEW>
hipError_t launch_gate(const GateArgs& g, hipStream_t st) {
    constexpr int lds = 2 * S * (1 << CLS) * 2 * kFragBytes + (2 * kGateRows + 2 * (8 << CLS) * 16 + 16 * 2 * kScanCounters) * (int)sizeof(int);
    static_assert(lds <= 160 * 1024 && (S > kBand || CLS == 2 || 2 * lds <= 160 * 1024) && (!FEW || S > kBand || 4 * lds <= 160 * 1024),
                  "the LDS of a compute unit: two workgroups of eight wavefronts (four of four) up to eight slices, else one workgroup");
    hipError_t e = allow_dynamic_lds<&gate_kernel<S, CLS, SCAN, FEW>>(lds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((g.m + kGateRows - 1) / kGateRows);
    gate_kernel<S, CLS, SCAN, FEW><<<dim3(grid), dim3(64 * gate_waves(CLS, FEW)), lds, st>>>(g);
    return hipGetLastError();
}
template <int S, int CLS>
hipError_t launch_gate(const GateArgs& g, hipStream_t st) {
    if constexpr (CLS == 0) {
        if (g.k <= 32 && g.n <= 32) return g.scan ? launch_gate<S, 0, true, 1>(g, st) : launch_gate<S, 0, false, 1>(g, st);
        return g.scan ? launch_gate<S, 0, true, 2>(g, st) : launch_gate<S, 0, false, 2>(g, st);
    } else {
        return g.scan ? launch_gate<S, CLS, true, 0>(g, st) : launch_gate<S, CLS, false, 0>(g, st);
    }
}

inline int gate_class(int64_t k, int64_t n) { return k > 128 || n > 128 ? 2 : k > 64 || n > 64 ? 1 : 0; }
inline int64_t gate_limit(int s) { return s <= kBand ? kGateMaxFew : kGateMax; }

}  // namespace

bool gate_product_applies(const double* Z, const double* B, const double* Cz, int64_t n, int64_t k, int s) {
    return s >= 1 && s <= OZIMMU_MAX_SLICES && n >= 1 && n <= gate_limit(s) && k >= 1 && k <= gate_limit(s) &&
           reinterpret_cast<uintptr_t>(Z) % 16 == 0 && reinterpret_cast<uintptr_t>(B) % 16 == 0 && reinterpret_cast<uintptr_t>(Cz) % 16 == 0;
}

size_t gate_scratch_bytes(int64_t n, int64_t k, int s) {
    if (s < 1 || s > OZIMMU_MAX_SLICES || n < 1 || n > gate_limit(s) || k < 1 || k > gate_limit(s)) return 0;
    const size_t nfr = (size_t)8 << gate_class(k, n), ks = (size_t)1 << gate_class(k, n);
    return 2 * nfr * 16 * sizeof(int32_t) + (size_t)2 * s * nfr * ks * kFragBytes;
}

size_t gate_scan_bytes(int64_t m) {
    return ((size_t)((m + kGateRows - 1) / kGateRows) * 2 * kScanCounters + 4 * (8 << 2)) * sizeof(unsigned);
}

hipError_t launch_gate_product(const double* Z, int64_t ldz, int64_t m, int64_t k, int64_t n, const double* B, int64_t ldb,
                               int s, void* scratch, double* Cz, int64_t ldcz, hipStream_t st, unsigned* scan_partials,
                               unsigned long long* scan_sums) {
    if (m <= 0) return hipSuccess;
    if (!gate_product_applies(Z, B, Cz, n, k, s)) return hipErrorInvalidValue;
    const int cls = gate_class(k, n), ks = 1 << cls, nfr = 8 << cls;
    int32_t* E = static_cast<int32_t*>(scratch);
    int8_t* T = reinterpret_cast<int8_t*>(E + 2 * nfr * 16);
    const unsigned split_threads = cls == 2 ? 512 : 256;   // a thread per word of four positions and column of the fragment
    const int64_t tiles = (m + kGateRows - 1) / kGateRows;
    unsigned* scan_gate = scan_partials ? scan_partials + 2 * kScanCounters * tiles : nullptr;
    if (s > 9) gate_split_kernel<true><<<dim3(nfr), dim3(split_threads), 0, st>>>(B, ldb, (int)k, (int)n, s, ks, nfr, T, E, scan_gate);
    else gate_split_kernel<false><<<dim3(nfr), dim3(split_threads), 0, st>>>(B, ldb, (int)k, (int)n, s, ks, nfr, T, E, scan_gate);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    GateArgs g{};
    g.Z = Z;
    g.ldz = ldz;
    g.m = m;
    g.k = (int)k;
    g.n = (int)n;
    g.T = T;
    g.E = E;
    g.Cz = Cz;
    g.ldcz = ldcz;
    g.scan = scan_partials;
    e = hipErrorInvalidValue;
    switch (s) {
#define OZ_CASE(S_) case S_: e = cls == 2 ? launch_gate<S_, 2>(g, st) : cls == 1 ? launch_gate<S_, 1>(g, st) : launch_gate<S_, 0>(g, st); break;
        OZ_CASE(1) OZ_CASE(2) OZ_CASE(3) OZ_CASE(4) OZ_CASE(5) OZ_CASE(6) OZ_CASE(7) OZ_CASE(8)
#undef OZ_CASE
#define OZ_CASE(S_) case S_: e = cls == 1 ? launch_gate<S_, 1>(g, st) : launch_gate<S_, 0>(g, st); break;
        OZ_CASE(9) OZ_CASE(10) OZ_CASE(11) OZ_CASE(12) OZ_CASE(13) OZ_CASE(14) OZ_CASE(15) OZ_CASE(16)
#undef OZ_CASE
    }
    if (e == hipSuccess && scan_partials) {
        gate_scan_reduce_kernel<<<dim3(1), dim3(1024), 0, st>>>(scan_partials, tiles, nfr, s, scan_sums);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace ozimmu
