// A gate on a state vector (Section 4.4): the complex product of a tall operand Z (m x k, the reshaped state,
// interleaved re/im) with a small one (B: k x n, the gate), k and n at most 128, up to eight slices, in ONE kernel
// that reads Z once and writes the result once.
//
// With so short an inner dimension the product is bound by the memory traffic of the state and by the vector
// work around the matrix cores, and splitting the state in a kernel of its own doubles that traffic (slices
// written, slices read back). Here a workgroup of four wavefronts takes 64 rows of Z (32 when k or n exceeds 64, so
// that the slices of a tile still take half the LDS of a compute unit at most): it finds the exponents of
// their real and imaginary parts and cuts both planes into slices (SplitInt, Section 3.1; the same bit operations as
// the splitter kernels) straight into LDS, in the fragment layout of the MFMA operand.
//
// The gate is split beforehand (gate_split_kernel) into two slice tensors whose 32-row fragments interleave its
// planes: fragment f of T1 holds columns 16 f .. 16 f + 15 of Br in rows 0..15 and the same columns of Bi in rows
// 16..31, T2 the other way round. A wavefront owns 32 rows and 16 complex columns at a time: Ar times a T1
// fragment gives G(Ar,Br) in lanes 0..15 (of each half) and G(Ar,Bi) in lanes 16..31, Ai times the T2 fragment
// gives G(Ai,Bi) and G(Ai,Br) in the same lanes, so that one rounded FP64 operation per lane forms
// re = G(Ar,Br) - G(Ai,Bi) or im = G(Ar,Bi) + G(Ai,Br); lanes 16 apart exchange half of their values and every lane
// stores whole (re, im) pairs. All anti-diagonals of a product are resident in registers, every product is folded
// in FP64 in the fixed order, least significant first, and scaled by 2^(EA_i + EB_j) (the summing-up step of the
// algorithm, Section 3.1). Two workgroups share a compute unit, so one loads, splits, folds or stores while the other
// multiplies.
//
// Unlike the large product kernel this one leaves register allocation to the compiler: at two wavefronts per SIMD
// and with no accumulation-register operand in inline assembly the MFMA results land in ordinary vector registers,
// where the FP64 fold reads them directly, and a product's first MFMA per diagonal takes the constant 0 as its
// addend instead of cleared registers.
#include "mfma_common.h"
#include "split_common.h"

namespace ozimmu {
namespace {

constexpr int kGateSmall = 64;    // k and n up to here: tiles of 64 rows, 2 x 2 wavefronts, four fragments of 16 columns of B
constexpr int kGateLarge = 128;   // beyond, up to here: tiles of 32 rows, 1 x 4 wavefronts, eight fragments, four steps

// ---------------------------------------------------------------------------- the gate -> T1, T2, exponents
// One workgroup per fragment f (16 columns of B). Thread (c, w) = (tid % 16, tid / 16) owns column 16 f + c and the
// four positions 4 w .. 4 w + 3 of k. T: tensor t at t * s * nfr * ks KiB, slice q at q * nfr * ks KiB, fragment
// (f, step) at (f ks + step) KiB. E: [t][f][32] exponents of the fragments' rows.
__global__ __launch_bounds__(512) void gate_split_kernel(const double* __restrict__ B, int64_t ldb, int k, int n, int s,
                                                         int ks, int nfr, int8_t* __restrict__ T, int32_t* __restrict__ E) {
    const int tid = threadIdx.x, r16 = tid & 15, w = tid >> 4, f = blockIdx.x, c = f * 16 + r16;
    const int words = blockDim.x >> 4;   // 16 (k <= 64) or 32
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
    __shared__ unsigned long long colmax[32][16][2];
    colmax[w][r16][0] = mx_re;
    colmax[w][r16][1] = mx_im;
    __syncthreads();
    for (int i = 0; i < words; ++i) {
        mx_re = colmax[i][r16][0] > mx_re ? colmax[i][r16][0] : mx_re;
        mx_im = colmax[i][r16][1] > mx_im ? colmax[i][r16][1] : mx_im;
    }
    const int e_re = exponent_of_max(mx_re), e_im = exponent_of_max(mx_im);
    if (w == 0) {
        E[f * 32 + r16] = e_re;
        E[f * 32 + 16 + r16] = e_im;
        E[nfr * 32 + f * 32 + r16] = e_im;
        E[nfr * 32 + f * 32 + 16 + r16] = e_re;
    }
    if (4 * w >= kSlab * ks) return;
    const int64_t slice = (int64_t)nfr * ks * kFragBytes, tensor = (int64_t)s * slice;
    Fixed xr[4], xi[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        xr[u] = to_fixed<false>(v[u].x, e_re);
        xi[u] = to_fixed<false>(v[u].y, e_im);
    }
    const SignMask sr = sign_mask(v[0].x, v[1].x, v[2].x, v[3].x);
    const SignMask si = sign_mask(v[0].y, v[1].y, v[2].y, v[3].y);
    const int l0 = 4 * w, step = l0 >> 5, ll = l0 & 31;
    // rows r16 (first plane of the fragment) and 16 + r16 (second): both have the same bit 3, hence the same swap of halves
    const int64_t lo = (int64_t)(f * ks + step) * kFragBytes + r16 * kSlab + ((((ll >> 4) ^ (r16 >> 3)) & 1) << 4) + (ll & 15);
    const int64_t hi = lo + 16 * kSlab;
#pragma unroll
    for (int p = 1; p <= kBand; ++p) {
        if (p <= s) {
            const uint32_t pr = packed_slice<false>(xr, sr, p), pi = packed_slice<false>(xi, si, p);
            int8_t* d = T + (p - 1) * slice;
            *reinterpret_cast<uint32_t*>(d + lo) = pr;
            *reinterpret_cast<uint32_t*>(d + hi) = pi;
            *reinterpret_cast<uint32_t*>(d + tensor + lo) = pi;
            *reinterpret_cast<uint32_t*>(d + tensor + hi) = pr;
        }
    }
}

// ---------------------------------------------------------------------------- the product
// S slices; KS steps of 32 positions of k; RF row fragments per tile: 2 (tiles of 64 rows, wavefronts 2 x 2, four
// fragments of B) with KS <= 2, or 1 (32 rows, wavefronts 1 x 4, eight fragments of B) with KS = 4.
template <int S, int KS, int RF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gate_kernel(const GateArgs g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int ROWS = 32 * RF;                 // rows of Z per workgroup
    constexpr int NFR = RF == 2 ? 4 : 8;          // fragments of 16 columns of B
    constexpr int SLICE = KS * RF * kFragBytes;   // one slice of one plane of the tile's rows: [step][row fragment]
    constexpr int PLANE = S * SLICE;
    // behind the two planes: exponents of the tile's rows, [plane][ROWS], then those of the gate's fragments, [tensor][NFR][32]
    int* ex = reinterpret_cast<int*>(lds + 2 * PLANE);
    int* ex_gate = ex + 2 * ROWS;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row_tile = (int64_t)blockIdx.x * ROWS;

    // ---- this wavefront's patches: rows 32 wm .. + 31 of the tile, complex columns 16 f .. 16 f + 15 for f = f0, f0 + 1
    const int wm = RF == 2 ? wave >> 1 : 0, f0 = RF == 2 ? 2 * (wave & 1) : 2 * wave;
    const int rr = lane & 31, half = lane >> 5;
    // MFMA operand: lane holds row (lane % 32), bytes 16 (lane / 32) .. + 16 of the 32-byte fragment row
    const unsigned rd_lane = (unsigned)(rr * 32 + ((half ^ ((rr >> 3) & 1)) << 4));
    const unsigned char* a_rd = lds + wm * kFragBytes + rd_lane;
    constexpr int BSLICE = NFR * KS * kFragBytes, TENSOR = S * BSLICE;
    auto read_a = [&](int plane, int p, int step) __attribute__((always_inline)) -> v4i {
        return *reinterpret_cast<const v4i*>(a_rd + plane * PLANE + p * SLICE + step * RF * kFragBytes);
    };
    auto load_b = [&](int t, int f, int q, int step) __attribute__((always_inline)) -> v4i {
        return *reinterpret_cast<const v4i*>(g.T + t * TENSOR + q * BSLICE + (f * KS + step) * kFragBytes + rd_lane);
    };
    // the gate's fragments of the first walk are requested before anything else: they are on their way while Z is split
    v4i b[S];
    static_for<0, S>([&](auto pc) __attribute__((always_inline)) { b[decltype(pc)::value] = load_b(0, f0, decltype(pc)::value, 0); });

    // ---- the rows of Z -> exponents and slices in LDS. Sixteen lanes work on a row; a lane owns W words of four
    // consecutive complex elements of it (words c16 and, with four steps, 16 + c16); a wavefront takes a quarter of the
    // tile's rows, four at a time: sixteen complex elements per lane in every shape.
    {
        constexpr int W = KS > 2 ? 2 : 1, G = ROWS / 16;   // words per lane and row; groups of four rows per wavefront
        static_assert(G * W == 4, "sixteen complex elements per lane");
        const int r4 = lane >> 4, c16 = lane & 15;
        for (int i = tid; i < 2 * NFR * 32; i += 256) ex_gate[i] = g.E[i];
        ulonglong2 v[G][W][4];
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const int64_t row = row_tile + wave * (4 * G) + gi * 4 + r4;
            const bool live = row < g.m;
            const ulonglong2* src = reinterpret_cast<const ulonglong2*>(g.Z) + (live ? row : 0) * g.ldz;
#pragma unroll
            for (int j = 0; j < W; ++j)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int l = (c16 + 16 * j) * 4 + u;
                    v[gi][j][u] = ulonglong2{0ull, 0ull};
                    if (live && l < g.k) v[gi][j][u] = src[l];
                }
        }
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            unsigned long long mx_re = 0, mx_im = 0;
#pragma unroll
            for (int j = 0; j < W; ++j)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned long long a = v[gi][j][u].x & kAbsMask, b2 = v[gi][j][u].y & kAbsMask;
                    mx_re = a > mx_re ? a : mx_re;
                    mx_im = b2 > mx_im ? b2 : mx_im;
                }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                const unsigned long long o = __shfl_xor(mx_re, off, 64), q = __shfl_xor(mx_im, off, 64);
                mx_re = o > mx_re ? o : mx_re;
                mx_im = q > mx_im ? q : mx_im;
            }
            const int e_re = exponent_of_max(mx_re), e_im = exponent_of_max(mx_im);
            const int lrow = wave * (4 * G) + gi * 4 + r4;
            if (c16 == 0) {
                ex[lrow] = e_re;
                ex[ROWS + lrow] = e_im;
            }
#pragma unroll
            for (int j = 0; j < W; ++j) {
                const int word = c16 + 16 * j;
                if (word * 4 < kSlab * KS) {   // (a one-step product has no second fragment to fill)
                    Fixed xr[4], xi[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        xr[u] = to_fixed<false>(v[gi][j][u].x, e_re);
                        xi[u] = to_fixed<false>(v[gi][j][u].y, e_im);
                    }
                    const SignMask sr = sign_mask(v[gi][j][0].x, v[gi][j][1].x, v[gi][j][2].x, v[gi][j][3].x);
                    const SignMask si = sign_mask(v[gi][j][0].y, v[gi][j][1].y, v[gi][j][2].y, v[gi][j][3].y);
                    // the fragment layout of the slice tensors: rows of 32 bytes, their two halves swapped in rows 8..15 and 24..31
                    const int fr = lrow & 31, l0 = (word & 7) * 4;
                    unsigned char* dst = lds + ((word >> 3) * RF + (lrow >> 5)) * kFragBytes + fr * kSlab +
                                         ((((l0 >> 4) ^ (fr >> 3)) & 1) << 4) + (l0 & 15);
                    static_for<1, S + 1>([&](auto pc) __attribute__((always_inline)) {
                        constexpr int p = decltype(pc)::value;
                        *reinterpret_cast<uint32_t*>(dst + (p - 1) * SLICE) = packed_slice<false>(xr, sr, p);
                        *reinterpret_cast<uint32_t*>(dst + PLANE + (p - 1) * SLICE) = packed_slice<false>(xi, si, p);
                    });
                }
                __builtin_amdgcn_sched_barrier(0);   // one word's temporaries at a time
            }
        }
    }
    __syncthreads();

    // ---- the products
    // accumulator layout of the 32x32 MFMA: lane holds column (lane % 32); register u holds row 8 (u / 4) + 4 (lane / 32) + u % 4
    const int lrow0 = wm * 32 + 4 * half;
    // patches of this wavefront that hold a column of C at all (wave-uniform)
    const int nf = g.n > (f0 + 1) * 16 ? 2 : g.n > f0 * 16 ? 1 : 0;
    if (nf == 0) return;

    v16i acc[S];
    v4i a[S];
    double part[16];
    // iteration it: patch it / 2, pass it % 2 (0: Ar with T1, 1: Ai with T2)
    for (int it = 0; it < 2 * nf; ++it) {
        const int pass = it & 1, f = f0 + (it >> 1);
        const int nit = it + 1 < 2 * nf ? it + 1 : 0;   // (after the last one the first one's fragments again, unused)
        const int npass = nit & 1, nfr = f0 + (nit >> 1);
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
                    if constexpr (step == 0 && q == 0) acc[p] = mfma(a[p], b[0], v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0});
                    else acc[p + q] = mfma(a[p], b[q], acc[p + q]);
                });
                if constexpr (last_step) {
                    b[q] = load_b(npass, nfr, q, 0);
                } else {
                    b[q] = load_b(pass, f, q, step + 1);
                    a[pmax] = read_a(pass, pmax, step + 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        // G = the diagonals, least significant first: acc = RN(acc + S_e 2^(-7 (e + 2))) (the product of an integer
        // below 2^31 and a power of two is exact, so the fused operation rounds like the sum it stands for) ...
        double sum[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) sum[u] = 0.0;
#pragma unroll
        for (int e = S - 1; e >= 0; --e) {
            const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * (e + 2)) << 52);
#pragma unroll
            for (int u = 0; u < 16; ++u) sum[u] = fma((double)acc[e][u], sc, sum[u]);
            __builtin_amdgcn_sched_barrier(0);   // one diagonal's temporaries at a time
        }
        // ... times 2^(EA_i + EB_j)
        const int* exa = ex + pass * ROWS + lrow0;
        const int eb = ex_gate[pass * (NFR * 32) + f * 32 + rr];
#pragma unroll
        for (int u4 = 0; u4 < 4; ++u4) {
            const v4i ea = *reinterpret_cast<const v4i*>(exa + 8 * u4);   // four consecutive rows
#pragma unroll
            for (int uu = 0; uu < 4; ++uu) sum[4 * u4 + uu] = ldexp(sum[4 * u4 + uu], ea[uu] + eb);
        }
        if (pass == 0) {
#pragma unroll
            for (int u = 0; u < 16; ++u) part[u] = sum[u];
        } else {
            // lanes 0..15 of each half: re = G(Ar,Br) - G(Ai,Bi); lanes 16..31: im = G(Ar,Bi) + G(Ai,Br)
            // (the subtraction as the addition of the negated term: one flipped sign bit, no selection)
            const bool is_im = (lane & 16) != 0;
            const long long flip = is_im ? 0ll : (long long)(1ull << 63);
#pragma unroll
            for (int u = 0; u < 16; ++u) sum[u] = part[u] + __longlong_as_double(__double_as_longlong(sum[u]) ^ flip);
            // Lanes 16 apart hold the two parts of the same elements. Swapping the upper 16 lanes of the register
            // with rows u against the lower 16 of the one with rows u + 8 leaves (re, im) of row u in the lanes
            // 0..15 and (re, im) of row u + 8 in the lanes 16..31: whole pairs to store, nothing to select.
            const int col = f * 16 + (rr & 15);
            const int64_t row0 = row_tile + lrow0 + (is_im ? 16 : 0);
            double* c = g.Cz + 2 * (row0 * g.ldcz + col);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const unsigned long long x = (unsigned long long)__double_as_longlong(sum[u]);
                const unsigned long long y = (unsigned long long)__double_as_longlong(sum[u + 8]);
                const auto lo = __builtin_amdgcn_permlane16_swap((unsigned)x, (unsigned)y, false, false);
                const auto hi = __builtin_amdgcn_permlane16_swap((unsigned)(x >> 32), (unsigned)(y >> 32), false, false);
                const int dr = 8 * (u >> 2) + (u & 3);   // (rows 16 .. of the patch for the upper lanes: in row0)
                double2 z;
                z.x = __longlong_as_double((long long)(((unsigned long long)hi[0] << 32) | lo[0]));
                z.y = __longlong_as_double((long long)(((unsigned long long)hi[1] << 32) | lo[1]));
                if (row0 + dr < g.m && col < g.n) *reinterpret_cast<double2*>(c + 2 * (int64_t)dr * g.ldcz) = z;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int S, int KS, int RF>
hipError_t launch_gate(const GateArgs& g, hipStream_t st) {
    constexpr int rows = 32 * RF, nfr = RF == 2 ? 4 : 8;
    constexpr int lds = 2 * S * KS * RF * kFragBytes + (2 * rows + 2 * nfr * 32) * (int)sizeof(int);
    static_assert(2 * lds <= 160 * 1024, "two workgroups per compute unit");
    hipError_t e = allow_dynamic_lds<&gate_kernel<S, KS, RF>>(lds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((g.m + rows - 1) / rows);
    gate_kernel<S, KS, RF><<<dim3(grid), dim3(256), lds, st>>>(g);
    return hipGetLastError();
}

// steps and fragments of a gate shape
inline int gate_steps(int64_t k, int64_t n) { return k > kGateSmall || n > kGateSmall ? 4 : k > kSlab ? 2 : 1; }
inline int gate_fragments(int64_t k, int64_t n) { return k > kGateSmall || n > kGateSmall ? 8 : 4; }

}  // namespace

bool gate_product_applies(const double* Z, const double* B, const double* Cz, int64_t n, int64_t k, int s) {
    return n >= 1 && n <= kGateLarge && k >= 1 && k <= kGateLarge && s <= kBand && reinterpret_cast<uintptr_t>(Z) % 16 == 0 &&
           reinterpret_cast<uintptr_t>(B) % 16 == 0 && reinterpret_cast<uintptr_t>(Cz) % 16 == 0;
}

size_t gate_scratch_bytes(int64_t n, int64_t k, int s) {
    if (n < 1 || n > kGateLarge || k < 1 || k > kGateLarge || s > kBand) return 0;
    const size_t nfr = (size_t)gate_fragments(k, n);
    return 2 * nfr * 32 * sizeof(int32_t) + (size_t)2 * s * nfr * gate_steps(k, n) * kFragBytes;
}

hipError_t launch_gate_product(const double* Z, int64_t ldz, int64_t m, int64_t k, int64_t n, const double* B, int64_t ldb,
                               int s, void* scratch, double* Cz, int64_t ldcz, hipStream_t st) {
    if (m <= 0) return hipSuccess;
    if (!gate_product_applies(Z, B, Cz, n, k, s) || s < 1) return hipErrorInvalidValue;
    const int ks = gate_steps(k, n), nfr = gate_fragments(k, n);
    int32_t* E = static_cast<int32_t*>(scratch);
    int8_t* T = reinterpret_cast<int8_t*>(E + 2 * nfr * 32);
    gate_split_kernel<<<dim3(nfr), dim3(ks == 4 ? 512 : 256), 0, st>>>(B, ldb, (int)k, (int)n, s, ks, nfr, T, E);
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
    switch (s) {
#define OZ_CASE(S_) case S_: return ks == 4 ? launch_gate<S_, 4, 1>(g, st) : ks == 2 ? launch_gate<S_, 2, 2>(g, st) : launch_gate<S_, 1, 2>(g, st);
        OZ_CASE(1) OZ_CASE(2) OZ_CASE(3) OZ_CASE(4) OZ_CASE(5) OZ_CASE(6) OZ_CASE(7) OZ_CASE(8)
#undef OZ_CASE
    }
    return hipErrorInvalidValue;
}

}  // namespace ozimmu
