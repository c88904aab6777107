// SplitInt (Section 3.1, splitting algorithm for integer arithmetic) on gfx950.
//
// One power-of-two exponent per row of M = A or B^T (exponent step of SplitInt), then every element
// is cut by bit operations (Section 4.1) into signed 7-bit chunks of its significand, placed
// relative to the row exponent (its slice-extraction loop). Output: padded INT8 slice tensors, zero outside the
// matrix, in the fragment layout that the slice-product kernel copies linearly into LDS (fragments of
// 32 rows x 32 bytes, the MFMA operand of one wavefront; the layout is defined with the C ABI).
//
// Both kernels are HBM-bound: 8 B read per element (16 B for B, whose column maxima need a
// pass of their own) and num_slices bytes written.
#include "ozimmu_internal.h"
#include "split_common.h"

namespace ozimmu {
namespace {

// Byte offset, inside one slice, of the 4-byte word that holds positions l0 .. l0+3 (l0 % 4 == 0)
// of padded row r: fragments of 32 rows x 32 bytes, the two 16-byte halves of a row swapped in
// rows 8..15 and 24..31 of a fragment.
__device__ __forceinline__ int64_t word_offset(int64_t r, int64_t l0, int64_t k_pad) {
    const int64_t rr = r & (kFragRows - 1);
    const int64_t h = (l0 & (kSlab - 1)) >> 4;
    return ((r / kFragRows) * (k_pad / kSlab) + l0 / kSlab) * kFragBytes + rr * kSlab + ((h ^ ((rr >> 3) & 1)) << 4) + (l0 & 15);
}

// ------------------------------------------------------------------------------ rows of A
// One workgroup per four consecutive padded rows: a quarter of a wavefront (16 lanes) works on a row,
// a thread owns words of four consecutive elements (one 32-bit store per slice), a wave-wide load
// covers 64 consecutive elements of each of the four rows, and a wave-wide store fills, per 32
// positions of k, the 128 contiguous bytes that four consecutive rows occupy in a fragment: full
// lines both ways. Pass 1: maximum of the |x| bit patterns (monotone in |x|), shuffles within the
// 16 lanes, then LDS across the wavefronts. Pass 2: emission. Rows of up to 8192 elements stay in
// registers between the two passes (CACHED), so A is read from memory once; longer rows are read twice.
constexpr int kRowCacheWords = 8;   // words of 4 elements per thread that fit the register cache
constexpr int kRowGroup = 4;        // rows per workgroup
constexpr int kRowWavesMax = 16;

template <bool VEC>   // VEC: unit stride and 16-byte aligned rows, two 16-byte loads per word
__device__ __forceinline__ void load_word(const unsigned long long* src, int64_t l0, int64_t k, int inc,
                                          unsigned long long (&b)[4]) {
    if (VEC && l0 + 4 <= k) {
        const ulonglong2 v0 = *reinterpret_cast<const ulonglong2*>(src + l0);
        const ulonglong2 v1 = *reinterpret_cast<const ulonglong2*>(src + l0 + 2);
        b[0] = v0.x; b[1] = v0.y; b[2] = v1.x; b[3] = v1.y;
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) b[u] = (l0 + u < k) ? src[(l0 + u) * inc] : 0ull;
    }
}

template <bool WIDE>
__device__ __forceinline__ void emit_word(const unsigned long long (&b)[4], int E, int s, int8_t* dst,
                                          int64_t slice_stride, unsigned long long flip) {
    Fixed x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) x[u] = to_fixed<WIDE>(b[u], E);
    const SignMask sm = sign_mask(b[0] ^ flip, b[1] ^ flip, b[2] ^ flip, b[3] ^ flip);
#pragma unroll
    for (int p = 1; p <= (WIDE ? OZIMMU_MAX_SLICES : 9); ++p)   // unrolled: p is a constant in field()
        if (p <= s) *reinterpret_cast<uint32_t*>(dst + (int64_t)(p - 1) * slice_stride) = packed_slice<WIDE>(x, sm, p);
}

template <bool WIDE, bool CACHED, bool VEC, bool SCAN>   // SCAN: also count for the slice-count check (scan.slots is set)
__global__ __launch_bounds__(64 * kRowWavesMax) void split_rows_kernel(const double* __restrict__ A, int64_t lda,
                                                                       int inc, int m, int64_t k, int s,
                                                                       int8_t* __restrict__ S, int64_t m_pad,
                                                                       int64_t k_pad, int32_t* __restrict__ Eout,
                                                                       unsigned long long flip,    // sign bit, or 0: slices of -A
                                                                       ScanTarget scan) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int r4 = lane >> 4, c16 = lane & 15;
    const int row = blockIdx.x * kRowGroup + r4;
    const bool live = row < m;                       // padding rows: zeros in every slice
    __shared__ unsigned scan_lds[SCAN ? kScanCounters : 1];
    if (SCAN && tid < kScanCounters) scan_lds[tid] = 0u;   // (the barrier after the maxima publishes it)
    ScanCount cnt = {};
    const int64_t slice_stride = m_pad * k_pad;
    // chunk c of a row = its elements [64 c, 64 c + 64); the wavefronts take the chunks round-robin
    const int64_t chunks = (k_pad + 63) / 64;
    const unsigned long long* src = reinterpret_cast<const unsigned long long*>(A) + (int64_t)(live ? row : 0) * lda;
    const int64_t k_live = live ? k : 0;             // a padding row reads nothing

    unsigned long long cache[CACHED ? kRowCacheWords : 1][4];
    unsigned long long mx = 0;
    if (CACHED) {
#pragma unroll
        for (int j = 0; j < kRowCacheWords; ++j) {
            const int64_t l0 = ((int64_t)(wave + nwaves * j) * 16 + c16) * 4;
            if (l0 < k_live) load_word<VEC>(src, l0, k_live, inc, cache[j]);
            else cache[j][0] = cache[j][1] = cache[j][2] = cache[j][3] = 0ull;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned long long a = cache[j][u] & kAbsMask;
                mx = a > mx ? a : mx;
            }
        }
    } else {
        for (int64_t c = wave; c < chunks; c += nwaves) {
            const int64_t l0 = (c * 16 + c16) * 4;
            unsigned long long b[4];
            load_word<VEC>(src, l0, k_live, inc, b);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned long long a = b[u] & kAbsMask;
                mx = a > mx ? a : mx;
            }
        }
    }
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(mx, off, 64);
        mx = o > mx ? o : mx;
    }
    __shared__ unsigned long long wmax[kRowWavesMax][kRowGroup];
    if (c16 == 0) wmax[wave][r4] = mx;
    __syncthreads();
    mx = wmax[0][r4];
    for (int w = 1; w < nwaves; ++w) mx = wmax[w][r4] > mx ? wmax[w][r4] : mx;
    const int E = exponent_of_max(mx);
    if (live && wave == 0 && c16 == 0) Eout[row] = E;

    if (CACHED) {
#pragma unroll
        for (int j = 0; j < kRowCacheWords; ++j) {
            const int64_t l0 = ((int64_t)(wave + nwaves * j) * 16 + c16) * 4;
            if (l0 < k_pad) emit_word<WIDE>(cache[j], E, s, S + word_offset(row, l0, k_pad), slice_stride, flip);
            if constexpr (SCAN) scan_count4(cnt, cache[j], E, scan.edge_g, scan.edge_h);
        }
    } else {
        for (int64_t c = wave; c < chunks; c += nwaves) {
            const int64_t l0 = (c * 16 + c16) * 4;
            if (l0 < k_pad) {
                unsigned long long b[4];
                load_word<VEC>(src, l0, k_live, inc, b);
                emit_word<WIDE>(b, E, s, S + word_offset(row, l0, k_pad), slice_stride, flip);
                if constexpr (SCAN) scan_count4(cnt, b, E, scan.edge_g, scan.edge_h);
            }
        }
    }
    if constexpr (SCAN) scan_flush(cnt, scan_lds, scan);
}

// Rows of an interleaved complex operand, both planes in one pass: the same mapping as above, a thread's
// word being four consecutive complex elements (four 16-byte loads), whose real parts go to one set of
// slices and exponents and whose imaginary parts to the other. Read once (a pass per plane with element
// stride 2 fetches every line twice). Rows of up to 4096 elements (they stay in registers); longer
// ones take the two strided passes.
constexpr int kZRowCacheWords = 4;
template <bool WIDE, bool SCAN>
__global__ __launch_bounds__(64 * kRowWavesMax) void split_rows_complex_kernel(
    const double* __restrict__ Z, int64_t ldz, int m, int64_t k, int s, int8_t* __restrict__ S_re,
    int8_t* __restrict__ S_im, int64_t m_pad, int64_t k_pad, int32_t* __restrict__ E_re, int32_t* __restrict__ E_im,
    unsigned long long flip_re, unsigned long long flip_im, ScanTarget scan) {   // scan: the real plane's counters, the imaginary one's five behind
    __shared__ unsigned scan_lds[2][SCAN ? kScanCounters : 1];
    if (SCAN && threadIdx.x < 2 * kScanCounters) (&scan_lds[0][0])[threadIdx.x] = 0u;   // (published by the barrier after the maxima)
    ScanCount cnt_re = {}, cnt_im = {};
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int r4 = lane >> 4, c16 = lane & 15;
    const int row = blockIdx.x * kRowGroup + r4;
    const bool live = row < m;
    const int64_t slice_stride = m_pad * k_pad;
    const ulonglong2* src = reinterpret_cast<const ulonglong2*>(Z) + (int64_t)(live ? row : 0) * ldz;
    const int64_t k_live = live ? k : 0;

    unsigned long long re[kZRowCacheWords][4], im[kZRowCacheWords][4];
    unsigned long long mx_re = 0, mx_im = 0;
#pragma unroll
    for (int j = 0; j < kZRowCacheWords; ++j) {
        const int64_t l0 = ((int64_t)(wave + nwaves * j) * 16 + c16) * 4;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            ulonglong2 v = {0ull, 0ull};
            if (l0 + u < k_live) v = src[l0 + u];
            re[j][u] = v.x;
            im[j][u] = v.y;
            const unsigned long long a = v.x & kAbsMask, b = v.y & kAbsMask;
            mx_re = a > mx_re ? a : mx_re;
            mx_im = b > mx_im ? b : mx_im;
        }
    }
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(mx_re, off, 64), q = __shfl_xor(mx_im, off, 64);
        mx_re = o > mx_re ? o : mx_re;
        mx_im = q > mx_im ? q : mx_im;
    }
    __shared__ unsigned long long wmax[kRowWavesMax][kRowGroup][2];
    if (c16 == 0) {
        wmax[wave][r4][0] = mx_re;
        wmax[wave][r4][1] = mx_im;
    }
    __syncthreads();
    mx_re = wmax[0][r4][0];
    mx_im = wmax[0][r4][1];
    for (int w = 1; w < nwaves; ++w) {
        mx_re = wmax[w][r4][0] > mx_re ? wmax[w][r4][0] : mx_re;
        mx_im = wmax[w][r4][1] > mx_im ? wmax[w][r4][1] : mx_im;
    }
    const int e_re = exponent_of_max(mx_re), e_im = exponent_of_max(mx_im);
    if (live && wave == 0 && c16 == 0) {
        E_re[row] = e_re;
        E_im[row] = e_im;
    }
#pragma unroll
    for (int j = 0; j < kZRowCacheWords; ++j) {
        const int64_t l0 = ((int64_t)(wave + nwaves * j) * 16 + c16) * 4;
        if (l0 < k_pad) {
            const int64_t off = word_offset(row, l0, k_pad);
            emit_word<WIDE>(re[j], e_re, s, S_re + off, slice_stride, flip_re);
            emit_word<WIDE>(im[j], e_im, s, S_im + off, slice_stride, flip_im);
        }
        if constexpr (SCAN) {
            scan_count4(cnt_re, re[j], e_re, scan.edge_g, scan.edge_h);
            scan_count4(cnt_im, im[j], e_im, scan.edge_g, scan.edge_h);
        }
    }
    if constexpr (SCAN) {
        scan_flush(cnt_re, scan_lds[0], scan);
        ScanTarget second = scan;
        second.slots += kScanCounters;
        scan_flush(cnt_im, scan_lds[1], second);
    }
}

// ------------------------------------------------------------------------------ columns of B
__global__ __launch_bounds__(256) void fill_u64_kernel(unsigned long long* p, int64_t n,
                                                       unsigned long long v) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// The column kernels take a second plane of the same operand in the same launch (the imaginary part of an
// interleaved complex operand): workgroups with blockIdx.z = 1 work on it, its pointers at these distances
// from the first plane's.
struct SecondPlane {
    int64_t b;        // elements of B
    int64_t colmax;   // entries
    int64_t slices;   // bytes
    int64_t e;        // entries
    unsigned long long flip;   // its sign flip (0 or the sign bit)
    int64_t sums;     // entries (slice-count scan)
};

// Column maxima of |B|: a lane owns a column (loads are contiguous across lanes), a workgroup
// owns a band of rows, bands are combined with a 64-bit atomic maximum on the bit patterns.
constexpr int kColBand = 256;   // rows per band when the matrix is tall enough to fill the chip
__global__ __launch_bounds__(256) void col_max_kernel(const double* __restrict__ B, int64_t ldb,
                                                      int inc, int64_t k, int64_t n, int band,
                                                      unsigned long long* __restrict__ colmax, SecondPlane second = SecondPlane{}) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    if (blockIdx.z) {
        B += second.b;
        colmax += second.colmax;
    }
    const int64_t l0 = (int64_t)blockIdx.y * band;
    const int64_t l1 = l0 + band < k ? l0 + band : k;
    const unsigned long long* src = reinterpret_cast<const unsigned long long*>(B);
    unsigned long long mx = 0;
    for (int64_t l = l0; l < l1; ++l) {
        unsigned long long b = src[(l * ldb + j) * inc] & kAbsMask;
        mx = b > mx ? b : mx;
    }
    if (mx) atomicMax(&colmax[j], mx);
}

__global__ __launch_bounds__(256) void col_exponent_kernel(const unsigned long long* __restrict__ colmax,
                                                           int64_t n, int32_t* __restrict__ E) {
    int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j < n) E[j] = exponent_of_max(colmax[j]);
}

// Slice emission for B^T: a workgroup takes a 64 (l) x 64 (j) tile of B. Lane (jj, lg) reads
// 16 elements of column jj (contiguous across lanes for each l), packs four consecutive l per
// slice into one word and transposes through LDS so that the global stores run along l. The
// tile is kept this small for the registers: 16 fixed-point fractions per thread leave room for
// five or six wavefronts per SIMD, and it is occupancy that keeps the loads of this pass in flight.
constexpr int kColTileL = 64, kColTileJ = 64;
constexpr int kColWords = kColTileL / 4 / 4;   // words of four consecutive l per thread
constexpr int kColGroup = 4;   // slices transposed through LDS at a time
constexpr int kColLdsStride = kColTileL / 4 + 1;  // words per LDS row (+1: conflict-free columns)
template <bool WIDE, bool SCAN>
__global__ __launch_bounds__(256) void split_cols_kernel(const double* __restrict__ B, int64_t ldb,
                                                         int inc, int64_t k, int64_t n, int s,
                                                         int8_t* __restrict__ S, int64_t n_pad,
                                                         int64_t k_pad,
                                                         const unsigned long long* __restrict__ colmax,
                                                         int32_t* __restrict__ Eout, int j_tiles,
                                                         unsigned long long flip,    // sign bit, or 0: slices of -B
                                                         SecondPlane second = SecondPlane{}, ScanTarget scan = ScanTarget{}) {
    __shared__ uint32_t tile[kColGroup][kColTileJ][kColLdsStride];
    __shared__ unsigned scan_lds[SCAN ? kScanCounters : 1];
    if (SCAN && threadIdx.x < kScanCounters) scan_lds[threadIdx.x] = 0u;   // (published by the barriers of the write-out)
    ScanCount cnt = {};
    if (blockIdx.z) {
        B += second.b;
        colmax += second.colmax;
        S += second.slices;
        Eout += second.e;
        flip = second.flip;
        if (SCAN) scan.slots += kScanCounters;
    }
    const int tid = threadIdx.x;
    const int jj = tid & 63, lg = tid >> 6;
    const int64_t jt = blockIdx.x % j_tiles, lt = blockIdx.x / j_tiles;
    const int64_t j = jt * kColTileJ + jj;
    const int64_t lbase = lt * kColTileL;
    const int64_t slice_stride = n_pad * k_pad;
    const unsigned long long* src = reinterpret_cast<const unsigned long long*>(B);
    const int E = (j < n) ? exponent_of_max(colmax[j]) : 0;
    if (lt == 0 && lg == 0 && j < n) Eout[j] = E;

    Fixed x[kColWords][4];
    SignMask sm[kColWords];
#pragma unroll
    for (int u4 = 0; u4 < kColWords; ++u4) {
        unsigned long long b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t l = lbase + lg * (4 * kColWords) + u4 * 4 + u;
            b[u] = (j < n && l < k) ? src[(l * ldb + j) * inc] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u4][u] = to_fixed<WIDE>(b[u], E);
        sm[u4] = sign_mask(b[0] ^ flip, b[1] ^ flip, b[2] ^ flip, b[3] ^ flip);
        if constexpr (SCAN) scan_count4(cnt, b, E, scan.edge_g, scan.edge_h);
    }
#pragma unroll
    for (int p0 = 1; p0 <= (WIDE ? OZIMMU_MAX_SLICES : 9); p0 += kColGroup) {   // unrolled: slice numbers are constants
        if (p0 > s) continue;   // uniform
        const int np = (s - p0 + 1) < kColGroup ? (s - p0 + 1) : kColGroup;
#pragma unroll
        for (int pp = 0; pp < kColGroup; ++pp) {
            if (pp < np && p0 + pp <= OZIMMU_MAX_SLICES) {
#pragma unroll
                for (int u4 = 0; u4 < kColWords; ++u4) tile[pp][jj][lg * kColWords + u4] = packed_slice<WIDE>(x[u4], sm[u4], p0 + pp);
            }
        }
        __syncthreads();
        // Write-out: per slice the tile is 2 row groups x 2 slabs = 4 fragments of 1 KiB, each
        // contiguous in the slice tensor: consecutive lanes store consecutive 16-byte units.
        for (int pp = 0; pp < np; ++pp) {
            int8_t* dst = S + (int64_t)(p0 + pp - 1) * slice_stride;
            const int f = tid >> 6;                 // fragment inside the tile
            const int ks = f >> 1, rg = f & 1;      // its slab and its row group
            const int pos = tid & 63;               // 16-byte unit inside the fragment
            const int rr = pos >> 1;                // fragment row
            const int h = (pos & 1) ^ ((rr >> 3) & 1);   // which half of the row's 32 positions is stored there
            const int r = rg * kFragRows + rr;      // row inside the tile (a column of B)
            const int w0 = ks * 8 + h * 4;          // first word of that half in the LDS row
            uint4 v = {tile[pp][r][w0], tile[pp][r][w0 + 1], tile[pp][r][w0 + 2], tile[pp][r][w0 + 3]};
            const int64_t slab = lbase / kSlab + ks;
            if (slab < k_pad / kSlab) {
                const int64_t off = ((jt * 2 + rg) * (k_pad / kSlab) + slab) * kFragBytes + pos * 16;
                *reinterpret_cast<uint4*>(dst + off) = v;
            }
        }
        __syncthreads();
    }
    if constexpr (SCAN) scan_flush(cnt, scan_lds, scan);
}

// The slots of a counting splitter -> the bits each of the operand's planes loses with s and with s - 1 slices:
// out[plane * 16 + s - 1] and out[plane * 16 + s - 2] (the layout of the slice-count sums; `out` may be mapped host
// memory). One workgroup of 256 threads.
__global__ __launch_bounds__(256) void scan_reduce_kernel(const unsigned long long* __restrict__ slots, int nc, int s,
                                                          unsigned long long* __restrict__ out) {
    __shared__ unsigned long long sums[2 * kScanCounters];
    if (threadIdx.x < 2 * kScanCounters) sums[threadIdx.x] = 0ull;
    __syncthreads();
    for (int i = 0; i < nc; ++i) {
        unsigned long long v = 0;
        for (int t = threadIdx.x; t < kScanSlots; t += 256) v += slots[(size_t)t * nc + i];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
        if ((threadIdx.x & 63) == 0 && v) atomicAdd(&sums[i], v);
    }
    __syncthreads();
    if ((int)threadIdx.x < nc / kScanCounters) {
        const unsigned long long* c = sums + threadIdx.x * kScanCounters;
        out[threadIdx.x * OZIMMU_MAX_SLICES + s - 1] = (c[0] - c[1] + c[4]) >> 1;
        if (s > 1) out[threadIdx.x * OZIMMU_MAX_SLICES + s - 2] = (c[2] - c[3] + c[4]) >> 1;
    }
}

// ------------------------------------------------------------------------------ slice-count scan
// Automatic choice of the number of slices (Section 4.4, "INT8-AUTO"): every element is
// inspected and, for each candidate s = 1 .. 16, the mantissa bits that s slices would cut off
// are added up. An element whose leading bit sits z places below the binary point of
// |x| 2^(-E) and that stores L significant bits (53, fewer for a subnormal) has its lowest bit
// at position v = z + L; s slices keep positions 1 .. 7 s, so it loses min(L, max(0, v - 7 s))
// bits. The host divides the sums by the element counts and picks the smallest s whose average
// is within the threshold.
//
// With z clamped to [0, 112] (an element that far down loses all L bits for every s <= 16 either
// way) and v = z + L <= 165, lost(s) = max(0, v - 7 s) - max(0, z - 7 s) = (|v - 7 s| - |z - 7 s| + L) / 2.
// v and z of four elements fit the four bytes of a register, so one v_sad_u8 per candidate adds
// |v - 7 s| of all four to a counter (and one more |z - 7 s|): 32 instructions per four elements
// for the 16 candidates. The halving is done once, when the counters are flushed.
struct LossAcc {
    uint32_t sad_v[OZIMMU_MAX_SLICES];   // sum of |v - 7 s|
    uint32_t sad_z[OZIMMU_MAX_SLICES];   // sum of |z - 7 s|
    uint32_t bits;                       // sum of L
};
__device__ __forceinline__ void loss_clear(LossAcc& a) {
#pragma unroll
    for (int s = 0; s < OZIMMU_MAX_SLICES; ++s) a.sad_v[s] = a.sad_z[s] = 0u;
    a.bits = 0u;
}
// Four elements that share the exponent E (zeros count nothing: v = z = L = 0).
__device__ __forceinline__ void loss_add4(LossAcc& a, const unsigned long long b[4], int E) {
    uint32_t pz = 0, pl = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        uint32_t z, L;
        loss_position(b[u], E, z, L);
        pz |= z << (8 * u);
        pl |= L << (8 * u);
    }
    const uint32_t pv = pz + pl;          // bytewise: no byte exceeds 165
    a.bits = __builtin_amdgcn_sad_u8(pl, 0u, a.bits);
#pragma unroll
    for (int s = 1; s <= OZIMMU_MAX_SLICES; ++s) {
        const uint32_t edge = 0x01010101u * (uint32_t)(OZIMMU_SLICE_BITS * s);
        a.sad_v[s - 1] = __builtin_amdgcn_sad_u8(pv, edge, a.sad_v[s - 1]);
        a.sad_z[s - 1] = __builtin_amdgcn_sad_u8(pz, edge, a.sad_z[s - 1]);
    }
}
// Workgroup-wide sum of the per-thread counters (64-bit from here on: a workgroup may have scanned
// many rows), then one 64-bit atomic per slice count.
__device__ __forceinline__ void loss_flush(const LossAcc& a, unsigned long long* lds16, unsigned long long* sums) {
    if (threadIdx.x < OZIMMU_MAX_SLICES) lds16[threadIdx.x] = 0ull;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < OZIMMU_MAX_SLICES; ++s) {
        unsigned long long v = (a.sad_v[s] - a.sad_z[s] + a.bits) >> 1;   // this thread's lost bits: exact, no wrap
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
        if ((threadIdx.x & 63) == 0 && v) atomicAdd(&lds16[s], v);
    }
    __syncthreads();
    if (threadIdx.x < OZIMMU_MAX_SLICES && lds16[threadIdx.x]) atomicAdd(&sums[threadIdx.x], lds16[threadIdx.x]);
}

// Rows of A: a group of ROWS rows at a time, 64 / ROWS lanes of a wavefront on each (four rows for short
// ones as in the row splitter, one for long ones), `wpg` wavefronts per group (1, 2 or 4: rows of up to
// 8192 elements wait in registers between the maximum and the scan). A workgroup is four wavefronts,
// that is 4 / wpg groups side by side; it walks many of them and flushes its counters once at the end:
// the sums are 16 atomics on 16 addresses per flush, and thousands of flushes serialise on them.
constexpr int kLossWavesMax = 4;
template <int ROWS, bool CACHED, bool VEC>
__global__ __launch_bounds__(64 * kLossWavesMax) void loss_rows_kernel(const double* __restrict__ A, int64_t lda, int inc,
                                                                       int64_t m, int64_t k, int wpg,
                                                                       unsigned long long* __restrict__ sums) {
    constexpr int LPR = 64 / ROWS;   // lanes per row
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int sub = wave / wpg, wi = wave % wpg, side = kLossWavesMax / wpg;   // group inside the workgroup, wavefront inside the group
    const int rsub = lane / LPR, c = lane % LPR;
    const int64_t chunks = (k + 4 * LPR - 1) / (4 * LPR);
    __shared__ unsigned long long wmax[kLossWavesMax][ROWS];
    __shared__ unsigned long long lds16[OZIMMU_MAX_SLICES];
    LossAcc acc;
    loss_clear(acc);
    for (int64_t first = (int64_t)blockIdx.x * side; first * ROWS < m; first += (int64_t)gridDim.x * side) {
        const int64_t row = (first + sub) * ROWS + rsub;
        const bool live = row < m;
        const unsigned long long* src = reinterpret_cast<const unsigned long long*>(A) + (live ? row : 0) * lda;
        const int64_t k_live = live ? k : 0;
        unsigned long long cache[CACHED ? kRowCacheWords : 1][4];
        unsigned long long mx = 0;
        if (CACHED) {
#pragma unroll
            for (int j = 0; j < kRowCacheWords; ++j) {
                const int64_t l0 = ((int64_t)(wi + wpg * j) * LPR + c) * 4;
                if (l0 < k_live) load_word<VEC>(src, l0, k_live, inc, cache[j]);
                else cache[j][0] = cache[j][1] = cache[j][2] = cache[j][3] = 0ull;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned long long a = cache[j][u] & kAbsMask;
                    mx = a > mx ? a : mx;
                }
            }
        } else {
            for (int64_t ch = wi; ch < chunks; ch += wpg) {
                unsigned long long b[4];
                load_word<VEC>(src, (ch * LPR + c) * 4, k_live, inc, b);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned long long a = b[u] & kAbsMask;
                    mx = a > mx ? a : mx;
                }
            }
        }
#pragma unroll
        for (int off = LPR / 2; off >= 1; off >>= 1) {
            const unsigned long long o = __shfl_xor(mx, off, 64);
            mx = o > mx ? o : mx;
        }
        __syncthreads();   // the maxima of the previous groups have been read by everybody
        if (c == 0) wmax[wave][rsub] = mx;
        __syncthreads();
        mx = wmax[sub * wpg][rsub];
        for (int w = 1; w < wpg; ++w) mx = wmax[sub * wpg + w][rsub] > mx ? wmax[sub * wpg + w][rsub] : mx;
        const int E = exponent_of_max(mx);
        if (CACHED) {
#pragma unroll
            for (int j = 0; j < kRowCacheWords; ++j)   // short rows: whole words beyond the row are skipped (same for all lanes)
                if (ROWS == 1 || (int64_t)(wi + wpg * j) * LPR * 4 < k) loss_add4(acc, cache[j], E);
        } else {
            for (int64_t ch = wi; ch < chunks; ch += wpg) {
                unsigned long long b[4];
                load_word<VEC>(src, (ch * LPR + c) * 4, k_live, inc, b);
                loss_add4(acc, b, E);
            }
        }
    }
    loss_flush(acc, lds16, sums);
}

// Rows of an interleaved complex operand, both planes in one pass (four short rows per wavefront, rows of up
// to 1024 elements in registers; anything else takes the two strided passes). Workgroup shape as above.
__global__ __launch_bounds__(64 * kLossWavesMax) void loss_rows_complex_kernel(const double* __restrict__ Z, int64_t ldz,
                                                                               int64_t m, int64_t k, int wpg,
                                                                               unsigned long long* __restrict__ sums_re,
                                                                               unsigned long long* __restrict__ sums_im) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int sub = wave / wpg, wi = wave % wpg, side = kLossWavesMax / wpg;
    const int r4 = lane >> 4, c16 = lane & 15;
    __shared__ unsigned long long wmax[kLossWavesMax][kRowGroup][2];
    __shared__ unsigned long long lds16[OZIMMU_MAX_SLICES];
    LossAcc acc_re, acc_im;
    loss_clear(acc_re);
    loss_clear(acc_im);
    for (int64_t first = (int64_t)blockIdx.x * side; first * kRowGroup < m; first += (int64_t)gridDim.x * side) {
        const int64_t row = (first + sub) * kRowGroup + r4;
        const bool live = row < m;
        const ulonglong2* src = reinterpret_cast<const ulonglong2*>(Z) + (live ? row : 0) * ldz;
        const int64_t k_live = live ? k : 0;
        unsigned long long re[kZRowCacheWords][4], im[kZRowCacheWords][4];
        unsigned long long mx_re = 0, mx_im = 0;
#pragma unroll
        for (int j = 0; j < kZRowCacheWords; ++j) {
            const int64_t l0 = ((int64_t)(wi + wpg * j) * 16 + c16) * 4;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ulonglong2 v = {0ull, 0ull};
                if (l0 + u < k_live) v = src[l0 + u];
                re[j][u] = v.x;
                im[j][u] = v.y;
                const unsigned long long a = v.x & kAbsMask, b = v.y & kAbsMask;
                mx_re = a > mx_re ? a : mx_re;
                mx_im = b > mx_im ? b : mx_im;
            }
        }
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) {
            const unsigned long long o = __shfl_xor(mx_re, off, 64), q = __shfl_xor(mx_im, off, 64);
            mx_re = o > mx_re ? o : mx_re;
            mx_im = q > mx_im ? q : mx_im;
        }
        __syncthreads();   // the maxima of the previous groups have been read by everybody
        if (c16 == 0) {
            wmax[wave][r4][0] = mx_re;
            wmax[wave][r4][1] = mx_im;
        }
        __syncthreads();
        mx_re = wmax[sub * wpg][r4][0];
        mx_im = wmax[sub * wpg][r4][1];
        for (int w = 1; w < wpg; ++w) {
            mx_re = wmax[sub * wpg + w][r4][0] > mx_re ? wmax[sub * wpg + w][r4][0] : mx_re;
            mx_im = wmax[sub * wpg + w][r4][1] > mx_im ? wmax[sub * wpg + w][r4][1] : mx_im;
        }
        const int e_re = exponent_of_max(mx_re), e_im = exponent_of_max(mx_im);
#pragma unroll
        for (int j = 0; j < kZRowCacheWords; ++j) {   // whole words beyond the row are skipped (same for all lanes)
            if ((int64_t)(wi + wpg * j) * 64 < k) {
                loss_add4(acc_re, re[j], e_re);
                loss_add4(acc_im, im[j], e_im);
            }
        }
    }
    loss_flush(acc_re, lds16, sums_re);
    __syncthreads();   // lds16 is reused
    loss_flush(acc_im, lds16, sums_im);
}

// The same for rows of at most 64 W elements (the state vector under a gate of up to seven qubits, Section 4.4): sixteen
// lanes per row, four rows per wavefront and pass, nothing shared between wavefronts until the final sums, and the next
// rows are requested before the current ones are counted. The exponents come from the high words of the bit patterns
// (rotations inside the row of 16 lanes) unless some row's maximum is zero or subnormal.
template <int W>
__global__ __launch_bounds__(64 * kLossWavesMax) void loss_rows_complex_short_kernel(const double* __restrict__ Z, int64_t ldz,
                                                                                     int64_t m, int k,
                                                                                     unsigned long long* __restrict__ sums_re,
                                                                                     unsigned long long* __restrict__ sums_im) {
    const int lane = threadIdx.x & 63, r4 = lane >> 4, c16 = lane & 15;
    __shared__ unsigned long long lds16[OZIMMU_MAX_SLICES];
    LossAcc acc_re, acc_im;
    loss_clear(acc_re);
    loss_clear(acc_im);
    const int64_t groups = (m + kRowGroup - 1) / kRowGroup;
    const int64_t stride = (int64_t)gridDim.x * kLossWavesMax;
    ulonglong2 cur[W][4], nxt[W][4];
    auto request = [&](int64_t group, ulonglong2 (&v)[W][4]) __attribute__((always_inline)) {
        const int64_t row = group * kRowGroup + r4;
        const bool live = group < groups && row < m;
        const ulonglong2* src = reinterpret_cast<const ulonglong2*>(Z) + (live ? row : 0) * ldz;
#pragma unroll
        for (int j = 0; j < W; ++j)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int l = (c16 + 16 * j) * 4 + u;
                v[j][u] = ulonglong2{0ull, 0ull};
                if (live && l < k) v[j][u] = src[l];
            }
    };
    int64_t group = (int64_t)blockIdx.x * kLossWavesMax + (threadIdx.x >> 6);
    request(group, cur);
    for (; group < groups; group += stride) {
        request(group + stride, nxt);
        unsigned hw_re = 0, hw_im = 0;
#pragma unroll
        for (int j = 0; j < W; ++j)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned a = (unsigned)(cur[j][u].x >> 32) & 0x7fffffffu, b = (unsigned)(cur[j][u].y >> 32) & 0x7fffffffu;
                hw_re = a > hw_re ? a : hw_re;
                hw_im = b > hw_im ? b : hw_im;
            }
        hw_re = row_max_step<1>(row_max_step<2>(row_max_step<4>(row_max_step<8>(hw_re))));
        hw_im = row_max_step<1>(row_max_step<2>(row_max_step<4>(row_max_step<8>(hw_im))));
        int e_re = (int)(hw_re >> 20) - 1022, e_im = (int)(hw_im >> 20) - 1022;   // as exponent_of_max for a normal maximum
        if (!__all(hw_re >= 0x00100000u && hw_im >= 0x00100000u)) {   // a zero or subnormal maximum somewhere: 64-bit maxima
            unsigned long long mx_re = 0, mx_im = 0;
#pragma unroll
            for (int j = 0; j < W; ++j)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned long long a = cur[j][u].x & kAbsMask, b = cur[j][u].y & kAbsMask;
                    mx_re = a > mx_re ? a : mx_re;
                    mx_im = b > mx_im ? b : mx_im;
                }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                const unsigned long long o = __shfl_xor(mx_re, off, 64), q = __shfl_xor(mx_im, off, 64);
                mx_re = o > mx_re ? o : mx_re;
                mx_im = q > mx_im ? q : mx_im;
            }
            e_re = exponent_of_max(mx_re);
            e_im = exponent_of_max(mx_im);
        }
#pragma unroll
        for (int j = 0; j < W; ++j) {
            if (j * 64 < k) {   // whole words beyond the row are skipped (same for all lanes)
                const unsigned long long re[4] = {cur[j][0].x, cur[j][1].x, cur[j][2].x, cur[j][3].x};
                const unsigned long long im[4] = {cur[j][0].y, cur[j][1].y, cur[j][2].y, cur[j][3].y};
                loss_add4(acc_re, re, e_re);
                loss_add4(acc_im, im, e_im);
            }
        }
#pragma unroll
        for (int j = 0; j < W; ++j)
#pragma unroll
            for (int u = 0; u < 4; ++u) cur[j][u] = nxt[j][u];
    }
    loss_flush(acc_re, lds16, sums_re);
    __syncthreads();   // lds16 is reused
    loss_flush(acc_im, lds16, sums_im);
}

// Both planes of a small interleaved complex operand whose groups are its columns (k x n, both at most 128: a gate),
// in one launch instead of three per plane: a workgroup per 8 columns, thread (c, w) = (tid % 8, tid / 8) owns four
// consecutive positions of column c; column maxima through LDS, then the scan.
__global__ __launch_bounds__(256) void loss_cols_complex_small_kernel(const double* __restrict__ B, int64_t ldb, int k, int n,
                                                                      unsigned long long* __restrict__ sums_re,
                                                                      unsigned long long* __restrict__ sums_im) {
    const int tid = threadIdx.x, r8 = tid & 7, w = tid >> 3, c = blockIdx.x * 8 + r8;
    const ulonglong2* src = reinterpret_cast<const ulonglong2*>(B);
    unsigned long long re[4], im[4], mx_re = 0, mx_im = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int l = 4 * w + u;
        ulonglong2 v = {0ull, 0ull};
        if (l < k && c < n) v = src[(int64_t)l * ldb + c];
        re[u] = v.x;
        im[u] = v.y;
        const unsigned long long a = v.x & kAbsMask, b = v.y & kAbsMask;
        mx_re = a > mx_re ? a : mx_re;
        mx_im = b > mx_im ? b : mx_im;
    }
    __shared__ unsigned long long colmax[32][8][2];
    __shared__ unsigned long long lds16[OZIMMU_MAX_SLICES];
    colmax[w][r8][0] = mx_re;
    colmax[w][r8][1] = mx_im;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        mx_re = colmax[i][r8][0] > mx_re ? colmax[i][r8][0] : mx_re;
        mx_im = colmax[i][r8][1] > mx_im ? colmax[i][r8][1] : mx_im;
    }
    LossAcc acc_re, acc_im;
    loss_clear(acc_re);
    loss_clear(acc_im);
    loss_add4(acc_re, re, exponent_of_max(mx_re));
    loss_add4(acc_im, im, exponent_of_max(mx_im));
    loss_flush(acc_re, lds16, sums_re);
    __syncthreads();   // lds16 is reused
    loss_flush(acc_im, lds16, sums_im);
}

// Columns of B: as the column-maximum pass, a lane owns a column and a workgroup a band of rows.
__global__ __launch_bounds__(256) void loss_cols_kernel(const double* __restrict__ B, int64_t ldb, int inc,
                                                        int64_t k, int64_t n, int band,
                                                        const unsigned long long* __restrict__ colmax,
                                                        unsigned long long* __restrict__ sums, SecondPlane second = SecondPlane{}) {
    __shared__ unsigned long long lds16[OZIMMU_MAX_SLICES];
    if (blockIdx.z) {
        B += second.b;
        colmax += second.colmax;
        sums += second.sums;
    }
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    LossAcc acc;
    loss_clear(acc);
    if (j < n) {
        const int E = exponent_of_max(colmax[j]);
        const int64_t l0 = (int64_t)blockIdx.y * band;
        const int64_t l1 = l0 + band < k ? l0 + band : k;
        const unsigned long long* src = reinterpret_cast<const unsigned long long*>(B);
        for (int64_t l = l0; l < l1; l += 4) {   // four elements of the column at a time; zeros past the band
            unsigned long long b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) b[u] = l + u < l1 ? src[((l + u) * ldb + j) * inc] : 0ull;
            loss_add4(acc, b, E);
        }
    }
    loss_flush(acc, lds16, sums);
}

__global__ __launch_bounds__(256) void fill_f64_kernel(double* C, int64_t ldc, int c_inc, int64_t m,
                                                       int64_t n, double v) {
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < m * n; idx += (int64_t)gridDim.x * 256)
        C[(idx / n) * ldc + (idx % n) * c_inc] = v;
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t* P, int64_t ldp, int64_t m, int64_t n,
                                                       int32_t v) {
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < m * n; idx += (int64_t)gridDim.x * 256)
        P[(idx / n) * ldp + (idx % n)] = v;
}

__global__ __launch_bounds__(256) void scale_f64_kernel(double* C, int64_t ldc, int64_t m, int64_t n, double beta) {
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < m * n; idx += (int64_t)gridDim.x * 256) {
        double* c = C + (idx / n) * ldc + (idx % n);
        *c = beta == 0.0 ? 0.0 : beta * *c;
    }
}

__global__ __launch_bounds__(256) void zaxpby_kernel(const double* T, int64_t ldt, double* C, int64_t ldc,
                                                     int64_t rows, int64_t cols, double ar, double ai, double br,
                                                     double bi) {
    const bool beta_zero = br == 0.0 && bi == 0.0;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < rows * cols; idx += (int64_t)gridDim.x * 256) {
        const int64_t r = idx / cols, c = idx % cols;
        double* dst = C + 2 * (r * ldc + c);
        double tr = 0.0, ti = 0.0;
        if (T) {
            const double gr = T[2 * (r * ldt + c)], gi = T[2 * (r * ldt + c) + 1];
            tr = ar * gr - ai * gi;
            ti = ar * gi + ai * gr;
        }
        if (!beta_zero) {
            const double cr = dst[0], ci = dst[1];
            const double ur = br * cr - bi * ci, ui = br * ci + bi * cr;
            tr = T ? tr + ur : ur;
            ti = T ? ti + ui : ui;
        }
        dst[0] = tr;
        dst[1] = ti;
    }
}

// Grid of a grid-stride fill: enough blocks to cover the range, capped so the count fits any grid limit.
unsigned fill_blocks(int64_t elems) {
    const int64_t b = (elems + 255) / 256;
    return (unsigned)(b < (1 << 20) ? b : (1 << 20));
}

}  // namespace

// Band height of the column passes: 256 rows, thinner when the matrix is short so that a few
// thousand workgroups exist.
static int column_band(int64_t k, int64_t n) {
    const int64_t bx = (n + 255) / 256;
    const int64_t want_y = (2048 + bx - 1) / bx;
    int64_t band = (k + want_y - 1) / want_y;
    return (int)(band < 8 ? 8 : (band > kColBand ? kColBand : band));
}

static ScanTarget scan_target(unsigned long long* slots, int nc, int s) {
    return ScanTarget{slots, nc, 0x01010101u * (uint32_t)(OZIMMU_SLICE_BITS * s), 0x01010101u * (uint32_t)(OZIMMU_SLICE_BITS * (s > 1 ? s - 1 : 1))};
}

size_t scan_slots_bytes(int planes) { return (size_t)kScanSlots * kScanCounters * planes * sizeof(unsigned long long); }

hipError_t launch_scan_reduce(const unsigned long long* slots, int planes, int s, unsigned long long* out, hipStream_t st) {
    scan_reduce_kernel<<<dim3(1), dim3(256), 0, st>>>(slots, kScanCounters * planes, s, out);
    return hipGetLastError();
}

hipError_t launch_split_rows(const double* A, int64_t lda, int inc, int64_t m, int64_t k, int s,
                             int8_t* S, int64_t m_pad, int64_t k_pad, int32_t* E, hipStream_t st, bool negate,
                             unsigned long long* scan_slots, int scan_nc) {
    if (m_pad == 0 || k_pad == 0) return hipSuccess;
    const ScanTarget scan = scan_target(scan_slots, scan_nc, s);
    const unsigned long long flip = negate ? 1ull << 63 : 0ull;
    const bool wide = s > 9;
    // a wavefront covers 64 elements of each of its four rows per word it caches
    const int64_t want = (k_pad + 64 * kRowCacheWords - 1) / (64 * kRowCacheWords);
    const int nwaves = (int)(want < 1 ? 1 : want > kRowWavesMax ? kRowWavesMax : want);
    const bool cached = k_pad <= (int64_t)64 * kRowCacheWords * nwaves;
    const bool vec = inc == 1 && lda % 2 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0;
    const dim3 grid((unsigned)(m_pad / kRowGroup)), block(64 * nwaves);
#define OZ_ROWS(W, C, V) do { if (scan.slots) split_rows_kernel<W, C, V, true><<<grid, block, 0, st>>>(A, lda * inc, inc, (int)m, k, s, S, m_pad, k_pad, E, flip, scan); \
                              else split_rows_kernel<W, C, V, false><<<grid, block, 0, st>>>(A, lda * inc, inc, (int)m, k, s, S, m_pad, k_pad, E, flip, scan); } while (0)
    if (wide) {
        if (cached) { if (vec) OZ_ROWS(true, true, true); else OZ_ROWS(true, true, false); }
        else        { if (vec) OZ_ROWS(true, false, true); else OZ_ROWS(true, false, false); }
    } else {
        if (cached) { if (vec) OZ_ROWS(false, true, true); else OZ_ROWS(false, true, false); }
        else        { if (vec) OZ_ROWS(false, false, true); else OZ_ROWS(false, false, false); }
    }
#undef OZ_ROWS
    return hipGetLastError();
}

bool complex_rows_in_one_pass(const double* Z, int64_t k_pad) {
    return k_pad <= (int64_t)64 * kZRowCacheWords * kRowWavesMax && reinterpret_cast<uintptr_t>(Z) % 16 == 0;
}

hipError_t launch_split_rows_complex(const double* Z, int64_t ldz, int64_t m, int64_t k, int s, int8_t* S_re,
                                     int8_t* S_im, int64_t m_pad, int64_t k_pad, int32_t* E_re, int32_t* E_im,
                                     hipStream_t st, bool negate_im, unsigned long long* scan_slots) {
    if (m_pad == 0 || k_pad == 0) return hipSuccess;
    if (!complex_rows_in_one_pass(Z, k_pad)) return hipErrorInvalidValue;
    const ScanTarget scan = scan_target(scan_slots, 2 * kScanCounters, s);
    const int64_t want = (k_pad + 64 * kZRowCacheWords - 1) / (64 * kZRowCacheWords);
    const int nwaves = (int)(want < 1 ? 1 : want);
    const unsigned long long flip_im = negate_im ? 1ull << 63 : 0ull;
    const dim3 grid((unsigned)(m_pad / kRowGroup)), block(64 * nwaves);
#define OZ_ZROWS(W, SC) split_rows_complex_kernel<W, SC><<<grid, block, 0, st>>>(Z, ldz, (int)m, k, s, S_re, S_im, m_pad, k_pad, E_re, E_im, 0ull, flip_im, scan)
    if (s > 9) { if (scan.slots) OZ_ZROWS(true, true); else OZ_ZROWS(true, false); }
    else       { if (scan.slots) OZ_ZROWS(false, true); else OZ_ZROWS(false, false); }
#undef OZ_ZROWS
    return hipGetLastError();
}

bool complex_scan_in_one_pass(const double* Z, int64_t k) {
    return k <= (int64_t)64 * kZRowCacheWords * kLossWavesMax && reinterpret_cast<uintptr_t>(Z) % 16 == 0;
}

// Wavefronts per row group for rows of k elements when one wavefront covers per_wave of them: 1, 2 or 4.
static int loss_waves_per_group(int64_t k, int64_t per_wave) {
    const int64_t want = (k + per_wave - 1) / per_wave;
    return want <= 1 ? 1 : want <= 2 ? 2 : kLossWavesMax;
}
// Workgroups of four wavefronts for `groups` row groups, 4 / wpg of them side by side: as many as fill the chip
// a few times over, few enough that their final flushes do not queue up.
static unsigned loss_grid(int64_t groups, int wpg, int64_t cap) {
    const int64_t side = kLossWavesMax / wpg, wgs = (groups + side - 1) / side;
    return (unsigned)(wgs < cap ? wgs : cap);
}

hipError_t launch_loss_scan_rows_complex(const double* Z, int64_t ldz, int64_t m, int64_t k,
                                         unsigned long long* sums_re, unsigned long long* sums_im, hipStream_t st) {
    if (m == 0 || k == 0) return hipSuccess;
    if (!complex_scan_in_one_pass(Z, k)) return hipErrorInvalidValue;
    if (k <= 128) {   // short rows: wavefronts on their own, up to four per SIMD
        const int64_t row_groups = (m + kRowGroup - 1) / kRowGroup;
        const int64_t want = (row_groups + kLossWavesMax - 1) / kLossWavesMax;
        const unsigned grid = (unsigned)(want < 1024 ? want : 1024);
        if (k <= 64) loss_rows_complex_short_kernel<1><<<dim3(grid), dim3(64 * kLossWavesMax), 0, st>>>(Z, ldz, m, (int)k, sums_re, sums_im);
        else loss_rows_complex_short_kernel<2><<<dim3(grid), dim3(64 * kLossWavesMax), 0, st>>>(Z, ldz, m, (int)k, sums_re, sums_im);
        return hipGetLastError();
    }
    const int wpg = loss_waves_per_group(k, 64 * kZRowCacheWords);
    const int64_t groups = (m + kRowGroup - 1) / kRowGroup;
    loss_rows_complex_kernel<<<dim3(loss_grid(groups, wpg, 512)), dim3(64 * kLossWavesMax), 0, st>>>(Z, ldz, m, k, wpg, sums_re, sums_im);
    return hipGetLastError();
}

bool complex_cols_scan_in_one_launch(const double* B, int64_t k, int64_t n) {
    return k <= 128 && n <= 128 && reinterpret_cast<uintptr_t>(B) % 16 == 0;
}

hipError_t launch_loss_scan_cols_complex_small(const double* B, int64_t ldb, int64_t k, int64_t n,
                                               unsigned long long* sums_re, unsigned long long* sums_im, hipStream_t st) {
    if (k == 0 || n == 0) return hipSuccess;
    if (!complex_cols_scan_in_one_launch(B, k, n)) return hipErrorInvalidValue;
    loss_cols_complex_small_kernel<<<dim3((unsigned)((n + 7) / 8)), dim3(256), 0, st>>>(B, ldb, (int)k, (int)n, sums_re, sums_im);
    return hipGetLastError();
}

hipError_t launch_split_cols(const double* B, int64_t ldb, int inc, int64_t k, int64_t n, int s,
                             int8_t* S, int64_t n_pad, int64_t k_pad, int32_t* E,
                             unsigned long long* colmax, hipStream_t st, bool negate, unsigned long long* scan_slots,
                             int scan_nc) {
    if (n_pad == 0) return hipSuccess;
    const ScanTarget scan = scan_target(scan_slots, scan_nc, s);
    const unsigned long long flip = negate ? 1ull << 63 : 0ull;
    fill_u64_kernel<<<dim3((unsigned)((n_pad + 255) / 256)), dim3(256), 0, st>>>(colmax, n_pad, 0ull);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (k > 0 && n > 0) {
        const int64_t bx = (n + 255) / 256;
        const int band = column_band(k, n);
        col_max_kernel<<<dim3((unsigned)bx, (unsigned)((k + band - 1) / band)), dim3(256), 0, st>>>(
            B, ldb, inc, k, n, band, colmax);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (k_pad == 0) {   // no slices to write: only the exponents (all zero)
        if (n > 0) col_exponent_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(colmax, n, E);
        return hipGetLastError();
    }
    const int64_t l_tiles = (k_pad + kColTileL - 1) / kColTileL;
    const int j_tiles = (int)(n_pad / kColTileJ);
    if (j_tiles * l_tiles > 0x7fffffffll) return hipErrorInvalidValue;   // beyond any grid (and any memory)
    const dim3 grid((unsigned)(j_tiles * l_tiles));
#define OZ_COLS(W, SC) split_cols_kernel<W, SC><<<grid, dim3(256), 0, st>>>(B, ldb, inc, k, n, s, S, n_pad, k_pad, colmax, E, j_tiles, flip, SecondPlane{}, scan)
    if (s > 9) { if (scan.slots) OZ_COLS(true, true); else OZ_COLS(true, false); }
    else       { if (scan.slots) OZ_COLS(false, true); else OZ_COLS(false, false); }
#undef OZ_COLS
    return hipGetLastError();
}

// Both planes of an interleaved complex operand (element stride 2) in three launches: colmax holds 2 n_pad entries.
hipError_t launch_split_cols_complex(const double* B, int64_t ldb, int64_t k, int64_t n, int s, int8_t* S_re, int8_t* S_im,
                                     int64_t n_pad, int64_t k_pad, int32_t* E_re, int32_t* E_im,
                                     unsigned long long* colmax, hipStream_t st, bool negate_im,
                                     unsigned long long* scan_slots) {
    if (n_pad == 0) return hipSuccess;
    const ScanTarget scan = scan_target(scan_slots, 2 * kScanCounters, s);
    fill_u64_kernel<<<dim3((unsigned)((2 * n_pad + 255) / 256)), dim3(256), 0, st>>>(colmax, 2 * n_pad, 0ull);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    SecondPlane second{1, n_pad, S_im - S_re, E_im - E_re, negate_im ? 1ull << 63 : 0ull, 0};
    if (k > 0 && n > 0) {
        const int64_t bx = (n + 255) / 256;
        const int band = column_band(k, n);
        col_max_kernel<<<dim3((unsigned)bx, (unsigned)((k + band - 1) / band), 2), dim3(256), 0, st>>>(
            B, ldb, 2, k, n, band, colmax, second);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (k_pad == 0) {   // no slices to write: only the exponents (all zero)
        if (n > 0) {
            col_exponent_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(colmax, n, E_re);
            col_exponent_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(colmax + n_pad, n, E_im);
        }
        return hipGetLastError();
    }
    const int64_t l_tiles = (k_pad + kColTileL - 1) / kColTileL;
    const int j_tiles = (int)(n_pad / kColTileJ);
    if (j_tiles * l_tiles > 0x7fffffffll) return hipErrorInvalidValue;   // beyond any grid (and any memory)
    const dim3 grid((unsigned)(j_tiles * l_tiles), 1, 2);
#define OZ_COLS(W, SC) split_cols_kernel<W, SC><<<grid, dim3(256), 0, st>>>(B, ldb, 2, k, n, s, S_re, n_pad, k_pad, colmax, E_re, j_tiles, 0ull, second, scan)
    if (s > 9) { if (scan.slots) OZ_COLS(true, true); else OZ_COLS(true, false); }
    else       { if (scan.slots) OZ_COLS(false, true); else OZ_COLS(false, false); }
#undef OZ_COLS
    return hipGetLastError();
}

template <int ROWS>
static hipError_t launch_loss_rows(const double* A, int64_t lda, int inc, int64_t m, int64_t k,
                                   unsigned long long* sums, hipStream_t st) {
    // a wavefront covers 4 * (64 / ROWS) elements of each of its rows per word it caches
    const int64_t per_wave = (int64_t)4 * (64 / ROWS) * kRowCacheWords;
    const int wpg = loss_waves_per_group(k, per_wave);
    const bool cached = k <= per_wave * wpg;
    const bool vec = inc == 1 && lda % 2 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0;
    const dim3 grid(loss_grid((m + ROWS - 1) / ROWS, wpg, 1024)), block(64 * kLossWavesMax);
    if (cached) {
        if (vec) loss_rows_kernel<ROWS, true, true><<<grid, block, 0, st>>>(A, lda * inc, inc, m, k, wpg, sums);
        else loss_rows_kernel<ROWS, true, false><<<grid, block, 0, st>>>(A, lda * inc, inc, m, k, wpg, sums);
    } else {
        if (vec) loss_rows_kernel<ROWS, false, true><<<grid, block, 0, st>>>(A, lda * inc, inc, m, k, wpg, sums);
        else loss_rows_kernel<ROWS, false, false><<<grid, block, 0, st>>>(A, lda * inc, inc, m, k, wpg, sums);
    }
    return hipGetLastError();
}

hipError_t launch_loss_scan_rows(const double* A, int64_t lda, int inc, int64_t m, int64_t k,
                                 unsigned long long* sums, hipStream_t st) {
    if (m == 0 || k == 0) return hipSuccess;
    // four rows per wavefront while four wavefronts still hold them in registers (k <= 2048)
    if (k <= (int64_t)4 * 16 * kRowCacheWords * kLossWavesMax) return launch_loss_rows<4>(A, lda, inc, m, k, sums, st);
    return launch_loss_rows<1>(A, lda, inc, m, k, sums, st);
}

hipError_t launch_loss_scan_cols(const double* B, int64_t ldb, int inc, int64_t k, int64_t n,
                                 unsigned long long* colmax, unsigned long long* sums, hipStream_t st) {
    if (k == 0 || n == 0) return hipSuccess;
    const int64_t bx = (n + 255) / 256;
    fill_u64_kernel<<<dim3((unsigned)bx), dim3(256), 0, st>>>(colmax, n, 0ull);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int band = column_band(k, n);
    const dim3 grid((unsigned)bx, (unsigned)((k + band - 1) / band));
    col_max_kernel<<<grid, dim3(256), 0, st>>>(B, ldb, inc, k, n, band, colmax);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    loss_cols_kernel<<<grid, dim3(256), 0, st>>>(B, ldb, inc, k, n, band, colmax, sums);
    return hipGetLastError();
}

// Both planes of an interleaved complex operand scanned by columns, in three launches; colmax: 2 n entries.
hipError_t launch_loss_scan_cols_complex(const double* B, int64_t ldb, int64_t k, int64_t n, unsigned long long* colmax,
                                         unsigned long long* sums_re, unsigned long long* sums_im, hipStream_t st) {
    if (k == 0 || n == 0) return hipSuccess;
    const int64_t bx = (n + 255) / 256;
    fill_u64_kernel<<<dim3((unsigned)((2 * n + 255) / 256)), dim3(256), 0, st>>>(colmax, 2 * n, 0ull);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int band = column_band(k, n);
    const dim3 grid((unsigned)bx, (unsigned)((k + band - 1) / band), 2);
    SecondPlane second{1, n, 0, 0, 0ull, sums_im - sums_re};
    col_max_kernel<<<grid, dim3(256), 0, st>>>(B, ldb, 2, k, n, band, colmax, second);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    loss_cols_kernel<<<grid, dim3(256), 0, st>>>(B, ldb, 2, k, n, band, colmax, sums_re, second);
    return hipGetLastError();
}

hipError_t launch_scale_f64(double* C, int64_t ldc, int64_t m, int64_t n, double beta, hipStream_t st) {
    if (m * n == 0) return hipSuccess;
    scale_f64_kernel<<<dim3(fill_blocks(m * n)), dim3(256), 0, st>>>(C, ldc, m, n, beta);
    return hipGetLastError();
}

hipError_t launch_zaxpby(const double* T, int64_t ldt, double* C, int64_t ldc, int64_t rows, int64_t cols,
                         double ar, double ai, double br, double bi, hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    zaxpby_kernel<<<dim3(fill_blocks(rows * cols)), dim3(256), 0, st>>>(T, ldt, C, ldc, rows, cols, ar, ai, br, bi);
    return hipGetLastError();
}

hipError_t launch_fill_u64(unsigned long long* p, int64_t count, unsigned long long v, hipStream_t st) {
    if (count == 0) return hipSuccess;
    fill_u64_kernel<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(p, count, v);
    return hipGetLastError();
}

hipError_t launch_fill_f64(double* C, int64_t ldc, int c_inc, int64_t m, int64_t n, double v,
                           hipStream_t st) {
    if (m * n == 0) return hipSuccess;
    fill_f64_kernel<<<dim3(fill_blocks(m * n)), dim3(256), 0, st>>>(C, ldc, c_inc, m, n, v);
    return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* P, int64_t ldp, int64_t m, int64_t n, int32_t v, hipStream_t st) {
    if (m * n == 0) return hipSuccess;
    fill_i32_kernel<<<dim3(fill_blocks(m * n)), dim3(256), 0, st>>>(P, ldp, m, n, v);
    return hipGetLastError();
}

}  // namespace ozimmu
