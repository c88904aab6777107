// SplitInt (Section 3.1, splitting algorithm for integer arithmetic) on gfx950.
//
// One power-of-two exponent per row of M = A or B^T (line 2 of SplitInt), then every element
// is cut by bit operations (Section 4.1) into signed 7-bit chunks of its significand, placed
// relative to the row exponent (lines 3-5). Output: padded INT8 slice tensors, zero outside the
// matrix, in the tiled and column-swizzled block layout that the slice-product kernel copies
// linearly into LDS (blocks of 256 rows x 64 bytes; the layout is defined with the C ABI).
//
// Both kernels are HBM-bound: 8 B read per element (16 B for B, whose column maxima need a
// pass of their own) and num_slices bytes written.
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

// An element prepared for chunk extraction: |x| = M * 2^(-g) * 2^E with M < 2^53.
struct Prepared {
    unsigned long long M;
    int g;      // chunk p = floor(M * 2^(7p - g)) mod 128
    int neg;
};

__device__ __forceinline__ Prepared prepare(unsigned long long bits, int E) {
    Prepared r;
    int e = (int)((bits >> 52) & 0x7ff);
    unsigned long long mant = bits & kMantMask;
    r.M = e ? (mant | (1ull << 52)) : mant;
    r.g = E + 1075 - (e ? e : 1);
    r.neg = (int)(bits >> 63);
    return r;
}

__device__ __forceinline__ int chunk(const Prepared& x, int p) {
    int nsh = x.g - OZIMMU_SLICE_BITS * p;  // right shift that brings chunk p to the low 7 bits
    unsigned int c;
    if (nsh >= 64) c = 0;
    else if (nsh >= 0) c = (unsigned int)(x.M >> nsh) & 127u;
    else if (nsh > -OZIMMU_SLICE_BITS) c = (unsigned int)(x.M << (-nsh)) & 127u;
    else c = 0;
    return x.neg ? -(int)c : (int)c;
}

// Byte offset, inside one slice, of the 4-byte word that holds positions l0 .. l0+3 (l0 % 4 == 0)
// of padded row r: blocks of 256 rows x 64 bytes, 16-byte columns swizzled with bits 2..3 of the row.
__device__ __forceinline__ int64_t word_offset(int64_t r, int64_t l0, int64_t k_pad) {
    const int64_t rr = r & (kTile - 1);
    const int64_t c = (l0 & (kStep - 1)) >> 4;
    return ((r / kTile) * (k_pad / kStep) + l0 / kStep) * kBlockBytes + rr * kStep + ((c ^ ((rr >> 2) & 3)) << 4) + (l0 & 15);
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        unsigned long long o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// ------------------------------------------------------------------------------ rows of A
// One workgroup per padded row. Pass 1: maximum of |x| bit patterns (monotone in |x|), wave
// reduction then LDS. Pass 2: the row is read again (it was just streamed through L2) and
// four consecutive elements per lane are packed into one 32-bit store per slice.
__global__ __launch_bounds__(256) void split_rows_kernel(const double* __restrict__ A, int64_t lda,
                                                         int inc, int m, int64_t k, int s,
                                                         int8_t* __restrict__ S, int64_t m_pad,
                                                         int64_t k_pad, int32_t* __restrict__ Eout) {
    const int row = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t slice_stride = m_pad * k_pad;
    const int64_t words = k_pad / 4;

    if (row >= m) {  // padding rows: zeros in every slice
        for (int64_t w = tid; w < words; w += 256) {
            const int64_t off = word_offset(row, w * 4, k_pad);
            for (int p = 0; p < s; ++p) *reinterpret_cast<uint32_t*>(S + p * slice_stride + off) = 0u;
        }
        return;
    }

    const unsigned long long* src = reinterpret_cast<const unsigned long long*>(A) + (int64_t)row * lda * 1;
    unsigned long long mx = 0;
    for (int64_t l = tid; l < k; l += 256) {
        unsigned long long b = src[l * inc] & kAbsMask;
        mx = b > mx ? b : mx;
    }
    mx = wave_max_u64(mx);
    __shared__ unsigned long long wmax[4];
    if ((tid & 63) == 0) wmax[tid >> 6] = mx;
    __syncthreads();
    mx = wmax[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) mx = wmax[w] > mx ? wmax[w] : mx;
    const int E = exponent_of_max(mx);
    if (tid == 0) Eout[row] = E;

    for (int64_t w = tid; w < words; w += 256) {
        const int64_t l0 = w * 4;
        Prepared x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            unsigned long long b = (l0 + u < k) ? src[(l0 + u) * inc] : 0ull;
            x[u] = prepare(b, E);
        }
        const int64_t off = word_offset(row, l0, k_pad);
        for (int p = 1; p <= s; ++p) {
            uint32_t packed = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) packed |= ((uint32_t)chunk(x[u], p) & 0xffu) << (8 * u);
            *reinterpret_cast<uint32_t*>(S + (int64_t)(p - 1) * slice_stride + off) = packed;
        }
    }
}

// ------------------------------------------------------------------------------ columns of B
__global__ __launch_bounds__(256) void fill_u64_kernel(unsigned long long* p, int64_t n,
                                                       unsigned long long v) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// Column maxima of |B|: a lane owns a column (loads are contiguous across lanes), a workgroup
// owns a band of rows, bands are combined with a 64-bit atomic maximum on the bit patterns.
constexpr int kColBand = 256;   // rows per band when the matrix is tall enough to fill the chip
__global__ __launch_bounds__(256) void col_max_kernel(const double* __restrict__ B, int64_t ldb,
                                                      int inc, int64_t k, int64_t n, int band,
                                                      unsigned long long* __restrict__ colmax) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
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

// Slice emission for B^T: a workgroup takes a 128 (l) x 64 (j) tile of B. Lane (jj, lg) reads
// 32 elements of column jj (contiguous across lanes for each l), packs four consecutive l per
// slice into one word and transposes through LDS so that the global stores run along l.
constexpr int kColTileL = 128, kColTileJ = 64, kColGroup = 7;
constexpr int kColLdsStride = kColTileL / 4 + 1;  // words per LDS row (+1: conflict-free columns)
__global__ __launch_bounds__(256) void split_cols_kernel(const double* __restrict__ B, int64_t ldb,
                                                         int inc, int64_t k, int64_t n, int s,
                                                         int8_t* __restrict__ S, int64_t n_pad,
                                                         int64_t k_pad,
                                                         const unsigned long long* __restrict__ colmax) {
    __shared__ uint32_t tile[kColGroup][kColTileJ][kColLdsStride];
    const int tid = threadIdx.x;
    const int jj = tid & 63, lg = tid >> 6;
    const int64_t j = (int64_t)blockIdx.x * kColTileJ + jj;
    const int64_t lbase = (int64_t)blockIdx.y * kColTileL;
    const int64_t slice_stride = n_pad * k_pad;
    const unsigned long long* src = reinterpret_cast<const unsigned long long*>(B);
    const int E = (j < n) ? exponent_of_max(colmax[j]) : 0;

    Prepared x[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) {
        const int64_t l = lbase + lg * 32 + u;
        unsigned long long b = (j < n && l < k) ? src[(l * ldb + j) * inc] : 0ull;
        x[u] = prepare(b, E);
    }
    for (int p0 = 1; p0 <= s; p0 += kColGroup) {
        const int np = (s - p0 + 1) < kColGroup ? (s - p0 + 1) : kColGroup;
        for (int pp = 0; pp < np; ++pp) {
#pragma unroll
            for (int u4 = 0; u4 < 8; ++u4) {
                uint32_t packed = 0;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    packed |= ((uint32_t)chunk(x[u4 * 4 + u], p0 + pp) & 0xffu) << (8 * u);
                tile[pp][jj][lg * 8 + u4] = packed;
            }
        }
        __syncthreads();
        // Write-out: per slice the tile is 2 k-steps x 64 rows x four 16-byte columns; in the
        // block layout 16 consecutive rows of one k-step are 1 KiB contiguous, so consecutive
        // lanes store consecutive 16-byte columns.
        for (int pp = 0; pp < np; ++pp) {
            int8_t* dst = S + (int64_t)(p0 + pp - 1) * slice_stride;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int unit = it * 256 + tid;       // 0..511
                const int ks2 = unit >> 8;              // k-step inside the tile
                const int r = (unit >> 2) & 63;         // row inside the tile
                const int pc = unit & 3;                // physical 16-byte column
                const int64_t jr = (int64_t)blockIdx.x * kColTileJ + r;
                const int rr = (int)(jr & (kTile - 1));
                const int c = pc ^ ((rr >> 2) & 3);     // logical column stored there
                const int w0 = ks2 * 16 + c * 4;        // first word of that column in the LDS row
                uint4 v = {tile[pp][r][w0], tile[pp][r][w0 + 1], tile[pp][r][w0 + 2], tile[pp][r][w0 + 3]};
                const int64_t off = ((jr / kTile) * (k_pad / kStep) + (lbase / kStep + ks2)) * kBlockBytes + rr * kStep + pc * 16;
                *reinterpret_cast<uint4*>(dst + off) = v;
            }
        }
        __syncthreads();
    }
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

// Grid of a grid-stride fill: enough blocks to cover the range, capped so the count fits any grid limit.
unsigned fill_blocks(int64_t elems) {
    const int64_t b = (elems + 255) / 256;
    return (unsigned)(b < (1 << 20) ? b : (1 << 20));
}

}  // namespace

hipError_t launch_split_rows(const double* A, int64_t lda, int inc, int64_t m, int64_t k, int s,
                             int8_t* S, int64_t m_pad, int64_t k_pad, int32_t* E, hipStream_t st) {
    if (m_pad == 0) return hipSuccess;
    split_rows_kernel<<<dim3((unsigned)m_pad), dim3(256), 0, st>>>(A, lda * inc, inc, (int)m, k, s, S,
                                                                   m_pad, k_pad, E);
    return hipGetLastError();
}

hipError_t launch_split_cols(const double* B, int64_t ldb, int inc, int64_t k, int64_t n, int s,
                             int8_t* S, int64_t n_pad, int64_t k_pad, int32_t* E,
                             unsigned long long* colmax, hipStream_t st) {
    if (n_pad == 0) return hipSuccess;
    fill_u64_kernel<<<dim3((unsigned)((n_pad + 255) / 256)), dim3(256), 0, st>>>(colmax, n_pad, 0ull);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (k > 0 && n > 0) {
        // short matrices: thinner bands, so that a few thousand workgroups exist
        const int64_t bx = (n + 255) / 256;
        const int64_t want_y = (2048 + bx - 1) / bx;
        int64_t band = (k + want_y - 1) / want_y;
        band = band < 8 ? 8 : (band > kColBand ? kColBand : band);
        col_max_kernel<<<dim3((unsigned)bx, (unsigned)((k + band - 1) / band)), dim3(256), 0, st>>>(
            B, ldb, inc, k, n, (int)band, colmax);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (n > 0) {
        col_exponent_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(colmax, n, E);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    split_cols_kernel<<<dim3((unsigned)(n_pad / kColTileJ), (unsigned)(k_pad / kColTileL)), dim3(256),
                        0, st>>>(B, ldb, inc, k, n, s, S, n_pad, k_pad, colmax);
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
