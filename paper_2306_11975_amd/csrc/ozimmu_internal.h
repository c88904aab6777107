// Internal declarations shared by the translation units of libozimmu (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ozimmu.h"

namespace ozimmu {

constexpr int kRowAlign = OZIMMU_ROW_ALIGN;   // slice rows are padded to a multiple of this (128)
constexpr int kSlab = OZIMMU_K_ALIGN;         // k-extent of one MFMA operand fragment and of one pipeline step (32)
constexpr int kFragRows = 32;                 // rows of one fragment
constexpr int kFragBytes = kFragRows * kSlab; // 1 KiB: what one wave-wide direct load moves and one ds_read_b128 reads
constexpr int kBand = 8;                      // anti-diagonals whose INT32 sums a wavefront holds at a time

static inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Wavefront grid of the product kernel: 2 x 4 wavefronts of 32 x 32 outputs (a 64 x 128 tile of C) while two
// pipeline stages of all slices fit the LDS, 2 x 2 (64 x 64) beyond. `small`: 2 x 2 also for up to nine slices,
// two such workgroups per compute unit (see use_small_tiles).
static inline void tile_waves(int s, bool small, int* wm, int* wn) {
    *wm = 2;
    *wn = (s > 13 || (small && s <= 9)) ? 2 : 4;
}
// Whether a product of this shape runs on 64 x 64 tiles, two workgroups per compute unit (a complex product in one
// launch: asked with k_pad = INT64_MAX, i.e. only for the second reason): when the inner
// dimension is short (a tile is then mostly start-up, fold and stores, and two independent workgroups overlap
// one's with the other's matrix-core work) or when the 64 x 128 tiling leaves compute units without a tile.
// Never with k-blocking, so that the workspace layout does not depend on it.
static inline bool use_small_tiles(int64_t m, int64_t n, int64_t k_pad, int s, bool wide) {
    if (s > 9 || wide) return false;
    const int64_t big_tiles = ((m + 63) / 64) * ((n + 127) / 128);
    return k_pad <= 512 || big_tiles < 256;
}

// Arguments of the slice-product kernel. One launch covers every tile of C.
struct GemmArgs {
    const int8_t* SA;        // slice tensor of A   (fragment layout, see ozimmu.h)
    const int8_t* SB;        // slice tensor of B^T
    int64_t a_slice_stride;  // bytes between consecutive slices of A
    int64_t b_slice_stride;
    int kslabs;              // padded row length in slabs of 32
    int t_begin, t_end;      // slab range of the walk along k
    int tiles_m, tiles_n;
    int tile_cols;           // 128, or 64 (2 x 2 wavefronts)
    int m, n;                // true extent of C
    int block_steps;         // steps after which the INT32 sums are moved into the INT64 sums in D (0: never)
    long long* D;            // INT64 diagonal sums (k-blocking only)
    int32_t* P;              // pair mode (P != nullptr): raw INT32 product of the slices SA, SB point at
    int64_t ldp;
    double* C;               // output, row-major
    int64_t ldc;             // in doubles
    int c_mode;              // 0: C = G, 1: C = C + G, 2: C = C - G, 3: C = alpha G (+ beta C if beta != 0),
                             // 4: (Zr, C + G) -> Cz as interleaved (re, im) pairs (C is read only)
    double* Zr;              // c_mode 4: finished real parts, same shape and leading dimension as C (complex
                             // mode: the plane the real part is formed in)
    double* Cz;              // c_mode 4: complex output
    int64_t ldcz;            // c_mode 4: its leading dimension in complex elements
    double alpha, beta;      // c_mode 3 only
    double* C_lo;            // low parts of a double-double result (double-double summing-up only)
    const int32_t* EA;
    const int32_t* EB;
    // complex mode only: the slice tensors and exponents of the imaginary planes (SA, SB, EA, EB: real planes)
    const int8_t* SA2;
    const int8_t* SB2;
    const int32_t* EA2;
    const int32_t* EB2;
};

// Arguments of the one-kernel complex product with a short inner dimension and few columns (a gate applied to
// a state vector, Section 4.4): Z is split inside the kernel, the small operand arrives as two slice tensors
// and exponent sets (gate.hip).
struct GateArgs {
    const double* Z;         // m x k complex elements, interleaved (re, im), 16-byte aligned
    int64_t ldz;             // in complex elements
    int64_t m;
    int k, n;                // 1 .. 128 each
    const int8_t* T;         // the gate's two slice tensors
    const int32_t* E;        // and their exponents
    double* Cz;              // m x n complex elements, interleaved, 16-byte aligned
    int64_t ldcz;            // in complex elements
    unsigned* scan;          // not null: per tile of 32 rows, ten counters for the check of the slice count (gate.hip)
};
// Whether that kernel serves a complex product Z (m x k) times B (k x n) -> Cz with s slices.
bool gate_product_applies(const double* Z, const double* B, const double* Cz, int64_t n, int64_t k, int s);
// Device scratch it needs for the gate's slices and exponents (0 if the shape is never served).
size_t gate_scratch_bytes(int64_t n, int64_t k, int s);
// Cz = Z . B: splits B (k x n complex elements, leading dimension ldb in complex elements) into `scratch`
// (16-byte aligned, gate_scratch_bytes), then the product kernel. Only where gate_product_applies.
// scan_partials (optional; gate_scan_bytes(m) bytes of device memory): the two kernels also count what the check of s
// as the automatic slice count needs, and scan_sums[plane * 16 + s - 1], [.. + s - 2] (planes 0, 1: real and imaginary
// part of Z, 2, 3: of B; the layout of the slice-count sums; device or mapped host memory) receive the bits the planes
// lose with s and with s - 1 slices.
size_t gate_scan_bytes(int64_t m);
hipError_t launch_gate_product(const double* Z, int64_t ldz, int64_t m, int64_t k, int64_t n, const double* B, int64_t ldb,
                               int s, void* scratch, double* Cz, int64_t ldcz, hipStream_t st,
                               unsigned* scan_partials = nullptr, unsigned long long* scan_sums = nullptr);

// negate: emit the slices of -A (-B) instead: same exponents, every slice with the opposite sign
// (how a conjugated operand's imaginary plane is split)
// Counting while splitting (the check of s as the automatic slice count, Section 4.4): scan_slots, if not null, is a
// zeroed array of scan_slots_bytes(planes of the operand) bytes; the splitter adds, per plane, five counters into one
// of its slots (scan_nc counters to a slot: 5 per plane of the operand; a one-plane launcher is handed the pointer to
// its plane's five), and launch_scan_reduce turns them into the bits lost with s and with s - 1 slices:
// out[plane * 16 + s - 1], out[plane * 16 + s - 2] (device or mapped host memory).
size_t scan_slots_bytes(int planes);
hipError_t launch_scan_reduce(const unsigned long long* slots, int planes, int s, unsigned long long* out, hipStream_t st);
hipError_t launch_split_rows(const double* A, int64_t lda, int inc, int64_t m, int64_t k, int s,
                             int8_t* S, int64_t m_pad, int64_t k_pad, int32_t* E, hipStream_t st,
                             bool negate = false, unsigned long long* scan_slots = nullptr, int scan_nc = 5);
hipError_t launch_split_cols(const double* B, int64_t ldb, int inc, int64_t k, int64_t n, int s,
                             int8_t* S, int64_t n_pad, int64_t k_pad, int32_t* E,
                             unsigned long long* colmax, hipStream_t st, bool negate = false,
                             unsigned long long* scan_slots = nullptr, int scan_nc = 5);
// Both planes of an interleaved complex B (k x n complex elements, leading dimension ldb in complex elements) in one
// set of launches; colmax: 2 n_pad entries. negate_im: the slices of -Im(B) (a conjugated operand).
hipError_t launch_split_cols_complex(const double* B, int64_t ldb, int64_t k, int64_t n, int s, int8_t* S_re, int8_t* S_im,
                                     int64_t n_pad, int64_t k_pad, int32_t* E_re, int32_t* E_im,
                                     unsigned long long* colmax, hipStream_t st, bool negate_im = false,
                                     unsigned long long* scan_slots = nullptr);
// Rows of an interleaved complex operand (Z: m x k complex elements, leading dimension ldz in complex
// elements), both planes in one pass; only where complex_rows_in_one_pass / complex_scan_in_one_pass say so
// (short enough rows, 16-byte aligned), otherwise one strided pass per plane with the functions above / below.
bool complex_rows_in_one_pass(const double* Z, int64_t k_pad);
hipError_t launch_split_rows_complex(const double* Z, int64_t ldz, int64_t m, int64_t k, int s, int8_t* S_re,
                                     int8_t* S_im, int64_t m_pad, int64_t k_pad, int32_t* E_re, int32_t* E_im,
                                     hipStream_t st, bool negate_im = false, unsigned long long* scan_slots = nullptr);
bool complex_scan_in_one_pass(const double* Z, int64_t k);
hipError_t launch_loss_scan_rows_complex(const double* Z, int64_t ldz, int64_t m, int64_t k,
                                         unsigned long long* sums_re, unsigned long long* sums_im, hipStream_t st);
// Both planes of a small interleaved complex operand scanned by columns (B: k x n complex elements, leading dimension
// ldb in complex elements, k and n at most 128, 16-byte aligned) in one launch.
bool complex_cols_scan_in_one_launch(const double* B, int64_t k, int64_t n);
hipError_t launch_loss_scan_cols_complex_small(const double* B, int64_t ldb, int64_t k, int64_t n,
                                               unsigned long long* sums_re, unsigned long long* sums_im, hipStream_t st);
// Slice products of the pairs p + q <= s + 1 with the FP64 sum. mode 0: FP64 sum; 1: double-double sum
// into C, C_lo; 2: the four real products of a complex one in one launch (no k-blocking: block_steps == 0),
// real part formed in the plane Zr, imaginary part in the plane C, result interleaved in Cz.
hipError_t launch_slice_gemm(const GemmArgs& args, int s, int mode, hipStream_t st);
// Slice-count scan: adds, for s = 1 .. 16, the mantissa bits s slices would lose into sums[s - 1].
hipError_t launch_loss_scan_rows(const double* A, int64_t lda, int inc, int64_t m, int64_t k,
                                 unsigned long long* sums, hipStream_t st);
hipError_t launch_loss_scan_cols(const double* B, int64_t ldb, int inc, int64_t k, int64_t n,
                                 unsigned long long* colmax, unsigned long long* sums, hipStream_t st);
// Both planes of an interleaved complex operand (k x n complex elements, ldb in complex elements) by columns; colmax: 2 n entries.
hipError_t launch_loss_scan_cols_complex(const double* B, int64_t ldb, int64_t k, int64_t n, unsigned long long* colmax,
                                         unsigned long long* sums_re, unsigned long long* sums_im, hipStream_t st);
// C = beta C (C = +0 if beta == 0, without reading C) on an m x n row-major array.
hipError_t launch_scale_f64(double* C, int64_t ldc, int64_t m, int64_t n, double beta, hipStream_t st);
// Complex update on rows x cols row-major arrays of interleaved (re, im) doubles, leading
// dimensions in complex elements: t = alpha T (T == nullptr: no product term), u = beta C
// (beta == 0: C is not read), C = t + u, each complex product as RN(RN(ar xr) - RN(ai xi)),
// RN(RN(ar xi) + RN(ai xr)). T may be C itself.
hipError_t launch_zaxpby(const double* T, int64_t ldt, double* C, int64_t ldc, int64_t rows, int64_t cols,
                         double ar, double ai, double br, double bi, hipStream_t st);
hipError_t launch_fill_u64(unsigned long long* p, int64_t count, unsigned long long v, hipStream_t st);
hipError_t launch_fill_f64(double* C, int64_t ldc, int c_inc, int64_t m, int64_t n, double v,
                           hipStream_t st);
hipError_t launch_fill_i32(int32_t* P, int64_t ldp, int64_t m, int64_t n, int32_t v, hipStream_t st);

}  // namespace ozimmu
