// Internal declarations shared by the translation units of libozimmu (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ozimmu.h"

namespace ozimmu {

constexpr int kTile = 256;          // macro tile edge in rows of A / rows of B^T (= OZIMMU_ROW_ALIGN)
constexpr int kChunk = 128;         // granularity of k in the API (= OZIMMU_K_ALIGN)
constexpr int kStep = 64;           // k-extent of one contiguous slice block and of one pipeline step (= OZIMMU_K_STEP)
constexpr int kBlockBytes = kTile * kStep;  // one block of a slice tensor: 256 rows x 64 bytes
constexpr int kTileElems = kTile * kTile;

static inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Arguments of the slice-product kernel. One launch covers every macro tile of C.
struct GemmArgs {
    const int8_t* SA;      // slice tensor of A   (tiled layout, see ozimmu.h)
    const int8_t* SB;      // slice tensor of B^T
    int64_t a_slice_stride;  // bytes between consecutive slices of A
    int64_t b_slice_stride;
    int k_pad;             // padded row length
    int tiles_m, tiles_n;
    int m, n;              // true extent of C
    int num_slices;        // full mode: diagonals num_slices+1 .. 2
    int pair_p, pair_q;    // pair mode (pair_p > 0): only this pair, raw INT32 out
    int kc_begin, kc_end;  // k-range in chunks of kChunk
    void* D;               // per-diagonal integer sums that leave the registers (INT32 or INT64)
    int32_t* P;            // pair mode output, row-major
    int64_t ldp;
    double* C;             // full mode output
    int64_t ldc;           // in doubles
    int c_inc;             // distance in doubles between consecutive columns (2 for a complex plane)
    int c_mode;            // 0: C = G, 1: C = C + G, 2: C = C - G, 3: C = alpha G (+ beta C if beta != 0)
    double alpha, beta;    // c_mode 3 only
    const int32_t* EA;
    const int32_t* EB;
    // several workgroups per macro tile (small problems): workgroup group g of a tile walks the
    // diagonals in diag_mask[g] (bit d = diagonal d) and a second kernel forms the FP64 sum
    int skip_final;                 // leave every diagonal sum in D and write no C (a separate kernel sums)
    double* C_lo;                   // low parts of a double-double result (sum kernel only)
    int split_groups;               // 0 or 1: off
    unsigned diag_mask[OZIMMU_MAX_SLICES];
    // second product of the register-resident kernel (dual != 0): C = G(SA,SB) + G(SA2,SB2) if
    // dual == 1, C = G(SA,SB) - G(SA2,SB2) if dual == 2, each G scaled by its own exponents
    int dual;
    const int8_t* SA2;
    const int8_t* SB2;
    const int32_t* EA2;
    const int32_t* EB2;
};

// negate: emit the slices of -A (-B) instead: same exponents, every slice with the opposite sign
// (how a conjugated operand's imaginary plane is split)
hipError_t launch_split_rows(const double* A, int64_t lda, int inc, int64_t m, int64_t k, int s,
                             int8_t* S, int64_t m_pad, int64_t k_pad, int32_t* E, hipStream_t st,
                             bool negate = false);
hipError_t launch_split_cols(const double* B, int64_t ldb, int inc, int64_t k, int64_t n, int s,
                             int8_t* S, int64_t n_pad, int64_t k_pad, int32_t* E,
                             unsigned long long* colmax, hipStream_t st, bool negate = false);
hipError_t launch_slice_gemm(const GemmArgs& args, bool wide, hipStream_t st);
// How many workgroups share a macro tile for a given tile count and slice count, and which diagonals each takes.
int plan_tile_sharing(int tiles, int s, unsigned* masks);
// Double-double sum of the diagonal sums left in D by a launch with skip_final (C = high, C_lo = low parts).
hipError_t launch_diag_sum_dd(const GemmArgs& args, bool wide, hipStream_t st);
// Variant for short inner dimensions that keeps the FP64 sum in registers (no use of args.D).
constexpr int kFusedMaxK = 1024;
bool fused_gemm_applies(const GemmArgs& args, bool wide);
hipError_t launch_fused_gemm(const GemmArgs& args, hipStream_t st);
// Slice-count scan: adds, for s = 1 .. 16, the mantissa bits s slices would lose into sums[s - 1].
hipError_t launch_loss_scan_rows(const double* A, int64_t lda, int inc, int64_t m, int64_t k,
                                 unsigned long long* sums, hipStream_t st);
hipError_t launch_loss_scan_cols(const double* B, int64_t ldb, int inc, int64_t k, int64_t n,
                                 unsigned long long* colmax, unsigned long long* sums, hipStream_t st);
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
