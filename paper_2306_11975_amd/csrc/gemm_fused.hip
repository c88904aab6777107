// Slice products with the FP64 sum kept in registers, for short inner dimensions.
//
// Same computation as the general slice-product kernel (Algorithm "Ozaki scheme on IMMU": for
// each diagonal d = s+1 .. 2 the exact integer sum S_d of the slice products with p + q = d, then
// acc = RN(acc + S_d 2^(-7d)) least significant diagonal first and G = 2^(EA_i + EB_j) acc), but
// a finished diagonal is folded into an FP64 register tile at once instead of being parked in
// the workspace. When k is small the parked INT32 matrices (8 bytes of traffic per element and
// diagonal) cost more than the matrix-core work itself (the accumulation of the products is the
// memory-bound part, Section 4.3); here the only traffic besides the slices is C.
//
// Two shapes of the same kernel:
//  * one product, C = G: 8 wavefronts (4 x 2) on a 256 x 128 tile, 64 x 64 per wavefront
//    (64 INT32 accumulators + 64 FP64 sums per lane);
//  * two products, C = G1 +- G2 (one part of a complex product, Section 4.4): 8 wavefronts
//    (2 x 4) on a 128 x 128 tile, 64 x 32 per wavefront (32 accumulators, 32 sums, 32 values
//    of the finished first product), so that neither product ever exists in memory.
// A step moves 128 bytes of k of the A rows and B rows of the tile (parts of two 16 KiB blocks
// of each slice tensor) into one of three or four LDS buffers with direct global->LDS loads,
// two or three steps ahead of the matrix cores; one barrier per step, before its last quarter,
// publishes the next buffer while the fragments of the current one are already in registers.
#include "mfma_common.h"

namespace ozimmu {
namespace {

constexpr int kFLdsBudget = 144 * 1024;

constexpr int kFBlocks = 2;            // 64-byte k-blocks per pipeline step (k is padded to 128)
constexpr int kFSlabs = 2 * kFBlocks;  // 32-wide MFMA slabs per step

template <int WM, int WN, int TM, int TN, bool DUAL>
struct FusedShape {
    static constexpr int kRows = WM * TM * 32, kCols = WN * TN * 32;
    static constexpr int kABytes = kRows * kStep, kBBytes = kCols * kStep;   // per k-block
    static constexpr int kStageBytes = kFBlocks * (kABytes + kBBytes);
    // with so little matrix-core work per step the loads are requested as many steps ahead as
    // LDS allows (3 x 48 KiB or 4 x 32 KiB)
    static constexpr int kStages = kFLdsBudget / kStageBytes > 4 ? 4 : kFLdsBudget / kStageBytes;
    static constexpr int kLds = kStages * kStageBytes;
    static constexpr int kLA = kABytes / 8 / 1024, kLB = kBBytes / 8 / 1024;  // 1 KiB direct loads per wavefront and k-block
    static constexpr int kLoads = kFBlocks * (kLA + kLB);                     // per wavefront and step
    static constexpr int kRowsBeforeBarrier = (kFSlabs - 1) * TM;             // MFMA rows of a step ahead of its barrier
    static constexpr int kLoads0 = kLoads < kRowsBeforeBarrier ? kLoads : kRowsBeforeBarrier;
    static_assert(WM * WN == 8, "eight wavefronts");
    static_assert(kStages >= 3 && (kStages - 1) * kLoads < 64, "vmcnt is a 6-bit counter");
    static_assert(kLoads - kLoads0 <= TM, "one load per MFMA row");
    static_assert(kLA >= 1 && kLB >= 1 && kTile % kRows == 0 && kTile % kCols == 0, "tile shape");
};

template <int WM, int WN, int TM, int TN, bool DUAL>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void fused_gemm_kernel(const GemmArgs g) {
    using Sh = FusedShape<WM, WN, TM, TN, DUAL>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int tiles_mr = g.tiles_m * (kTile / Sh::kRows), tiles_nc = g.tiles_n * (kTile / Sh::kCols);

    int tmr, tnc;
    tile_of_block(blockIdx.x, tiles_mr, tiles_nc, tmr, tnc);

    const int s = g.num_slices;
    const int ks_end = g.k_pad / (kStep * kFBlocks);   // steps per pair

    // source of this wavefront's share of the A rows and B rows of the tile inside block (.., ks = 0)
    const unsigned ld_lane_off = (unsigned)lane * 16u;
    const int64_t a_off = (int64_t)((tmr * Sh::kRows) / kTile) * (g.k_pad / kStep) * kBlockBytes + ((tmr * Sh::kRows) % kTile) * kStep +
                          wave * (Sh::kLA * 1024);
    const int64_t b_off = (int64_t)((tnc * Sh::kCols) / kTile) * (g.k_pad / kStep) * kBlockBytes + ((tnc * Sh::kCols) % kTile) * kStep +
                          wave * (Sh::kLB * 1024);
    const unsigned lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char*)lds;

    const int rd_row = lane & 31;
    const int rd_half = lane >> 5;
    const int rd_sw = (lane >> 2) & 3;
    const int a_rd = (wm * TM * 32 + rd_row) * kStep;
    const int b_rd = kFBlocks * Sh::kABytes + (wn * TN * 32 + rd_row) * kStep;

    // walk over (product, diagonal, pair, k-step): diagonals s+1 .. 2, pairs (1, d-1) .. (d-1, 1).
    // The source addresses of this wavefront's loads are carried along: within a pair the next
    // step is the next block of both slice tensors, so the scalar unit has one addition per
    // operand and step to do (a step has only a few MFMAs to hide address arithmetic behind).
    struct Pos { int prod, d, p, ks; const int8_t* pa; const int8_t* pb; };
    auto locate = [&](Pos& x) {
        const int8_t* sa = (DUAL && x.prod) ? g.SA2 : g.SA;
        const int8_t* sb = (DUAL && x.prod) ? g.SB2 : g.SB;
        x.pa = sa + a_off + (int64_t)(x.p - 1) * g.a_slice_stride;
        x.pb = sb + b_off + (int64_t)(x.d - x.p - 1) * g.b_slice_stride;
    };
    auto advance = [&](Pos& x) -> bool {
        if (++x.ks < ks_end) {
            x.pa += kFBlocks * kBlockBytes;
            x.pb += kFBlocks * kBlockBytes;
            return true;
        }
        x.ks = 0;
        if (++x.p >= x.d) {
            x.p = 1;
            if (--x.d < 2) {
                x.d = s + 1;
                if (!DUAL || ++x.prod >= 2) return false;
            }
        }
        locate(x);
        return true;
    };
    // One of the kLoads direct loads of a step. Per k-block: `w` < kLA copies KiB `w` of this
    // wavefront's share of the A rows, the others the same of the B rows.
    auto issue_load = [&](const Pos& x, int buf, int which) {
        const int blk = which / (Sh::kLA + Sh::kLB), w = which % (Sh::kLA + Sh::kLB);
        const unsigned dst = lds_base + (unsigned)buf * Sh::kStageBytes;
        if (w < Sh::kLA) {
            dma_load16(x.pa + blk * kBlockBytes + w * 1024, ld_lane_off,
                       dst + blk * Sh::kABytes + (wave * Sh::kLA + w) * 1024);
        } else {
            const int i = w - Sh::kLA;
            dma_load16(x.pb + blk * kBlockBytes + i * 1024, ld_lane_off,
                       dst + kFBlocks * Sh::kABytes + blk * Sh::kBBytes + (wave * Sh::kLB + i) * 1024);
        }
    };
    auto issue_step = [&](const Pos& x, int buf) {
#pragma unroll
        for (int w = 0; w < Sh::kLoads; ++w) issue_load(x, buf, w);
    };
    // Past the end of the walk the last step is requested again (into a buffer nobody reads any
    // more), so that the number of loads in flight, which the vmcnt of the step barrier counts
    // on, is the same in every step.
    auto advance_clamped = [&](Pos& x) {
        Pos cand = x;
        if (advance(cand)) x = cand;
    };
    auto read_frags = [&](v4i (&fa)[TM], v4i (&fb)[TN], int buf, int slab) {
        const unsigned char* base = lds + buf * Sh::kStageBytes;
        const int blk = slab >> 1, kk = slab & 1;
        const int col = (((kk << 1) | rd_half) ^ rd_sw) << 4;
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[j] = *reinterpret_cast<const v4i*>(base + blk * Sh::kBBytes + b_rd + j * 32 * kStep + col);
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const v4i*>(base + blk * Sh::kABytes + a_rd + i * 32 * kStep + col);
    };

    // prologue: steps 0 .. kStages-2 requested, step 0 awaited and published
    Pos nxt = {0, s + 1, 1, 0, nullptr, nullptr};
    locate(nxt);
    issue_step(nxt, 0);
#pragma unroll
    for (int b = 1; b < Sh::kStages - 1; ++b) {
        advance_clamped(nxt);
        issue_step(nxt, b);
    }
    wait_loads_and_barrier<(Sh::kStages - 2) * Sh::kLoads>();
    v4i fa[2][TM], fb[2][TN];   // fragments of the slab in the matrix cores and of the next one
    read_frags(fa[0], fb[0], 0, 0);

    // accumulator layout of the 32x32 MFMA: lane holds column (lane % 32); register r holds
    // row 8 (r / 4) + 4 (lane / 32) + r % 4.
    const int row0 = tmr * Sh::kRows + wm * TM * 32 + 4 * rd_half;
    const int col0 = tnc * Sh::kCols + wn * TN * 32 + rd_row;

    double sum[TM][TN][16];
    double first[DUAL ? TM : 1][DUAL ? TN : 1][16];   // the finished first product, scaled
    int buf = 0;                     // LDS buffer of the step in the matrix cores
    int prev = Sh::kStages - 1;      // the buffer released at the previous barrier
#pragma unroll 1
    for (int prod = 0; prod < (DUAL ? 2 : 1); ++prod) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int u = 0; u < 16; ++u) sum[i][j][u] = 0.0;
#pragma unroll 1
        for (int d = s + 1; d >= 2; --d) {
            v16i acc[TM][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = acc_zero();

            const int steps = (d - 1) * ks_end;
#pragma unroll 1
            for (int t = 0; t < steps; ++t) {
                const int nbuf = buf + 1 == Sh::kStages ? 0 : buf + 1;
                // The loads of the step kStages-1 ahead go into the buffer released at the previous
                // barrier, one after each MFMA row: the texture-address unit takes about 18 cycles
                // per wave-wide load and a wavefront stalls at issue while it is busy, so a burst
                // of loads would serialise with the matrix-core work.
                advance_clamped(nxt);
#pragma unroll
                for (int sl = 0; sl < kFSlabs; ++sl) {
                    if (sl + 1 < kFSlabs) {
                        read_frags(fa[(sl + 1) & 1], fb[(sl + 1) & 1], buf, sl + 1);
                    } else {
                        // before the last slab: every wavefront has read its last fragments of this
                        // buffer and its loads of the next step have landed (those of the steps
                        // after may still be in flight)
                        wait_loads_and_barrier<(Sh::kStages - 3) * Sh::kLoads + Sh::kLoads0>();
                        read_frags(fa[0], fb[0], nbuf, 0);
                    }
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[sl & 1][i], fb[sl & 1][j], acc[i][j], 0, 0, 0);
                        if (sl * TM + i < Sh::kLoads) issue_load(nxt, prev, sl * TM + i);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                prev = buf;
                buf = nbuf;
            }
            // fold the finished diagonal: exact conversion, exact power-of-two scale, one rounded add
            // (the product inside the fused multiply-add is exact, so it rounds exactly like the add)
            const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * d) << 52);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int u = 0; u < 16; ++u) sum[i][j][u] = fma((double)acc_read(acc[i][j][u]), sc, sum[i][j][u]);
        }
        if (DUAL && prod == 0) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = col0 + j * 32;
                const int eb = col < g.n ? g.EB[col] : 0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const int row = row0 + i * 32 + 8 * (u >> 2) + (u & 3);
                        first[i][j][u] = ldexp(sum[i][j][u], (row < g.m ? g.EA[row] : 0) + eb);
                    }
            }
        }
    }
    // direct loads of the clamped tail may still be in flight: they must land before this
    // workgroup's LDS can be handed to another one
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    const int32_t* ea = DUAL ? g.EA2 : g.EA;
    const int32_t* ebp = DUAL ? g.EB2 : g.EB;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = col0 + j * 32;
        if (col >= g.n) continue;
        const int eb = ebp[col];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int row = row0 + i * 32 + 8 * (u >> 2) + (u & 3);
                if (row < g.m) {
                    double val = ldexp(sum[i][j][u], ea[row] + eb);
                    if (DUAL) val = g.dual == 2 ? first[i][j][u] - val : first[i][j][u] + val;
                    double* c = g.C + (int64_t)row * g.ldc + (int64_t)col * g.c_inc;
                    if (g.c_mode == 0) *c = val;
                    else if (g.c_mode == 1) *c = *c + val;
                    else if (g.c_mode == 2) *c = *c - val;
                    else {   // BLAS update: RN(alpha G), then RN(RN(alpha G) + RN(beta C)); C is not read if beta == 0
                        double v = g.alpha * val;
                        if (g.beta != 0.0) v = v + g.beta * *c;
                        *c = v;
                    }
                }
            }
    }
}

template <int WM, int WN, int TM, int TN, bool DUAL>
hipError_t launch_shape(const GemmArgs& args, hipStream_t st) {
    using Sh = FusedShape<WM, WN, TM, TN, DUAL>;
    const int blocks = args.tiles_m * (kTile / Sh::kRows) * args.tiles_n * (kTile / Sh::kCols);
    if (blocks == 0) return hipSuccess;
    auto kernel = &fused_gemm_kernel<WM, WN, TM, TN, DUAL>;
    hipError_t e = allow_dynamic_lds<&fused_gemm_kernel<WM, WN, TM, TN, DUAL>>(Sh::kLds);
    if (e != hipSuccess) return e;
    kernel<<<dim3(blocks), dim3(512), Sh::kLds, st>>>(args);
    return hipGetLastError();
}

}  // namespace

bool fused_gemm_applies(const GemmArgs& args, bool wide) {
    return !wide && args.pair_p == 0 && args.k_pad <= kFusedMaxK && args.kc_begin == 0 &&
           args.kc_end * kChunk == args.k_pad;
}

hipError_t launch_fused_gemm(const GemmArgs& args, hipStream_t st) {
    if (args.dual) return launch_shape<2, 4, 2, 1, true>(args, st);
    // few tiles: the smaller tile shape puts twice as many workgroups on the chip
    if (args.tiles_m * args.tiles_n * 2 <= 128) return launch_shape<2, 4, 2, 1, false>(args, st);
    return launch_shape<4, 2, 2, 2, false>(args, st);
}

}  // namespace ozimmu
