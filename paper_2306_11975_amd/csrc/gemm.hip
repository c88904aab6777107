// Slice products on the CDNA4 INT8 matrix cores with the FP64 sum fused in
// (the pair loop of the IMMU algorithm with its product and summing-up steps, Section 3.1).
//
// One workgroup (8 wavefronts, two per SIMD) owns a 256 x 256 tile of C for the whole computation. It walks
// the anti-diagonals d = s+1 .. 2 and, inside a diagonal, the pairs (p, d-p) and the k-steps,
// accumulating everything that shares the scale 2^(-7d) into the same INT32 registers
// (integer addition is exact, so a diagonal is one long INT8 dot product of length (d-1) k).
// A finished diagonal leaves the registers as one coalesced INT32 store into the workspace; at
// the end every thread reads its own values back, adds the diagonals in the fixed order
// least-significant first, applies 2^(EA_i + EB_j) and writes C. When a diagonal is longer
// than 2^17 products (INT32 could overflow), the registers are flushed into INT64 sums in the
// workspace every 2^17 products instead (k-blocking, cf. Section 2.4 on splitting long k).
//
// Data path: the walk over (diagonal, pair, k) is cut into steps of 64 along k. A step moves
// global -> LDS directly (global_load_lds_dwordx4, no staging registers; the slice tensors are
// stored as ready-made LDS images, so every load is a linear run of full 128-byte lines, which
// keeps the number of requests the vector L1 must track per byte at its minimum) into one of
// kStages LDS buffers, kStages steps ahead of the matrix cores, so that an L2 miss has
// several step times to arrive; LDS -> registers with 16-byte reads, XOR-swizzled so that the
// 16 lanes the LDS serves per clock hit 16 distinct bank groups; registers ->
// v_mfma_i32_32x32x32_i8.
// Each wavefront computes 128 x 64 outputs as 4 x 2 MFMA tiles (128 accumulator registers), so
// that two wavefronts fit on a SIMD. The two take turns: one issues the 16 MFMAs of a step
// from fragments it holds in registers while the other reads its next fragments and issues
// its direct loads (two phases and two barriers per step, see the main loop).
#include "ozimmu_internal.h"

#include "mfma_common.h"

namespace ozimmu {
namespace {

constexpr int kStepsPerChunk = kChunk / kStep;        // the API counts k in chunks of kChunk
constexpr int kStages = 4;                            // LDS buffers: loads get kStages - 2 steps to land (3 buffers: 9 % slower at 8192^3; 5: no gain)
constexpr int kTileBytes = kBlockBytes;               // one operand tile of one step: 16 KiB
constexpr int kStageBytes = 2 * kTileBytes;           // A tile + B tile
constexpr int kLdsBytes = kStages * kStageBytes;
constexpr int kPairLdsBytes = 128 * kTile * 4;        // staging of the raw INT32 tile in pair mode
constexpr int kLdsAlloc = kLdsBytes > kPairLdsBytes ? kLdsBytes : kPairLdsBytes;
constexpr int kBlockSteps = OZIMMU_INT32_BLOCK / kStep;
constexpr int kWavesM = 2, kWavesN = 4;               // wavefront grid inside the workgroup
constexpr int kWaves = kWavesM * kWavesN;
constexpr int kThreads = 64 * kWaves;
constexpr int kTM = kTile / kWavesM / 32;             // 32x32 MFMA tiles per wavefront along m (4)
constexpr int kTN = kTile / kWavesN / 32;             // ... along n (2)
constexpr int kWaveShare = kBlockBytes / kWaves;      // bytes of each operand block a wavefront copies per step
constexpr int kLoadsPerOperand = kWaveShare / 1024;   // wave-wide 1 KiB direct loads per operand and step
constexpr int kLoadsPerStep = 2 * kLoadsPerOperand;   // direct loads per wavefront and step
constexpr int kResidentTiles = 256;                   // workgroups the chip runs at a time (one per CU)
static_assert(kStages >= 3 && kStages <= 5, "LDS budget");

// One element of the result: C (op)= 2^(EA_i + EB_j) * sum, with the combine mode of the call.
__device__ __forceinline__ void write_c_element(const GemmArgs& g, int row, int col, int eb, double sum) {
    if (row < g.m && col < g.n) {
        const double val = ldexp(sum, g.EA[row] + eb);
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

// Fixed-order FP64 sum of one macro tile: the INT32 diagonal sums come back from the workspace in
// the order the accumulator registers were stored (thread t of the 512 reads what thread t wrote),
// least significant diagonal first.
__device__ __forceinline__ void final_sum_narrow(const GemmArgs& g, int tile_id, int num_tiles, int row0, int col0,
                                                 unsigned lane_off16) {
    const int s = g.num_slices;
#pragma unroll 1
    for (int ij = 0; ij < kTM * kTN; ++ij) {
        const int i = ij / kTN, j = ij % kTN;
        const int col = col0 + j * 32;
        const int eb = col < g.n ? g.EB[col] : 0;
        double sum[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) sum[u] = 0.0;
        // all 16 accumulators of one MFMA tile at once: four independent 16-byte loads per
        // diagonal, several diagonals in flight
#pragma unroll 4
        for (int d = s + 1; d >= 2; --d) {
            const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * d) << 52);
            const unsigned char* src = reinterpret_cast<const unsigned char*>(g.D) +
                                       ((int64_t)(d - 2) * num_tiles + tile_id) * (int64_t)(kTileElems * 4);
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                v4i v = *reinterpret_cast<const v4i*>(src + (ij * 4 + r4) * (kThreads * 16) + lane_off16);
#pragma unroll
                for (int u = 0; u < 4; ++u) sum[4 * r4 + u] = fma((double)v[u], sc, sum[4 * r4 + u]);   // exact product: rounds like the add
            }
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) write_c_element(g, row0 + i * 32 + 8 * (u >> 2) + (u & 3), col, eb, sum[u]);
    }
}

struct Job {  // one k-step of one slice pair, with this wave's source addresses for it
    int d, p, ks;
    const int8_t* pa;
    const int8_t* pb;
};

template <bool WIDE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWaves / 4, kWaves / 4)))
void slice_gemm_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
    const int wm = wave / kWavesN, wn = wave % kWavesN;

    // Small problems have fewer macro tiles than the chip has CUs; then several workgroups share a
    // tile, each taking a subset of its diagonals (diag_mask), and a second kernel adds them up.
    // In that case the grid is 8 XCDs x groups x (largest tile run of an XCD): an XCD first walks
    // its run of tiles for group 0, then for group 1, ..., so that the workgroups resident on it at
    // any time still work on neighbouring tiles and the same slice pairs; surplus workgroups
    // leave at once.
    const int groups = g.split_groups > 1 ? g.split_groups : 1;
    int tm, tn, group = 0;
    if (groups > 1) {
        const int slot = (int)blockIdx.x >> 3;
        const int per_xcd = (g.tiles_m * g.tiles_n + 7) >> 3;
        group = slot / per_xcd;
        const int tile_slot = slot - group * per_xcd;
        int first, count;
        xcd_tile_range((int)blockIdx.x & 7, g.tiles_m * g.tiles_n, first, count);
        if (tile_slot >= count) return;
        tile_of_logical(first + tile_slot, g.tiles_m, g.tiles_n, tm, tn);
    } else {
        tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, tm, tn);
    }
    const int tile_id = tm * g.tiles_n + tn;
    const int num_tiles = g.tiles_m * g.tiles_n;

    // The diagonals this workgroup walks, as a bit mask (bit d = diagonal d), highest first.
    const bool pair_mode = g.pair_p > 0;
    const unsigned diag_mask = pair_mode ? 1u << (g.pair_p + g.pair_q)
                               : groups > 1 ? g.diag_mask[group] : (1u << (g.num_slices + 2)) - 4u;
    auto next_diag = [&](int d) -> int {   // the next lower diagonal in the mask, 0 if none
        const unsigned below = diag_mask & ((1u << d) - 1u);
        return below ? 31 - __builtin_clz(below) : 0;
    };
    const int d_first = 31 - __builtin_clz(diag_mask);
    const int ks_begin = g.kc_begin * kStepsPerChunk, ks_end = g.kc_end * kStepsPerChunk;

    // global -> LDS. The slice tensors are stored in blocks of 256 rows x 64 bytes that already
    // are the LDS image of one operand tile of one step (16-byte columns swizzled with bits 2..3
    // of the row: the LDS of gfx950 serves 16 lanes x 16 bytes per clock from 64 banks, and with
    // this swizzle the 16 rows a ds_read_b128 reads together fall into 16 distinct bank groups).
    // A wave-wide direct load copies 1 KiB; wave w copies bytes [kWaveShare w, kWaveShare (w+1))
    // of the A block and of the B block, every load a run of eight full 128-byte lines.
    const unsigned ld_lane_off = (unsigned)lane * 16u;
    const int64_t steps_total = g.k_pad / kStep;
    const int8_t* a_tile = g.SA + (int64_t)tm * steps_total * kBlockBytes + wave * kWaveShare;
    const int8_t* b_tile = g.SB + (int64_t)tn * steps_total * kBlockBytes + wave * kWaveShare;
    const unsigned lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char*)lds;
    const unsigned ld_lds_off = lds_base + (unsigned)wave * (unsigned)kWaveShare;

    // LDS -> MFMA operands: lane reads row (lane % 32) of a 32-row block, 16-byte column 2 kk + lane / 32
    const int rd_row = lane & 31;
    const int rd_half = lane >> 5;
    const int a_rd = (wm * 128 + rd_row) * kStep;
    const int b_rd = kTileBytes + (wn * 32 * kTN + rd_row) * kStep;
    const int rd_sw = (lane >> 2) & 3;

    const unsigned lane_off16 = (unsigned)tid * 16u;

    // One direct load of a step: `which` < kLoadsPerOperand copies KiB `which` of this wave's
    // share of the A block, the others the same of the B block.
    auto issue_load = [&](const Job& jb, int buf, int which) {
        const int i = which % kLoadsPerOperand;
        if (which < kLoadsPerOperand)
            dma_load16(jb.pa + i * 1024, ld_lane_off, ld_lds_off + (unsigned)buf * kStageBytes + i * 1024);
        else
            dma_load16(jb.pb + i * 1024, ld_lane_off, ld_lds_off + (unsigned)buf * kStageBytes + kTileBytes + i * 1024);
    };
    auto issue_loads = [&](const Job& jb, int buf, int first, int last) {
#pragma unroll
        for (int w = first; w < last; ++w) issue_load(jb, buf, w);
    };
    // Fragment read number f of one 32-wide k-slab, in the order the slab's MFMAs need them:
    // B fragments 0..kTN-1 first, then A fragments 0..kTM-1.
    auto read_one = [&](v4i (&a)[kTM], v4i (&b)[kTN], int buf, int kk, int f) {
        const unsigned char* base = lds + buf * kStageBytes;
        const int col = (((kk << 1) | rd_half) ^ rd_sw) << 4;
        if (f < kTN) b[f] = *reinterpret_cast<const v4i*>(base + b_rd + f * 32 * kStep + col);
        else a[f - kTN] = *reinterpret_cast<const v4i*>(base + a_rd + (f - kTN) * 32 * kStep + col);
    };
    auto read_frags = [&](v4i (&a)[kTM], v4i (&b)[kTN], int buf, int kk) {
#pragma unroll
        for (int f = 0; f < kTM + kTN; ++f) read_one(a, b, buf, kk, f);
    };
    auto locate = [&](Job& jb) {  // source addresses of the first step of pair (jb.p, jb.d - jb.p)
        jb.pa = a_tile + (int64_t)(jb.p - 1) * g.a_slice_stride + (int64_t)jb.ks * kBlockBytes;
        jb.pb = b_tile + (int64_t)(jb.d - jb.p - 1) * g.b_slice_stride + (int64_t)jb.ks * kBlockBytes;
    };
    auto advance = [&](Job& jb) -> bool {  // false when the walk is over
        if (++jb.ks < ks_end) {   // next step of the same pair: the next block of both tensors
            jb.pa += kBlockBytes;
            jb.pb += kBlockBytes;
            return true;
        }
        jb.ks = ks_begin;
        if (pair_mode || ++jb.p >= jb.d) {
            jb.d = next_diag(jb.d);
            jb.p = 1;
            if (jb.d == 0) return false;
        }
        locate(jb);
        return true;
    };
    // At the end of the walk the iterator stops advancing and the last step is simply loaded
    // again into a buffer nobody reads any more: the number of loads in flight stays the same in
    // every step, which is what the vmcnt of the step barrier counts on, and the loop body needs
    // no branch around the loads.
    auto advance_clamped = [&](Job& jb) {
        Job cand = jb;
        if (advance(cand)) jb = cand;
    };

    // INT32 registers -> workspace (narrow: plain store of a finished diagonal)
    auto store_diag32 = [&](v16i (&acc)[kTM][kTN], int d) {
        unsigned char* base = reinterpret_cast<unsigned char*>(g.D) +
                              ((int64_t)(d - 2) * num_tiles + tile_id) * (int64_t)(kTileElems * 4);
        const unsigned off = lane_off16 + opaque_zero();
#pragma unroll
        for (int i = 0; i < kTM; ++i)
#pragma unroll
            for (int j = 0; j < kTN; ++j)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    v4i v = {acc_read(acc[i][j][4 * r4]), acc_read(acc[i][j][4 * r4 + 1]), acc_read(acc[i][j][4 * r4 + 2]),
                             acc_read(acc[i][j][4 * r4 + 3])};
                    *reinterpret_cast<v4i*>(base + ((i * kTN + j) * 4 + r4) * (kThreads * 16) + off) = v;
                    __builtin_amdgcn_sched_barrier(0);  // keep register pressure flat
                }
    };
    // INT32 registers -> INT64 sums (wide: k-blocking)
    auto flush_diag64 = [&](v16i (&acc)[kTM][kTN], int d, bool first) {
        unsigned char* base = reinterpret_cast<unsigned char*>(g.D) +
                              ((int64_t)(d - 2) * num_tiles + tile_id) * (int64_t)(kTileElems * 8);
        const unsigned off = lane_off16 + opaque_zero();
#pragma unroll
        for (int i = 0; i < kTM; ++i)
#pragma unroll
            for (int j = 0; j < kTN; ++j)
#pragma unroll
                for (int r2 = 0; r2 < 8; ++r2) {
                    v2l v = {(long long)acc_read(acc[i][j][2 * r2]), (long long)acc_read(acc[i][j][2 * r2 + 1])};
                    v2l* q = reinterpret_cast<v2l*>(base + ((i * kTN + j) * 8 + r2) * (kThreads * 16) + off);
                    if (!first) v += *q;
                    *q = v;
                    __builtin_amdgcn_sched_barrier(0);
                }
    };
    auto zero_acc = [&](v16i (&acc)[kTM][kTN]) {
#pragma unroll
        for (int i = 0; i < kTM; ++i)
#pragma unroll
            for (int j = 0; j < kTN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = acc_zero();
    };

    // accumulator layout of the 32x32 MFMA: lane holds column (lane % 32); register r holds
    // row 8 (r / 4) + 4 (lane / 32) + r % 4.
    const int row0 = tm * kTile + wm * 128 + 4 * rd_half;
    const int col0 = tn * kTile + wn * 32 * kTN + rd_row;
    const int s = g.num_slices;

    // Pair mode: raw INT32 tile -> row-major P. The tile is staged through LDS (free once the
    // k-walk is over) in two halves of 128 rows so that the bounds-checked stores are a rolled
    // loop along rows of P.
    auto write_pair = [&](v16i (&acc)[kTM][kTN]) {
        int* tile = reinterpret_cast<int*>(lds);  // [128][256] INT32 = 128 KiB
        const unsigned tbase = (unsigned)(4 * rd_half * kTile + wn * 32 * kTN + rd_row) + opaque_zero();
        asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");  // no direct load may still land here
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if (wm == half) {
#pragma unroll
                for (int i = 0; i < kTM; ++i)
#pragma unroll
                    for (int j = 0; j < kTN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            tile[tbase + (i * 32 + 8 * (r >> 2) + (r & 3)) * kTile + j * 32] = acc_read(acc[i][j][r]);
                            if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                        }
            }
            __syncthreads();
#pragma unroll 1
            for (int rr = tid / kTile; rr < 128; rr += kThreads / kTile) {
                const int row = tm * kTile + half * 128 + rr;
                const int col = tn * kTile + (tid % kTile);
                if (row < g.m && col < g.n) g.P[(int64_t)row * g.ldp + col] = tile[rr * kTile + (tid % kTile)];
            }
            __syncthreads();
        }
    };
    auto write_c = [&](int row, int col, int eb, double sum) { write_c_element(g, row, col, eb, sum); };
    auto final_narrow = [&]() { final_sum_narrow(g, tile_id, num_tiles, row0, col0, lane_off16); };
    auto final_wide = [&]() {
#pragma unroll 1
        for (int ij = 0; ij < kTM * kTN; ++ij) {
            const int i = ij / kTN, j = ij % kTN;
            const int col = col0 + j * 32;
            const int eb = col < g.n ? g.EB[col] : 0;
#pragma unroll 1
            for (int r2 = 0; r2 < 8; ++r2) {
                double sum[2] = {0.0, 0.0};
                for (int d = s + 1; d >= 2; --d) {
                    const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * d) << 52);
                    const unsigned char* src = reinterpret_cast<const unsigned char*>(g.D) +
                                               ((int64_t)(d - 2) * num_tiles + tile_id) * (int64_t)(kTileElems * 8);
                    v2l v = *reinterpret_cast<const v2l*>(src + (ij * 8 + r2) * (kThreads * 16) + lane_off16);
                    sum[0] = sum[0] + (double)v[0] * sc;
                    sum[1] = sum[1] + (double)v[1] * sc;
                }
                const int r = 2 * r2;
                write_c(row0 + i * 32 + 8 * (r >> 2) + (r & 3), col, eb, sum[0]);
                write_c(row0 + i * 32 + 8 * (r >> 2) + (r & 3) + 1, col, eb, sum[1]);
            }
        }
    };

    // Pipeline prologue: steps 0 .. kStages-1 are requested; steps 0 and 1 are awaited and published.
    Job nxt = {d_first, pair_mode ? g.pair_p : 1, ks_begin, nullptr, nullptr};   // last step requested
    locate(nxt);
    issue_loads(nxt, 0, 0, kLoadsPerStep);
#pragma unroll
    for (int b = 1; b < kStages; ++b) {
        advance_clamped(nxt);
        issue_loads(nxt, b, 0, kLoadsPerStep);
    }
    wait_loads_and_barrier<(kStages - 2) * kLoadsPerStep>();
    v4i fa0[kTM], fb0[kTN], fa1[kTM], fb1[kTN];   // fragments of the two 32-wide k-slabs of a step
    read_frags(fa0, fb0, 0, 0);
    read_frags(fa1, fb1, 0, 1);

    const int nks = ks_end - ks_begin;
    int buf = 0;                // LDS buffer of the step in the matrix cores
    // One step = two phases. The two halves of the workgroup (wavefronts 0-3 and 4-7, one of each
    // on every SIMD) take turns: while one half issues the 16 MFMAs of a step from fragments it
    // already holds, the other half reads the fragments of its next step from LDS, issues its share
    // of the direct loads and waits for older ones; a barrier ends every phase and the second half
    // runs one phase behind the first. The matrix cores of a SIMD thus always have a wavefront that
    // does nothing but issue MFMAs, and LDS latency, load issue (the texture-address unit takes
    // about 18 cycles per wave-wide load and a wavefront stalls at issue while it is busy) and
    // barrier waits fall on the wavefront that has no MFMA to issue anyway. Memory phase of step u:
    //   read the fragments of step u+1; request step u+kStages into the buffer of step u (both
    //   halves read its fragments at least one barrier ago: the leading half two phases, the
    //   lagging half one phase earlier); wait until this wavefront's loads of step u+2 have landed.
    // Hence when a half reads the fragments of step u+1, every wavefront has confirmed its loads
    // of that step at least one barrier earlier (in its memory phase of step u-1, or the prologue).
    const bool lag = wave >= kWaves / 2;
    auto phase_barrier = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    auto mfma_slab = [&](v16i (&acc)[kTM][kTN], const v4i (&a)[kTM], const v4i (&b)[kTN]) {
#pragma unroll
        for (int i = 0; i < kTM; ++i)
#pragma unroll
            for (int j = 0; j < kTN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    };
    auto run_steps = [&](v16i (&acc)[kTM][kTN], int count) {
        if (lag) phase_barrier();        // fall one phase behind ...
        int t = 0;
        do {
            __builtin_amdgcn_s_setprio(1);   // the wavefront with MFMAs to issue goes first on its SIMD
            mfma_slab(acc, fa0, fb0);
            mfma_slab(acc, fa1, fb1);
            __builtin_amdgcn_s_setprio(0);
            phase_barrier();
            const int nbuf = buf + 1 == kStages ? 0 : buf + 1;
            read_frags(fa0, fb0, nbuf, 0);
            read_frags(fa1, fb1, nbuf, 1);
            advance_clamped(nxt);
            issue_loads(nxt, buf, 0, kLoadsPerStep);
            __builtin_amdgcn_sched_barrier(0);
            wait_loads_and_barrier<(kStages - 2) * kLoadsPerStep>();
            __builtin_amdgcn_sched_barrier(0);
            buf = nbuf;
        } while (++t < count);
        if (!lag) phase_barrier();       // ... and let it catch up: what follows is done by all together
    };

    for (int d = d_first; d != 0; d = next_diag(d)) {
        int jobs = pair_mode ? nks : (d - 1) * nks;
        if (WIDE) {
            // at most 2^17 products per output element may share one INT32 sum
            bool fresh = true;
            do {
                const int run = jobs > kBlockSteps ? kBlockSteps : jobs;
                jobs -= run;
                v16i acc[kTM][kTN];
                zero_acc(acc);
                run_steps(acc, run);
                flush_diag64(acc, d, fresh);
                fresh = false;
            } while (jobs > 0);
        } else {
            v16i acc[kTM][kTN];
            zero_acc(acc);
            run_steps(acc, jobs);
            if (pair_mode) write_pair(acc);
            else store_diag32(acc, d);
        }
    }
    // direct loads of the clamped tail may still be in flight: they must land before this
    // workgroup's LDS can be handed to another one
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (g.skip_final) return;   // uniform: the sums stay in the workspace for a kernel of their own
    if (WIDE) final_wide();
    else if (!pair_mode && groups == 1) final_narrow();
}

// FP64 sum of the stored diagonals as a kernel of its own, for launches in which several
// workgroups shared a macro tile: same thread-to-element mapping as the product kernel.
__global__ __launch_bounds__(kThreads) void diag_sum_kernel(const GemmArgs g) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / kWavesN, wn = wave % kWavesN;
    int tm, tn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, tm, tn);
    const int row0 = tm * kTile + wm * 128 + 4 * (lane >> 5);
    const int col0 = tn * kTile + wn * 32 * kTN + (lane & 31);
    final_sum_narrow(g, tm * g.tiles_n + tn, g.tiles_m * g.tiles_n, row0, col0, (unsigned)tid * 16u);
}

// Double-double sum of the stored diagonal sums (INT32, or INT64 if WIDE), least significant first:
// TwoSum of the running high part and the exact term, error into the low part, FastTwoSum to
// renormalise (Section 2.3.4: summing-up in higher precision). Same thread-to-element mapping as the
// stores of the product kernel.
__device__ __forceinline__ void dd_add(double& h, double& l, double t) {
    const double sh = h + t;
    const double bb = sh - h;
    const double e = (h - (sh - bb)) + (t - bb);
    const double l2 = l + e;
    const double hn = sh + l2;
    l = l2 - (hn - sh);
    h = hn;
}
template <bool WIDE>
__global__ __launch_bounds__(kThreads) void diag_sum_dd_kernel(const GemmArgs g) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / kWavesN, wn = wave % kWavesN;
    int tm, tn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, tm, tn);
    const int tile_id = tm * g.tiles_n + tn, num_tiles = g.tiles_m * g.tiles_n;
    const int row0 = tm * kTile + wm * 128 + 4 * (lane >> 5);
    const int col0 = tn * kTile + wn * 32 * kTN + (lane & 31);
    const int s = g.num_slices;
    const unsigned lane_off16 = (unsigned)tid * 16u;
    constexpr int kPer = WIDE ? 2 : 4;            // values per 16-byte group
    constexpr int kGroupsPerTile = 16 / kPer;     // 16-byte groups per MFMA tile and thread
#pragma unroll 1
    for (int ij = 0; ij < kTM * kTN; ++ij) {
        const int i = ij / kTN, j = ij % kTN;
        const int col = col0 + j * 32;
        if (col >= g.n) continue;
        const int eb = g.EB[col];
#pragma unroll 1
        for (int q = 0; q < kGroupsPerTile; ++q) {
            double h[kPer], l[kPer];
#pragma unroll
            for (int u = 0; u < kPer; ++u) h[u] = l[u] = 0.0;
            for (int d = s + 1; d >= 2; --d) {
                const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * d) << 52);
                const unsigned char* src = reinterpret_cast<const unsigned char*>(g.D) +
                                           ((int64_t)(d - 2) * num_tiles + tile_id) * (int64_t)(kTileElems * (WIDE ? 8 : 4)) +
                                           (ij * kGroupsPerTile + q) * (kThreads * 16) + lane_off16;
                if (WIDE) {
                    const v2l v = *reinterpret_cast<const v2l*>(src);
#pragma unroll
                    for (int u = 0; u < 2; ++u) dd_add(h[u], l[u], (double)v[u] * sc);
                } else {
                    const v4i v = *reinterpret_cast<const v4i*>(src);
#pragma unroll
                    for (int u = 0; u < 4; ++u) dd_add(h[u], l[u], (double)v[u] * sc);
                }
            }
#pragma unroll
            for (int u = 0; u < kPer; ++u) {
                const int r = q * kPer + u;       // accumulator register index 0 .. 15
                const int row = row0 + i * 32 + 8 * (r >> 2) + (r & 3);
                if (row < g.m) {
                    const int e = g.EA[row] + eb;
                    g.C[(int64_t)row * g.ldc + col] = ldexp(h[u], e);
                    g.C_lo[(int64_t)row * g.ldc + col] = ldexp(l[u], e);
                }
            }
        }
    }
}

// Diagonal d costs d - 1 slice products: longest first onto the least loaded group. Returns the
// largest load.
int balance_diagonals(int s, int groups, unsigned* masks) {
    int load[OZIMMU_MAX_SLICES] = {};
    for (int gidx = 0; gidx < groups; ++gidx) masks[gidx] = 0u;
    for (int d = s + 1; d >= 2; --d) {
        int best = 0;
        for (int gidx = 1; gidx < groups; ++gidx)
            if (load[gidx] < load[best]) best = gidx;
        masks[best] |= 1u << d;
        load[best] += d - 1;
    }
    int worst = 0;
    for (int gidx = 0; gidx < groups; ++gidx) worst = load[gidx] > worst ? load[gidx] : worst;
    return worst;
}

}  // namespace

// The chip runs kResidentTiles workgroups at a time. If the tile count is small, or not close to a
// multiple of that, several workgroups share a tile, each taking a balanced subset of its
// diagonals: the group count with the fewest slice products on the critical path (rounds of
// workgroups x products of the most loaded group) is taken; ties go to the smaller count. More
// than (s + 1) / 2 groups cannot be balanced (the longest diagonal alone has s of the
// s (s + 1) / 2 products). Returns the group count and fills masks[group] (bit d = diagonal d).
int plan_tile_sharing(int tiles, int s, unsigned* masks) {
    int groups = 1;
    long best_cost = 0;
    unsigned scratch_masks[OZIMMU_MAX_SLICES];
    for (int cand = 1; cand <= (s + 1) / 2; ++cand) {
        const long rounds = ((long)((tiles + 7) / 8) * 8 * cand + kResidentTiles - 1) / kResidentTiles;
        const long cost = rounds * balance_diagonals(s, cand, scratch_masks) + (cand > 1 ? 1 : 0);
        if (cand == 1 || cost < best_cost) { best_cost = cost; groups = cand; }
    }
    balance_diagonals(s, groups, masks);
    return groups;
}

hipError_t launch_slice_gemm(const GemmArgs& args, bool wide, hipStream_t st) {
    const int blocks = args.tiles_m * args.tiles_n;
    if (blocks == 0) return hipSuccess;
    hipError_t e;
    if (wide) {
        e = allow_dynamic_lds<&slice_gemm_kernel<true>>(kLdsAlloc);
        if (e != hipSuccess) return e;
        slice_gemm_kernel<true><<<dim3(blocks), dim3(kThreads), kLdsAlloc, st>>>(args);
    } else if (args.skip_final) {
        e = allow_dynamic_lds<&slice_gemm_kernel<false>>(kLdsAlloc);
        if (e != hipSuccess) return e;
        slice_gemm_kernel<false><<<dim3(blocks), dim3(kThreads), kLdsAlloc, st>>>(args);
    } else {
        e = allow_dynamic_lds<&slice_gemm_kernel<false>>(kLdsAlloc);
        if (e != hipSuccess) return e;
        const int s = args.num_slices;
        unsigned masks[OZIMMU_MAX_SLICES];
        const int groups = args.pair_p == 0 ? plan_tile_sharing(blocks, s, masks) : 1;
        if (args.pair_p == 0 && groups >= 2) {
            GemmArgs split = args;
            split.split_groups = groups;
            for (int gidx = 0; gidx < groups; ++gidx) split.diag_mask[gidx] = masks[gidx];
            const int per_xcd = (blocks + 7) / 8;   // the largest run of tiles an XCD owns
            slice_gemm_kernel<false><<<dim3(8 * per_xcd * groups), dim3(kThreads), kLdsAlloc, st>>>(split);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            diag_sum_kernel<<<dim3(blocks), dim3(kThreads), 0, st>>>(split);
        } else {
            slice_gemm_kernel<false><<<dim3(blocks), dim3(kThreads), kLdsAlloc, st>>>(args);
        }
    }
    return hipGetLastError();
}

hipError_t launch_diag_sum_dd(const GemmArgs& args, bool wide, hipStream_t st) {
    const int blocks = args.tiles_m * args.tiles_n;
    if (blocks == 0) return hipSuccess;
    if (wide) diag_sum_dd_kernel<true><<<dim3(blocks), dim3(kThreads), 0, st>>>(args);
    else diag_sum_dd_kernel<false><<<dim3(blocks), dim3(kThreads), 0, st>>>(args);
    return hipGetLastError();
}

}  // namespace ozimmu
