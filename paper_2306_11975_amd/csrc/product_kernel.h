// Slice products on the CDNA4 INT8 matrix cores with the FP64 sum fused in
// (the pair loop of the IMMU algorithm with its product and summing-up steps, Section 3.1).
//
// Loop nest: "all diagonals resident". A wavefront owns a 32 x 32 patch of C and keeps the exact
// INT32 sums of up to eight anti-diagonals d = p + q of that patch in its accumulation registers
// (16 registers per diagonal) for the whole walk along k. A workgroup of 2 x 4 wavefronts owns a
// 64 x 128 tile. One pipeline step covers 32 positions of k: the 32-row fragments of ALL slices of
// the tile's rows of A and of B^T (6 s KiB) are brought into LDS once, each wavefront reads its
// 2 s fragments (one ds_read_b128 each) and issues the s (s + 1) / 2 MFMAs of all pairs
// p + q <= s + 1, every one into the accumulator of its own diagonal. Integer addition is exact, so
// all pairs of a diagonal share one INT32 sum; nothing but the slices is read and nothing but C is
// written: no product and no diagonal sum ever exists in memory. At the end the diagonals are added
// in the fixed order (least significant first) in FP64, scaled by 2^(EA_i + EB_j), and stored.
//
// More than eight slices: the diagonals are walked in two bands, the upper eight first, then the
// remaining s - 8 (which are exactly the diagonals of the s - 8 slice problem); the FP64 sum of the
// first band waits in registers. Long k (more than 2^17 products per INT32 sum, cf. Section 2.4 on
// splitting long k): every block_steps steps the INT32 sums are added into INT64 sums in the
// workspace (k-blocking) and the FP64 sum is formed from those.
//
// Complex product (kModeComplex, Section 4.4): the workgroup of a tile walks the four real products
// Ar Br, Ai Bi, Ar Bi, Ai Br one after the other; up to eight slices they form one stream of steps whose
// loads run ahead across the product boundaries. After each product its diagonals are folded and the
// result is combined with the part formed so far, which waits in a plane of the workspace (real part:
// Zr, imaginary part: C) and is read back at the L2; the fourth epilogue writes (re, im) pairs.
//
// Data path of a step: global -> LDS with wave-wide direct loads (global_load_lds_dwordx4, no
// staging registers; a fragment is 1 KiB contiguous in memory and in LDS), two or three LDS stages
// (as many as fit 160 KiB);
// LDS -> registers with ds_read_b128 (fragment rows are 32 bytes with the two 16-byte halves
// swapped in rows 8..15 and 24..31, so that any 16 consecutive lanes cover all 64 banks);
// registers -> v_mfma_i32_32x32x32_i8.
#pragma once

#ifndef OZIMMU_TUNE_MAX_STAGES
#define OZIMMU_TUNE_MAX_STAGES 3
#endif

#include "ozimmu_internal.h"

#include "mfma_common.h"

namespace ozimmu {
namespace {

constexpr int kLdsLimit = 160 * 1024;
constexpr int kMaxStages = OZIMMU_TUNE_MAX_STAGES;   // LDS stages at most (loads are requested kMaxStages - 1 steps ahead)

// One band of a walk: the pairs (p, q), 0-based, with E0 <= p + q <= SB - 1 of an SB-slice problem.
template <int SB, int WM, int WN>
struct Band {
    static constexpr int ND = SB < kBand ? SB : kBand;    // resident diagonals
    static constexpr int E0 = SB - ND;                    // lowest one (e = p + q, 0-based; d = e + 2)
    static constexpr int NW = WM * WN;
    static constexpr int NFRAG = SB * (WM + WN);          // fragments per step
    static constexpr int STAGE = NFRAG * kFragBytes;
    // RESIDENT: all 2 SB fragments of a step are held in registers (8 SB of them) and re-read in place
    // for the next step; beyond 11 slices they no longer fit beside the accumulators and the B
    // fragments are streamed through three registers instead.
    static constexpr bool RESIDENT = SB <= 11;
    // 2 x 2 wavefronts with up to nine slices: two workgroups share a compute unit (and its LDS)
    static constexpr bool PAIRED = NW == 4 && SB <= 9;
    static constexpr int FIT = (PAIRED ? kLdsLimit / 2 - 1024 : kLdsLimit) / STAGE;
    static constexpr int NST = !RESIDENT ? 2 : FIT > kMaxStages ? kMaxStages : FIT;
    static constexpr int LDS = NST * STAGE;
    static constexpr int NLOAD = (NFRAG + NW - 1) / NW;   // direct loads per wavefront and step
    static_assert(NST >= 2, "two stages must fit the LDS");
    static_assert(NST * NLOAD < 64, "vmcnt is a 6-bit counter");
    static_assert(NLOAD <= SB, "one direct load per MFMA group");
};

template <int S, int WM, int WN>
struct Shape {
    static constexpr int LDS1 = Band<S, WM, WN>::LDS;
    static constexpr int LDS2 = S > kBand ? Band<(S > kBand ? S - kBand : 1), WM, WN>::LDS : 0;
    static constexpr int LDS = LDS1 > LDS2 ? LDS1 : LDS2;
};

typedef __attribute__((address_space(3))) long long lds_i64;

// What a wavefront needs to know about its place in the walk.
struct Walk {
    unsigned char* lds;      // dynamic LDS segment
    unsigned lds_base;       // its LDS address
    unsigned rd_lane;        // byte offset of this lane's 16 bytes inside a fragment
    int lane, wave, wm, wn;
    int tm, tn;
    int tid;
    lds_i64* switch_table;     // this wavefront's LDS table of source-address changes between products (streams of products only)
};

__device__ __forceinline__ const int8_t* uniform_ptr(const int8_t* p) {
    const unsigned long long v = (unsigned long long)p;
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v >> 32));
    return (const int8_t*)(((unsigned long long)hi << 32) | lo);
}

template <int N>
__device__ __forceinline__ void wait_loads() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ void workgroup_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// The walk of one band over the slabs [g.t_begin, g.t_end), for the products p_begin .. p_end - 1 one
// after the other: sources(p, sa, sb) names the slice tensors of product p, acc[e - E0] receives the
// pairs of diagonal e, after_step(steps done in this product) is called after every step (k-blocking
// hooks in there) and after_product(p) when a product's last step has been issued (it takes the sums
// and clears acc). STREAM (register-resident schedule only, at least NST steps per product): the
// products form one continuous stream of steps and only the first one pays for filling the pipeline.
// Stores that after_product issues may still be in flight when the walk resumes: they share the counter
// of the direct loads, but loads complete in order among themselves, so "at most N operations in flight"
// still proves that every load older than the N youngest has landed; a store in flight can only make
// such a wait longer.
template <int SB, int WM, int WN, bool STREAM, class Sources, class AfterStep, class AfterProduct>
__device__ __forceinline__ void band_walk(v16i (&acc)[kBand], const GemmArgs& g, const Walk& w, int p_begin, int p_end,
                                          Sources&& sources, AfterStep&& after_step, AfterProduct&& after_product) {
    using B = Band<SB, WM, WN>;
    constexpr int E0 = B::E0, NST = B::NST, NLOAD = B::NLOAD;

    // This wavefront's share of the step's fragments: fragment idx = wave + NW jj. Fragments are
    // numbered A(p, i) = p WM + i, then B(q, j) = SB WM + q WN + j, and sit in that order in a
    // stage. A wavefront without a jj-th fragment loads the last one again (same bytes to the same
    // place), so that every wavefront has the same number of loads in flight.
    const int8_t* src[NLOAD];
    unsigned dst[NLOAD];
    auto fragment_index = [&](int jj) __attribute__((always_inline)) -> int {
        const int idx = w.wave + B::NW * jj;
        return idx < B::NFRAG ? idx : B::NFRAG - 1;
    };
    auto fragment_ptr = [&](int prod, int jj) __attribute__((always_inline)) -> const int8_t* {
        const int8_t *sa, *sb;
        sources(prod, sa, sb);
        const int idx = fragment_index(jj);
        if (idx < SB * WM) {
            const int p = idx / WM, i = idx % WM;
            return sa + (int64_t)p * g.a_slice_stride + (int64_t)(w.tm * WM + i) * g.kslabs * kFragBytes;
        }
        const int r = idx - SB * WM;
        const int q = r / WN, j = r % WN;
        return sb + (int64_t)q * g.b_slice_stride + (int64_t)(w.tn * WN + j) * g.kslabs * kFragBytes;
    };
    auto set_sources = [&](int prod) __attribute__((always_inline)) {
#pragma unroll
        for (int jj = 0; jj < NLOAD; ++jj) {
            // wave-uniform by construction; say so, so that they live in scalar registers
            src[jj] = uniform_ptr(fragment_ptr(prod, jj));
            dst[jj] = (unsigned)__builtin_amdgcn_readfirstlane((int)(w.lds_base + (unsigned)fragment_index(jj) * kFragBytes));
        }
    };
    const int steps = g.t_end - g.t_begin;
    wait_loads<0>();   // stores of an earlier product's epilogue must not be counted as direct loads
    // The request side: step ld_t of the product, lane offset voff into its source fragments. Past the
    // last step of the last product the last step is requested again (into a stage nobody reads any
    // more), so that the number of loads in flight never changes.
    const unsigned voff_first = (unsigned)w.lane * 16u + (unsigned)g.t_begin * kFragBytes;
    unsigned voff = voff_first;
    int ld_t = 0;
    auto issue_one = [&](int jj, unsigned stage_off) __attribute__((always_inline)) {
        dma_load16(src[jj], voff, dst[jj] + stage_off);
        if (jj == NLOAD - 1) {   // the step is requested: move on
            if (++ld_t < steps) voff += kFragBytes;
            else --ld_t;
        }
    };
    auto issue = [&](unsigned stage_off) __attribute__((always_inline)) {
#pragma unroll
        for (int jj = 0; jj < NLOAD; ++jj) issue_one(jj, stage_off);
    };
    const unsigned char* rd_a = w.lds + w.wm * kFragBytes + w.rd_lane;
    const unsigned char* rd_b = w.lds + (SB * WM + w.wn) * kFragBytes + w.rd_lane;
    auto read_a = [&](int p, unsigned stage_off) __attribute__((always_inline)) -> v4i {
        return *reinterpret_cast<const v4i*>(rd_a + stage_off + p * WM * kFragBytes);
    };
    auto read_b = [&](int q, unsigned stage_off) __attribute__((always_inline)) -> v4i {
        return *reinterpret_cast<const v4i*>(rd_b + stage_off + q * WN * kFragBytes);
    };

    // Group q of a step = the MFMAs of B fragment q with the A fragments p = pmax(q) .. pmin(q),
    // highest first: a[SB - 1 - q] and b[q] have their last use of the step in group q.
    if constexpr (B::RESIDENT) {
        // All 2 SB fragments of a step live in registers; each is re-read from the stage of the next
        // step as soon as its last MFMA of this step is issued, a whole step before it is needed
        // again. The stage of step t is therefore read during step t - 1 only, and free from the
        // barrier of step t on: it takes the loads of step t + NST, which get NST - 1 steps to land.
        constexpr int AHEAD = NST - 1;
        v4i a[SB], b[SB];
        unsigned cur = 0;
        auto read_all = [&]() __attribute__((always_inline)) {
            static_for<0, SB>([&](auto pc) __attribute__((always_inline)) {
                constexpr int p = decltype(pc)::value;
                a[SB - 1 - p] = read_a(SB - 1 - p, cur);
                b[p] = read_b(p, cur);
            });
        };
        // One step; issue_q(jj, stage) requests this wavefront's jj-th fragment of the step NST ahead.
        auto step = [&](auto&& issue_q, auto await_next) __attribute__((always_inline)) {
            const unsigned nxt = cur + B::STAGE < (unsigned)B::LDS ? cur + B::STAGE : 0u;
            static_for<0, SB>([&](auto qc) __attribute__((always_inline)) {
                constexpr int q = decltype(qc)::value;
                constexpr int pmax = SB - 1 - q, pmin = E0 - q > 0 ? E0 - q : 0;
                static_for<0, pmax - pmin + 1>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int p = pmax - decltype(ic)::value;
                    acc[p + q - E0] = mfma(a[p], b[q], acc[p + q - E0]);
                });
                if constexpr (q == 0) {
                    // the next step has landed everywhere (its fragments may be read from here on) and
                    // every wavefront has read the last fragment of this one: its stage is free
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (decltype(await_next)::value) wait_loads<(AHEAD - 1) * NLOAD>();
                    workgroup_barrier();
                }
                // one direct load per group (NLOAD <= SB): a wavefront stalls while its load is issued,
                // and eight wavefronts that issue all their loads at once queue behind each other
                if constexpr (q < NLOAD) issue_q(q, cur);
                b[q] = read_b(q, nxt);
                a[pmax] = read_a(pmax, nxt);
                __builtin_amdgcn_sched_barrier(0);   // keep the re-reads where their registers fall free
            });
            cur = nxt;
        };
        if constexpr (!STREAM) {
            for (int prod = p_begin; prod < p_end; ++prod) {   // every product fills the pipeline anew
                cur = 0;
                ld_t = 0;
                voff = voff_first;
                set_sources(prod);
                static_for<0, NST>([&](auto sc) __attribute__((always_inline)) { issue(decltype(sc)::value * B::STAGE); });
                wait_loads<AHEAD * NLOAD>();    // step 0 has landed
                workgroup_barrier();
                read_all();
                for (int t = 0; t < steps; ++t) {
                    step(issue_one, std::true_type{});
                    after_step(t + 1);
                }
                after_product(prod);
                // direct loads of the repeated last step may still be in flight: they must land before the
                // LDS is used for anything else or handed to another workgroup
                wait_loads<0>();
                workgroup_barrier();
            }
        } else {
            // The products form one continuous stream of steps (steps >= NST is the caller's business):
            // the requests run NST steps ahead of the matrix cores straight across a product boundary,
            // so only the first product pays for filling the pipeline. While the matrix cores work on
            // the last NST steps of a product the requests are already in the next one; the step loop
            // is split there, so that the change of source addresses (amounts worked out before the
            // walk and kept in LDS) is outside both halves: a scalar load or a second path inside the
            // loop would turn every wait for LDS reads in it into a wait for all of them.
            unsigned inc = kFragBytes;
            auto issue_ahead = [&](int jj, unsigned stage_off) __attribute__((always_inline)) {
                dma_load16(src[jj], voff, dst[jj] + stage_off);
                if (jj == NLOAD - 1) voff += inc;
            };
            for (int p = p_begin; p + 1 < p_end; ++p) {
#pragma unroll
                for (int k = 0; k < NLOAD; ++k)
                    if (w.lane == 0) w.switch_table[(p - p_begin) * NLOAD + k] = fragment_ptr(p + 1, k) - fragment_ptr(p, k);
            }
            set_sources(p_begin);
            static_for<0, NST>([&](auto sc) __attribute__((always_inline)) {
#pragma unroll
                for (int jj = 0; jj < NLOAD; ++jj) issue_ahead(jj, decltype(sc)::value * B::STAGE);
            });
            wait_loads<AHEAD * NLOAD>();    // step 0 has landed
            workgroup_barrier();
            read_all();
            for (int prod = p_begin; prod < p_end; ++prod) {
                // Nothing that shares the counter of the LDS reads may be in flight when the step loops
                // are entered (a scalar load of a kernel argument that the epilogue wants, say): scalar
                // loads complete out of order, and with one possibly in flight on entry every wait for a
                // fragment inside the loops becomes a wait for all of them.
                __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
                int t = 0;
                for (; t < steps - NST; ++t) {
                    step(issue_ahead, std::true_type{});
                    after_step(t + 1);
                }
                if (prod + 1 < p_end) {
#pragma unroll
                    for (int k = 0; k < NLOAD; ++k) src[k] = uniform_ptr(src[k] + w.switch_table[(prod - p_begin) * NLOAD + k]);
                    // (formed here from the lane number, not kept in a register across the walk)
                    voff = (unsigned)lane_here() * 16u + (unsigned)g.t_begin * kFragBytes;
                } else {   // nothing follows: the last step again and again
                    voff -= kFragBytes;
                    inc = 0;
                }
                for (t = steps - NST; t < steps; ++t) {
                    step(issue_ahead, std::true_type{});
                    after_step(t + 1);
                }
                after_product(prod);
                // The fragments of the next product's first step were not kept in registers across the
                // epilogue (it needs them); they are read again from their stage, which the last barrier
                // has already published.
                if (prod + 1 < p_end) read_all();
            }
            wait_loads<0>();
            workgroup_barrier();
        }
    } else {
        // Two stages: the fragments of a step are read at its start, in the order of their first
        // use and two groups ahead of it (B fragments pass through three rotating registers).
        // Every product fills the pipeline anew.
        v4i a[SB], b[3];
        for (int prod = p_begin; prod < p_end; ++prod) {
            unsigned cur = 0, nxt = B::STAGE;
            ld_t = 0;
            voff = voff_first;
            set_sources(prod);
            issue(cur);
            for (int t = 0; t < steps; ++t) {
                // step t has landed everywhere and nobody reads the other stage any more
                wait_loads<0>();
                workgroup_barrier();
                issue(nxt);
                b[0] = read_b(0, cur);
                static_for<0, SB - E0>([&](auto ic) __attribute__((always_inline)) {
                    a[SB - 1 - decltype(ic)::value] = read_a(SB - 1 - decltype(ic)::value, cur);
                });
                if constexpr (SB > 1) b[1] = read_b(1, cur);
                if constexpr (E0 >= 1) a[E0 - 1] = read_a(E0 - 1, cur);
                __builtin_amdgcn_sched_barrier(0);
                static_for<0, SB>([&](auto qc) __attribute__((always_inline)) {
                    constexpr int q = decltype(qc)::value;
                    constexpr int pmax = SB - 1 - q, pmin = E0 - q > 0 ? E0 - q : 0;
                    if constexpr (q + 2 < SB) b[(q + 2) % 3] = read_b(q + 2, cur);
                    if constexpr (E0 - (q + 2) >= 0) a[E0 - (q + 2)] = read_a(E0 - (q + 2), cur);
                    static_for<0, pmax - pmin + 1>([&](auto ic) __attribute__((always_inline)) {
                        constexpr int p = pmax - decltype(ic)::value;
                        acc[p + q - E0] = mfma(a[p], b[q % 3], acc[p + q - E0]);
                    });
                    __builtin_amdgcn_sched_barrier(0);
                });
                const unsigned o = cur;
                cur = nxt; nxt = o;
                after_step(t + 1);
            }
            wait_loads<0>();
            workgroup_barrier();
            after_product(prod);
        }
    }
}

// Double-double running sum (Section 2.3.4: summing-up in higher precision): TwoSum of the high
// part and the exact term, error into the low part, FastTwoSum to renormalise.
__device__ __forceinline__ void dd_add(double& h, double& l, double t) {
    const double sh = h + t;
    const double bb = sh - h;
    const double e = (h - (sh - bb)) + (t - bb);
    const double l2 = l + e;
    const double hn = sh + l2;
    l = l2 - (hn - sh);
    h = hn;
}
template <int SB>
__device__ __forceinline__ void fold_band_dd(double (&h)[16], double (&l)[16], const v16i (&acc)[kBand]) {
    constexpr int ND = SB < kBand ? SB : kBand, E0 = SB - ND;
    mfma_results_ready();
#pragma unroll
    for (int e = SB - 1; e >= E0; --e) {
        const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * (e + 2)) << 52);
#pragma unroll
        for (int u = 0; u < 16; ++u) dd_add(h[u], l[u], (double)acc_read(acc[e - E0][u]) * sc);
    }
}

// Whether a combine mode reads the old contents of C.
__device__ __forceinline__ bool c_mode_reads(const GemmArgs& g, int c_mode) {
    return c_mode == 1 || c_mode == 2 || c_mode == 4 || (c_mode == 3 && g.beta != 0.0);
}

// One element of the result: C (op)= val with combine mode c_mode. `old_c` is the element of C (and
// `old_zr` that of Zr) fetched ahead of time for the modes that read them.
__device__ __forceinline__ void write_c_element(const GemmArgs& g, int c_mode, double* C, int row, int col, double val,
                                                double old_c, double old_zr) {
    if (row < g.m && col < g.n) {
        double* c = C + (int64_t)row * g.ldc + col;
        if (c_mode == 0) *c = val;
        else if (c_mode == 1) *c = old_c + val;
        else if (c_mode == 2) *c = old_c - val;
        else if (c_mode == 3) {   // BLAS update: RN(alpha G), then RN(RN(alpha G) + RN(beta C)); C is not read if beta == 0
            double v = g.alpha * val;
            if (g.beta != 0.0) v = v + g.beta * old_c;
            *c = v;
        } else {   // last of the four real products of a complex one: (re, im) = (Zr, C + val) -> interleaved Cz
            double2 z;
            z.x = old_zr;
            z.y = old_c + val;
            *reinterpret_cast<double2*>(g.Cz + 2 * ((int64_t)row * g.ldcz + col)) = z;
        }
    }
}

// kModeComplex: the four real products of a complex one, walked one after the other by every workgroup
// (planes SA/SA2, SB/SB2; real part formed in the plane Zr, imaginary part in C, result interleaved in Cz).
constexpr int kModeReal = 0, kModeDD = 1, kModeComplex = 2;

template <int S, int WM, int WN, int MODE>
__global__ __launch_bounds__(64 * WM * WN)
__attribute__((amdgpu_waves_per_eu((WM * WN == 4 && S <= 9) ? 2 : WM * WN / 4, (WM * WN == 4 && S <= 9) ? 2 : WM * WN / 4)))
void product_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int T = 64 * WM * WN;
    constexpr int S2 = S > kBand ? S - kBand : 1;   // slice count of the second band (unused if S <= 8)
    constexpr bool CPLX = MODE == kModeComplex;
    constexpr bool PLAIN = MODE != kModeDD;               // FP64 summing-up (real or complex)
    constexpr int NPROD = CPLX ? 4 : 1;                   // products walked one after the other by a workgroup
    constexpr int NEX = CPLX ? 2 : 1;                     // exponent sets staged (one per plane)
    constexpr int TR = 32 * WM, TC = 32 * WN;             // tile of C

    Walk w;
    w.tid = threadIdx.x;
    w.lane = w.tid & 63;
    w.wave = __builtin_amdgcn_readfirstlane(w.tid >> 6);   // wave-uniform, kept in a scalar register
    w.wm = w.wave / WN;
    w.wn = w.wave % WN;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, w.tm, w.tn);
    w.lds = lds;
    w.lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char*)lds;
    // MFMA operand: lane holds row (lane % 32), bytes 16 (lane / 32) .. + 16 of the 32-byte fragment row
    const int rr = w.lane & 31, half = w.lane >> 5;
    w.rd_lane = (unsigned)(rr * 32 + ((half ^ ((rr >> 3) & 1)) << 4));

    const int tile_id = w.tm * g.tiles_n + w.tn;
    const int64_t num_tiles = (int64_t)g.tiles_m * g.tiles_n;
    const bool wide = !CPLX && g.block_steps > 0;   // complex calls with k-blocking take four real launches

    // The exponents of the tile's rows and columns wait in LDS behind the pipeline stages (rows at
    // ex, columns at ex + TR): the epilogue must not stall on a round trip to memory. The first
    // barrier of the walk publishes them.
    int* ex = reinterpret_cast<int*>(lds + Shape<S, WM, WN>::LDS);   // complex: the imaginary planes' set follows at TR + TC
    // behind them (complex only): per wavefront, the changes of its source addresses from product to product
    constexpr int kSwitchEntries = 3 * 8;
    w.switch_table = (lds_i64*)(__attribute__((address_space(3))) unsigned char*)(lds + Shape<S, WM, WN>::LDS + NEX * (TR + TC) * 4) + w.wave * kSwitchEntries;
    static_assert(!CPLX || Band<(S < kBand ? S : kBand), WM, WN>::NLOAD <= 8, "switch table row");
    if (!g.P) {
        for (int i = w.tid; i < NEX * (TR + TC); i += T) {
            const int plane = i / (TR + TC), ii = i % (TR + TC);
            const bool is_a = ii < TR;
            const int pos = is_a ? w.tm * TR + ii : w.tn * TC + (ii - TR);
            const int32_t* E = is_a ? (plane ? g.EA2 : g.EA) : (plane ? g.EB2 : g.EB);
            ex[i] = pos < (is_a ? g.m : g.n) ? E[pos] : 0;
        }
    }

    v16i acc[kBand];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kBand; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = acc_zero();
    };
    // k-blocking: INT32 sums of the band with lowest diagonal e0 -> INT64 sums in the workspace.
    // Thread t of the workgroup owns element t of every 16 x (diagonal, tile) run: coalesced, and
    // nobody else ever touches it.
    auto flush = [&](int e0, int nd, bool first) __attribute__((always_inline)) {
        // one running pointer (made opaque so that it is formed here, not ahead of the k-walk)
        long long* q = g.D + (((int64_t)e0 * num_tiles + tile_id) * 16) * T + (w.wave * 64 + lane_here());
        const int64_t diag_stride = num_tiles * 16 * T - 16 * T;
        mfma_results_ready();
#pragma unroll
        for (int i = 0; i < kBand; ++i) {
            if (i < nd) {
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const long long v = (long long)acc_read(acc[i][u]);
                    // later blocks add with an atomic that returns nothing: no round trip per element
                    if (first) *q = v;
                    else __hip_atomic_fetch_add(q, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    q += T;
                    __builtin_amdgcn_sched_barrier(0);   // keep register pressure flat
                }
                q += diag_stride;
            }
        }
        // no store of this block may still be in flight when the walk goes back to counting its
        // direct loads (stores and loads share the counter)
        wait_loads<0>();
    };

    // accumulator layout of the 32x32 MFMA: lane holds column (lane % 32); register u holds
    // row 8 (u / 4) + 4 (lane / 32) + u % 4.
    // The coordinates are formed where the epilogue needs them, from the lane number read there: kept
    // across the walk they would be spilled, and a reload of a spilled register waits for every memory
    // operation in flight, the direct loads of the next steps included.
    struct Where { int lrow0, lcol, row0, col; };
    auto where = [&]() __attribute__((always_inline)) -> Where {
        const int lane = lane_here();
        Where p;
        p.lrow0 = w.wm * 32 + 4 * (lane >> 5);
        p.lcol = w.wn * 32 + (lane & 31);
        p.row0 = w.tm * TR + p.lrow0;
        p.col = w.tn * TC + p.lcol;
        return p;
    };

    double sum[16], lo[MODE == kModeDD ? 16 : 1];
    auto clear_sum = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 16; ++u) sum[u] = 0.0;
        if constexpr (MODE == kModeDD) {
#pragma unroll
            for (int u = 0; u < 16; ++u) lo[u] = 0.0;
        }
    };

    auto sources = [&](int prod, const int8_t*& sa, const int8_t*& sb) __attribute__((always_inline)) {
        sa = CPLX && (prod & 1) ? g.SA2 : g.SA;
        sb = CPLX && (prod == 1 || prod == 2) ? g.SB2 : g.SB;
    };
    // The elements of C that the combine mode reads are requested before the diagonals are folded, so
    // that they arrive while the fold runs (sixteen dependent round trips to memory otherwise); those of
    // Zr (complex interleave only) in one batch after it, when the fold's registers are free again.
    double old_c[PLAIN ? 16 : 1], old_zr[MODE == kModeReal ? 16 : 1];
    // whether the whole tile lies inside C (then the epilogue tests nothing per element); formed where it is used
    auto tile_inside = [&]() __attribute__((always_inline)) -> bool {
        const int z = opaque_scalar_zero();
        return (w.tm + 1 + z) * TR <= g.m && (w.tn + 1 + z) * TC <= g.n;
    };
    auto fetch_old = [&](double (&dst)[PLAIN ? 16 : 1], const double* src, bool wanted) __attribute__((always_inline)) {
        if constexpr (PLAIN) {
            if (!wanted) {
#pragma unroll
                for (int u = 0; u < 16; ++u) dst[u] = 0.0;
                return;
            }
            const Where at = where();
            const int row0 = at.row0, col = at.col;
            const double* c = src + (int64_t)row0 * g.ldc + col;
            if (CPLX && tile_inside()) {   // no test per element
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    dst[u] = __hip_atomic_load(c + (int64_t)(8 * (u >> 2) + (u & 3)) * g.ldc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int dr = 8 * (u >> 2) + (u & 3);
                const bool in = row0 + dr < g.m && col < g.n;
                // complex: the planes were written by this lane's own earlier stores (acknowledged by the
                // L2 since: the walk in between drains the counter they share with the direct loads) and
                // are read at the L2, not from a line the vector cache may still hold
                if constexpr (CPLX) dst[u] = in ? __hip_atomic_load(c + (int64_t)dr * g.ldc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0;
                else dst[u] = in ? c[(int64_t)dr * g.ldc] : 0.0;
            }
        }
    };
    // Product prod of a complex call: 0: Ar Br -> Zr, 1: Zr -= Ai Bi, 2: Ar Bi -> C, 3: (Zr, C + Ai Br) -> Cz.
    auto mode_of = [&](int prod) __attribute__((always_inline)) -> int {
        if constexpr (CPLX) return prod == 0 ? 0 : prod == 1 ? 2 : prod == 2 ? 0 : 4;
        else return g.c_mode;
    };
    auto plane_of = [&](int prod) __attribute__((always_inline)) -> double* {
        if constexpr (CPLX) return prod < 2 ? g.Zr : g.C;
        else return g.C;
    };
    // The sum of product `prod` is complete (in `sum`, or in the INT64 sums of the workspace): scale it,
    // combine it, store what is final.
    auto finish_product = [&](int prod) __attribute__((always_inline)) {
        // Everything this step addresses is formed here, from values made opaque, and not ahead of the
        // walk, where it would occupy registers the matrix-core loop needs.
        const Where at = where();
        const int oz = (int)opaque_zero();
        const int row0 = at.row0, col = at.col, lrow0 = at.lrow0, lcol = at.lcol;
        if (g.P) {   // pair mode (S == 1): the raw INT32 sums
            mfma_results_ready();
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int row = row0 + 8 * (u >> 2) + (u & 3);
                if (row < g.m && col < g.n) g.P[(int64_t)row * g.ldp + col] = acc_read(acc[0][u]);
            }
            return;
        }
        if (wide) {   // the FP64 sum from the INT64 sums, same order
            const long long* q = g.D + ((int64_t)tile_id * 16) * T + (w.wave * 64 + lane_here()) + oz;
            for (int e = S - 1; e >= 0; --e) {
                const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * (e + 2)) << 52);
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    // read at the L2, where the atomic adds of the blocks were applied
                    const long long s_e = __hip_atomic_load(q + ((int64_t)e * num_tiles * 16 + u) * T, __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
                    const double term = (double)s_e * sc;   // exact: |S_e| < 2^53
                    if constexpr (MODE == kModeDD) dd_add(sum[u], lo[u], term);
                    else sum[u] = sum[u] + term;
                }
            }
        }
        const int c_mode = mode_of(prod);
        double* const plane = plane_of(prod);
        const int* exa = ex + (CPLX && (prod & 1) ? TR + TC : 0);
        const int* exb = ex + (CPLX && (prod == 1 || prod == 2) ? TR + TC : 0) + TR;
        const int eb = exb[lcol];
        if constexpr (CPLX) {
            // Two passes, so that the finished real parts can take the registers of the old values:
            // first this product's scaled sum combined with the part formed so far, in place ...
#pragma unroll
            for (int u4 = 0; u4 < 4; ++u4) {
                const v4i ea = *reinterpret_cast<const v4i*>(exa + lrow0 + 8 * u4);   // four consecutive rows
#pragma unroll
                for (int uu = 0; uu < 4; ++uu) {
                    const int u = 4 * u4 + uu;
                    const double val = ldexp(sum[u], ea[uu] + eb);
                    sum[u] = c_mode == 0 ? val : c_mode == 2 ? old_c[u] - val : old_c[u] + val;
                }
            }
            // ... then, for the last product, the real parts, and the stores. Everything older is
            // awaited before the first store (the old values are needed now anyway; the direct loads of
            // the next product's first steps were requested before the fold and have landed), and the
            // loaded values are named as used on every path: the compiler then has no load of its own
            // left to wait for later, in the walk, where its wait would take the stores and the direct
            // loads with it.
            fetch_old(old_c, g.Zr, c_mode == 4);
            wait_loads<0>();
#pragma unroll
            for (int u = 0; u < 16; ++u) asm volatile("" : : "v"(old_c[u]));
            if (tile_inside()) {   // no test per element
                if (c_mode == 4) {
                    double* z = g.Cz + 2 * ((int64_t)row0 * g.ldcz + col);
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        double2 v;
                        v.x = old_c[u];
                        v.y = sum[u];
                        *reinterpret_cast<double2*>(z + 2 * (int64_t)(8 * (u >> 2) + (u & 3)) * g.ldcz) = v;
                    }
                } else {
                    double* c = plane + (int64_t)row0 * g.ldc + col;
#pragma unroll
                    for (int u = 0; u < 16; ++u) c[(int64_t)(8 * (u >> 2) + (u & 3)) * g.ldc] = sum[u];
                }
                return;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int row = row0 + 8 * (u >> 2) + (u & 3);
                if (row < g.m && col < g.n) {
                    if (c_mode == 4) {
                        double2 z;
                        z.x = old_c[u];
                        z.y = sum[u];
                        *reinterpret_cast<double2*>(g.Cz + 2 * ((int64_t)row * g.ldcz + col)) = z;
                    } else {
                        plane[(int64_t)row * g.ldc + col] = sum[u];
                    }
                }
            }
        } else {
            fetch_old(old_zr, g.Zr, c_mode == 4);
#pragma unroll
            for (int u4 = 0; u4 < 4; ++u4) {
                const v4i ea = *reinterpret_cast<const v4i*>(exa + lrow0 + 8 * u4);   // four consecutive rows
#pragma unroll
                for (int uu = 0; uu < 4; ++uu) {
                    const int u = 4 * u4 + uu;
                    const int row = row0 + 8 * u4 + uu;
                    const int e = ea[uu] + eb;
                    const double val = ldexp(sum[u], e);
                    if constexpr (MODE == kModeDD) {
                        if (row < g.m && col < g.n) {
                            g.C[(int64_t)row * g.ldc + col] = val;
                            g.C_lo[(int64_t)row * g.ldc + col] = ldexp(lo[u], e);
                        }
                    } else {
                        write_c_element(g, c_mode, plane, row, col, val, old_c[PLAIN ? u : 0], old_zr[PLAIN ? u : 0]);
                    }
                }
            }
        }
    };

    bool first_block = true;
    int until_flush = g.block_steps;
    auto run_band = [&](auto sb_tag, int p_begin, int p_end, bool first_band, bool last_band) __attribute__((always_inline)) {
        constexpr int SB = decltype(sb_tag)::value;
        using B = Band<SB, WM, WN>;
        zero_acc();
        band_walk<SB, WM, WN, (NPROD > 1 && S <= kBand)>(acc, g, w, p_begin, p_end, sources,
            [&](int done) __attribute__((always_inline)) {
                if (wide && (--until_flush == 0 || done == g.t_end - g.t_begin)) {
                    flush(B::E0, B::ND, first_block);
                    first_block = false;
                    until_flush = g.block_steps;
                    zero_acc();
                }
            },
            [&](int prod) __attribute__((always_inline)) {
                // nothing of the epilogue is to be scheduled up into the last step, where the fragment
                // registers are still in use and there is no room for its values
                __builtin_amdgcn_sched_barrier(0);
                if (first_band) clear_sum();
                // The old values are requested before the fold where accumulation registers are to spare
                // for them; with all eight diagonals resident there are none, and an accumulator would be
                // spilled to make room (its reload then waits for every memory operation in flight).
                constexpr bool EARLY = !CPLX || B::ND < kBand;
                if (last_band && EARLY) fetch_old(old_c, plane_of(prod), !g.P && c_mode_reads(g, mode_of(prod)));
                if (!wide && !g.P) {
                    if constexpr (MODE == kModeDD) fold_band_dd<SB>(sum, lo, acc);
                    else fold_band<SB>(sum, acc);
                }
                if (last_band && !EARLY) fetch_old(old_c, plane_of(prod), !g.P && c_mode_reads(g, mode_of(prod)));
                if (last_band) finish_product(prod);
                zero_acc();
                first_block = true;
                until_flush = g.block_steps;
            });
    };
    if constexpr (S <= kBand) {
        run_band(std::integral_constant<int, S>{}, 0, NPROD, true, true);
    } else {
        for (int prod = 0; prod < NPROD; ++prod) {
            run_band(std::integral_constant<int, S>{}, prod, prod + 1, true, false);
            run_band(std::integral_constant<int, S2>{}, prod, prod + 1, false, true);
        }
    }
}

template <int S, int WM, int WN, int MODE>
hipError_t launch_one(const GemmArgs& g, hipStream_t st) {
    constexpr int lds = Shape<S, WM, WN>::LDS + (MODE == kModeComplex ? 2 : 1) * 32 * (WM + WN) * (int)sizeof(int) + (MODE == kModeComplex ? WM * WN * 192 : 0);
    static_assert(lds <= kLdsLimit, "stages and exponents must fit the LDS");
    hipError_t e = allow_dynamic_lds<&product_kernel<S, WM, WN, MODE>>(lds);
    if (e != hipSuccess) return e;
    product_kernel<S, WM, WN, MODE><<<dim3((unsigned)(g.tiles_m * g.tiles_n)), dim3(64 * WM * WN), lds, st>>>(g);
    return hipGetLastError();
}

template <int MODE>
hipError_t launch_for(const GemmArgs& g, int s, hipStream_t st) {
    if (g.tile_cols == 64 && s <= 9) {   // 64 x 64 tiles, two workgroups per compute unit: not for the double-double sum
        if constexpr (MODE == kModeReal || MODE == kModeComplex) {
            switch (s) {
#define OZ_CASE(S_) case S_: return launch_one<S_, 2, 2, MODE>(g, st);
                OZ_CASE(1) OZ_CASE(2) OZ_CASE(3) OZ_CASE(4) OZ_CASE(5) OZ_CASE(6) OZ_CASE(7) OZ_CASE(8) OZ_CASE(9)
#undef OZ_CASE
            }
        }
        return hipErrorInvalidValue;
    }
    switch (s) {
#define OZ_CASE(S_, WN_) case S_: return launch_one<S_, 2, WN_, MODE>(g, st);
        OZ_CASE(1, 4) OZ_CASE(2, 4) OZ_CASE(3, 4) OZ_CASE(4, 4) OZ_CASE(5, 4) OZ_CASE(6, 4) OZ_CASE(7, 4) OZ_CASE(8, 4)
        OZ_CASE(9, 4) OZ_CASE(10, 4) OZ_CASE(11, 4) OZ_CASE(12, 4) OZ_CASE(13, 4) OZ_CASE(14, 2) OZ_CASE(15, 2) OZ_CASE(16, 2)
#undef OZ_CASE
    }
    return hipErrorInvalidValue;
}

}  // namespace

// One translation unit per mode instantiates this for its sixteen slice counts.
template <int MODE>
hipError_t launch_product_mode(const GemmArgs& g, int s, hipStream_t st) {
    return launch_for<MODE>(g, s, st);
}

}  // namespace ozimmu
