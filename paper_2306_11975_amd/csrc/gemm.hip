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
// Data path of a step: global -> LDS with wave-wide direct loads (global_load_lds_dwordx4, no
// staging registers; a fragment is 1 KiB contiguous in memory and in LDS), two or three LDS stages
// (as many as fit 160 KiB);
// LDS -> registers with ds_read_b128 (fragment rows are 32 bytes with the two 16-byte halves
// swapped in rows 8..15 and 24..31, so that any 16 consecutive lanes cover all 64 banks);
// registers -> v_mfma_i32_32x32x32_i8.
#include <type_traits>

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
    static constexpr int FIT = kLdsLimit / STAGE;
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

// What a wavefront needs to know about its place in the walk.
struct Walk {
    unsigned char* lds;      // dynamic LDS segment
    unsigned lds_base;       // its LDS address
    unsigned rd_lane;        // byte offset of this lane's 16 bytes inside a fragment
    int lane, wave, wm, wn;
    int tm, tn;
    int tid;
};

// Compile-time loop: f(integral_constant<int, I>) for I = BEGIN .. END - 1.
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}

__device__ __forceinline__ v16i mfma(const v4i& a, const v4i& b, const v16i& c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

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

// The walk of one band over the slabs [g.t_begin, g.t_end). acc[e - E0] receives the pairs of
// diagonal e. after_step(steps_done) is called after every step (k-blocking hooks in there).
template <int SB, int WM, int WN, class AfterStep>
__device__ __forceinline__ void band_walk(v16i (&acc)[kBand], const GemmArgs& g, const Walk& w, AfterStep&& after_step) {
    using B = Band<SB, WM, WN>;
    constexpr int E0 = B::E0, NST = B::NST, NLOAD = B::NLOAD;

    // This wavefront's share of the step's fragments: fragment idx = wave + NW jj. Fragments are
    // numbered A(p, i) = p WM + i, then B(q, j) = SB WM + q WN + j, and sit in that order in a
    // stage. A wavefront without a jj-th fragment loads the last one again (same bytes to the same
    // place), so that every wavefront has the same number of loads in flight.
    const int8_t* src[NLOAD];
    unsigned dst[NLOAD];
#pragma unroll
    for (int jj = 0; jj < NLOAD; ++jj) {
        int idx = w.wave + B::NW * jj;
        idx = idx < B::NFRAG ? idx : B::NFRAG - 1;
        if (idx < SB * WM) {
            const int p = idx / WM, i = idx % WM;
            src[jj] = g.SA + (int64_t)p * g.a_slice_stride + (int64_t)(w.tm * WM + i) * g.kslabs * kFragBytes;
        } else {
            const int r = idx - SB * WM;
            const int q = r / WN, j = r % WN;
            src[jj] = g.SB + (int64_t)q * g.b_slice_stride + (int64_t)(w.tn * WN + j) * g.kslabs * kFragBytes;
        }
        dst[jj] = w.lds_base + (unsigned)idx * kFragBytes;
        // wave-uniform by construction; say so, so that they live in scalar registers
        src[jj] = uniform_ptr(src[jj]);
        dst[jj] = (unsigned)__builtin_amdgcn_readfirstlane((int)dst[jj]);
    }
    // lane offset into the source fragment of the next step to request; past the end of the walk
    // the last step is requested again (into a stage nobody reads any more)
    unsigned voff = (unsigned)w.lane * 16u + (unsigned)g.t_begin * kFragBytes;
    const unsigned voff_last = (unsigned)w.lane * 16u + (unsigned)(g.t_end - 1) * kFragBytes;
    // Load jj of the step being requested; the last one moves on to the next step.
    auto issue_one = [&](int jj, unsigned stage_off) __attribute__((always_inline)) {
        dma_load16(src[jj], voff, dst[jj] + stage_off);
        if (jj == NLOAD - 1) {
            const unsigned nv = voff + kFragBytes;
            voff = nv < voff_last ? nv : voff_last;
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

    const int steps = g.t_end - g.t_begin;
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
        static_for<0, NST>([&](auto sc) __attribute__((always_inline)) { issue(decltype(sc)::value * B::STAGE); });
        wait_loads<AHEAD * NLOAD>();    // step 0 has landed
        workgroup_barrier();
        static_for<0, SB>([&](auto pc) __attribute__((always_inline)) {
            constexpr int p = decltype(pc)::value;
            a[SB - 1 - p] = read_a(SB - 1 - p, cur);
            b[p] = read_b(p, cur);
        });
        for (int t = 0; t < steps; ++t) {
            const unsigned nxt = cur + B::STAGE < (unsigned)B::LDS ? cur + B::STAGE : 0u;
            static_for<0, SB>([&](auto qc) __attribute__((always_inline)) {
                constexpr int q = decltype(qc)::value;
                constexpr int pmax = SB - 1 - q, pmin = E0 - q > 0 ? E0 - q : 0;
                static_for<0, pmax - pmin + 1>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int p = pmax - decltype(ic)::value;
                    acc[p + q - E0] = mfma(a[p], b[q], acc[p + q - E0]);
                });
                if constexpr (q == 0) {
                    // step t + 1 has landed everywhere (its fragments may be read from here on) and
                    // every wavefront has read the last fragment of step t: its stage is free
                    __builtin_amdgcn_sched_barrier(0);
                    wait_loads<(AHEAD - 1) * NLOAD>();
                    workgroup_barrier();
                }
                // one direct load per group (NLOAD <= SB): a wavefront stalls while its load is issued,
                // and eight wavefronts that issue all their loads at once queue behind each other
                if constexpr (q < NLOAD) issue_one(q, cur);
                b[q] = read_b(q, nxt);
                a[pmax] = read_a(pmax, nxt);
                __builtin_amdgcn_sched_barrier(0);   // keep the re-reads where their registers fall free
            });
            cur = nxt;
            after_step(t + 1);
        }
    } else {
        // Two stages: the fragments of a step are read at its start, in the order of their first
        // use and two groups ahead of it (B fragments pass through three rotating registers).
        v4i a[SB], b[3];
        unsigned cur = 0, nxt = B::STAGE;
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
    }
    // direct loads of the clamped tail may still be in flight: they must land before the LDS is
    // used for anything else or handed to another workgroup
    wait_loads<0>();
    workgroup_barrier();
}

// acc = RN(acc + S_e 2^(-7 (e + 2))) for the diagonals of a band, least significant first. The
// product of an integer below 2^31 and a power of two is exact, so the fused operation rounds
// exactly like the sum it stands for.
template <int SB>
__device__ __forceinline__ void fold_band(double (&sum)[16], const v16i (&acc)[kBand]) {
    constexpr int ND = SB < kBand ? SB : kBand, E0 = SB - ND;
#pragma unroll
    for (int e = SB - 1; e >= E0; --e) {
        const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * (e + 2)) << 52);
#pragma unroll
        for (int u = 0; u < 16; ++u) sum[u] = fma((double)acc_read(acc[e - E0][u]), sc, sum[u]);
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
#pragma unroll
    for (int e = SB - 1; e >= E0; --e) {
        const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * (e + 2)) << 52);
#pragma unroll
        for (int u = 0; u < 16; ++u) dd_add(h[u], l[u], (double)acc_read(acc[e - E0][u]) * sc);
    }
}

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

template <int S, int WM, int WN, bool DD>
__global__ __launch_bounds__(64 * WM * WN) __attribute__((amdgpu_waves_per_eu(WM * WN / 4, WM * WN / 4)))
void product_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int T = 64 * WM * WN;
    constexpr int S2 = S > kBand ? S - kBand : 1;   // slice count of the second band (unused if S <= 8)

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
    const bool wide = g.block_steps > 0;

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
        long long* q = g.D + (((int64_t)e0 * num_tiles + tile_id) * 16) * T + w.tid + opaque_zero();
        const int64_t diag_stride = num_tiles * 16 * T - 16 * T;
#pragma unroll
        for (int i = 0; i < kBand; ++i) {
            if (i < nd) {
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    long long v = (long long)acc_read(acc[i][u]);
                    if (!first) v += *q;
                    *q = v;
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
    const int row0 = (w.tm * WM + w.wm) * 32 + 4 * half;
    const int col = (w.tn * WN + w.wn) * 32 + rr;

    double sum[16], lo[DD ? 16 : 1];
#pragma unroll
    for (int u = 0; u < 16; ++u) sum[u] = 0.0;
    if (DD) {
#pragma unroll
        for (int u = 0; u < 16; ++u) lo[DD ? u : 0] = 0.0;
    }

    auto run_band = [&](auto sb_tag) __attribute__((always_inline)) {
        constexpr int SB = decltype(sb_tag)::value;
        using B = Band<SB, WM, WN>;
        zero_acc();
        bool first = true;
        int until_flush = g.block_steps;
        band_walk<SB, WM, WN>(acc, g, w, [&](int done) __attribute__((always_inline)) {
            if (wide && (--until_flush == 0 || done == g.t_end - g.t_begin)) {
                flush(B::E0, B::ND, first);
                first = false;
                until_flush = g.block_steps;
                zero_acc();
            }
        });
        if (!wide && !g.P) {
            if constexpr (DD) fold_band_dd<SB>(sum, lo, acc);
            else fold_band<SB>(sum, acc);
        }
    };
    run_band(std::integral_constant<int, S>{});
    if constexpr (S > kBand) run_band(std::integral_constant<int, S2>{});

    if (g.P) {   // pair mode (S == 1): the raw INT32 sums
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int row = row0 + 8 * (u >> 2) + (u & 3);
            if (row < g.m && col < g.n) g.P[(int64_t)row * g.ldp + col] = acc_read(acc[0][u]);
        }
        return;
    }
    if (wide) {   // the FP64 sum from the INT64 sums, same order
        const long long* q = g.D + ((int64_t)tile_id * 16) * T + w.tid;
        for (int e = S - 1; e >= 0; --e) {
            const double sc = __longlong_as_double((long long)(1023 - OZIMMU_SLICE_BITS * (e + 2)) << 52);
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const double term = (double)q[((int64_t)e * num_tiles * 16 + u) * T] * sc;   // exact: |S_e| < 2^53
                if (DD) dd_add(sum[u], lo[DD ? u : 0], term);
                else sum[u] = sum[u] + term;
            }
        }
    }
    const int eb = col < g.n ? g.EB[col] : 0;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int row = row0 + 8 * (u >> 2) + (u & 3);
        if (DD) {
            if (row < g.m && col < g.n) {
                const int e = g.EA[row] + eb;
                g.C[(int64_t)row * g.ldc + col] = ldexp(sum[u], e);
                g.C_lo[(int64_t)row * g.ldc + col] = ldexp(lo[DD ? u : 0], e);
            }
        } else {
            write_c_element(g, row, col, eb, sum[u]);
        }
    }
}

template <int S, int WM, int WN, bool DD>
hipError_t launch_one(const GemmArgs& g, hipStream_t st) {
    constexpr int lds = Shape<S, WM, WN>::LDS;
    hipError_t e = allow_dynamic_lds<&product_kernel<S, WM, WN, DD>>(lds);
    if (e != hipSuccess) return e;
    product_kernel<S, WM, WN, DD><<<dim3((unsigned)(g.tiles_m * g.tiles_n)), dim3(64 * WM * WN), lds, st>>>(g);
    return hipGetLastError();
}

template <bool DD>
hipError_t launch_for(const GemmArgs& g, int s, hipStream_t st) {
    switch (s) {
#define OZ_CASE(S_, WN_) case S_: return launch_one<S_, 2, WN_, DD>(g, st);
        OZ_CASE(1, 4) OZ_CASE(2, 4) OZ_CASE(3, 4) OZ_CASE(4, 4) OZ_CASE(5, 4) OZ_CASE(6, 4) OZ_CASE(7, 4) OZ_CASE(8, 4)
        OZ_CASE(9, 4) OZ_CASE(10, 4) OZ_CASE(11, 4) OZ_CASE(12, 4) OZ_CASE(13, 4) OZ_CASE(14, 2) OZ_CASE(15, 2) OZ_CASE(16, 2)
#undef OZ_CASE
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_slice_gemm(const GemmArgs& args, int s, bool dd, hipStream_t st) {
    if (args.tiles_m * args.tiles_n == 0 || args.t_end <= args.t_begin) return hipSuccess;
    return dd ? launch_for<true>(args, s, st) : launch_for<false>(args, s, st);
}

}  // namespace ozimmu
