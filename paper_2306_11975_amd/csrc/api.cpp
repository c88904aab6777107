// C ABI of libozimmu: argument validation, workspace carving and kernel sequencing.
// Everything that computes is in split.hip and gemm.hip.
#include <cstdint>
#include <cstring>

#include <algorithm>

#include "ozimmu_internal.h"

using namespace ozimmu;

namespace {

constexpr int64_t kMaxDim = OZIMMU_MAX_DIM;  // every launch grid (k / 128 blocks in grid.y at most) stays legal

inline size_t align_up(size_t x) { return (x + OZIMMU_WORKSPACE_ALIGN - 1) / OZIMMU_WORKSPACE_ALIGN * OZIMMU_WORKSPACE_ALIGN; }

bool dims_ok(int64_t a, int64_t b, int64_t c) {
    return a >= 0 && b >= 0 && c >= 0 && a <= kMaxDim && b <= kMaxDim && c <= kMaxDim;
}

// A diagonal d = p + q holds d - 1 pairs; the longest one (d = s + 1) sums s * k_pad products
// per output element. If that exceeds the INT32 block the kernel moves its INT32 sums into INT64
// sums in the workspace every block_steps steps of 32 products per pair (k-blocking).
bool needs_wide(int s, int64_t k_pad) { return (int64_t)s * k_pad > OZIMMU_INT32_BLOCK; }
int block_steps_for(int s) { return OZIMMU_INT32_BLOCK / (s * kSlab); }

struct Layout {
    int64_t m_pad, n_pad, k_pad;
    int tiles_m, tiles_n, tile_rows, tile_cols;
    bool wide;
    size_t sa_bytes, sb_bytes;      // one plane
    size_t off_scan;
    size_t off_sa[2], off_sb[2];    // planes (real GEMM uses plane 0)
    size_t off_ea[2], off_eb[2];
    size_t off_colmax, off_d, off_z, off_gate;
    size_t total;
};

// Tile shape and count (the byte offsets of a layout do not depend on them: D exists only with k-blocking,
// which never takes the small tiles).
void set_tiles(Layout& L, int64_t m, int64_t n, int s, bool small) {
    int wm, wn;
    tile_waves(s, small, &wm, &wn);
    L.tile_rows = wm * kFragRows;
    L.tile_cols = wn * kFragRows;
    L.tiles_m = (int)((m + L.tile_rows - 1) / L.tile_rows);
    L.tiles_n = (int)((n + L.tile_cols - 1) / L.tile_cols);
}

Layout make_layout(int64_t m, int64_t n, int64_t k, int s, bool cplx) {
    Layout L{};
    L.m_pad = round_up(m, kRowAlign);
    L.n_pad = round_up(n, kRowAlign);
    L.k_pad = round_up(k, kSlab);
    L.wide = needs_wide(s, L.k_pad);
    // a complex product walks its four real products in one launch from three steps on (on 64 x 64 tiles only where
    // the large ones would leave compute units without a tile: measured, a short inner dimension alone does not pay
    // there); shorter ones take four launches of the real kernel and its tile choice
    const bool one_launch = cplx && !L.wide && L.k_pad / kSlab >= 3;
    set_tiles(L, m, n, s, one_launch ? use_small_tiles(m, n, INT64_MAX, s, L.wide) : use_small_tiles(m, n, L.k_pad, s, L.wide));
    L.sa_bytes = (size_t)s * L.m_pad * L.k_pad;
    L.sb_bytes = (size_t)s * L.n_pad * L.k_pad;
    const int planes = cplx ? 2 : 1;
    size_t off = 0;
    for (int p = 0; p < planes; ++p) { L.off_sa[p] = off; off = align_up(off + L.sa_bytes); }
    for (int p = 0; p < planes; ++p) { L.off_sb[p] = off; off = align_up(off + L.sb_bytes); }
    for (int p = 0; p < planes; ++p) { L.off_ea[p] = off; off = align_up(off + sizeof(int32_t) * L.m_pad); }
    for (int p = 0; p < planes; ++p) { L.off_eb[p] = off; off = align_up(off + sizeof(int32_t) * L.n_pad); }
    L.off_colmax = off;
    off = align_up(off + sizeof(unsigned long long) * planes * (L.n_pad > L.m_pad ? L.n_pad : L.m_pad));  // either operand may be split by columns (complex: both planes at once)
    L.off_d = off;
    if (L.wide) off = align_up(off + (size_t)s * L.tiles_m * L.tiles_n * L.tile_rows * L.tile_cols * sizeof(long long));
    L.off_z = off;   // complex: the real and imaginary parts of the result as two m x n planes
    if (cplx) off = align_up(off + (size_t)2 * m * n * sizeof(double));
    L.off_gate = off;   // complex with a small B: its slice tensors for the kernel that splits A on the fly
    if (cplx) off = align_up(off + gate_scratch_bytes(n, k, s));
    L.off_scan = off;   // the counters of splitters that count for the slice-count check: first operand, then second
    off = align_up(off + 2 * scan_slots_bytes(planes));
    L.total = off;
    return L;
}

ozimmu_status_t hip_status(hipError_t e) { return e == hipSuccess ? OZIMMU_OK : OZIMMU_ERR_HIP; }

ozimmu_status_t check_gemm_args(int64_t m, int64_t n, int64_t k, const void* A, int64_t lda, const void* B,
                                int64_t ldb, const void* C, int64_t ldc, int s, const void* ws, size_t ws_bytes,
                                bool cplx, Layout* L) {
    if (!dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    if (s < 1 || s > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    if (m == 0 || n == 0) return OZIMMU_OK;
    if (lda < k || ldb < n || ldc < n) return OZIMMU_ERR_BAD_LD;
    if (!C || (k > 0 && (!A || !B))) return OZIMMU_ERR_NULL;
    *L = make_layout(m, n, k, s, cplx);
    if (k > 0) {
        if (!ws || (reinterpret_cast<uintptr_t>(ws) % OZIMMU_WORKSPACE_ALIGN) != 0 || ws_bytes < L->total)
            return OZIMMU_ERR_WORKSPACE;
    }
    return OZIMMU_OK;
}

// Both planes of an interleaved complex operand whose rows run along k (rows x k complex elements, leading
// dimension ld in complex elements) into the slice tensors and exponents at off_s[0..1], off_e[0..1]:
// one pass over the data when the rows are short enough to wait in registers, else one strided pass per
// plane. negate_im: the slices of the conjugated operand.
hipError_t split_complex_rows(const double* Z, int64_t ld, int64_t rows, int64_t k, int s, unsigned char* ws,
                              const size_t (&off_s)[2], const size_t (&off_e)[2], int64_t rows_pad, int64_t k_pad,
                              hipStream_t st, bool negate_im, unsigned long long* scan_slots = nullptr) {
    int8_t* S[2] = {reinterpret_cast<int8_t*>(ws + off_s[0]), reinterpret_cast<int8_t*>(ws + off_s[1])};
    int32_t* E[2] = {reinterpret_cast<int32_t*>(ws + off_e[0]), reinterpret_cast<int32_t*>(ws + off_e[1])};
    if (complex_rows_in_one_pass(Z, k_pad))
        return launch_split_rows_complex(Z, ld, rows, k, s, S[0], S[1], rows_pad, k_pad, E[0], E[1], st, negate_im, scan_slots);
    hipError_t e = launch_split_rows(Z, ld, 2, rows, k, s, S[0], rows_pad, k_pad, E[0], st, false, scan_slots, 10);
    if (e == hipSuccess)
        e = launch_split_rows(Z + 1, ld, 2, rows, k, s, S[1], rows_pad, k_pad, E[1], st, negate_im,
                              scan_slots ? scan_slots + 5 : nullptr, 10);
    return e;
}

// One real Ozaki product from already split planes: G = sum over diagonals, combined into C as
// c_mode says (C_lo != nullptr: double-double sum into C, C_lo).
hipError_t run_product(const Layout& L, int64_t m, int64_t n, int s, unsigned char* ws, int plane_a, int plane_b,
                       double* C, int64_t ldc, int c_mode, hipStream_t st, double alpha = 1.0, double beta = 0.0,
                       double* C_lo = nullptr, double* Zr = nullptr, double* Cz = nullptr, int64_t ldcz = 0) {
    GemmArgs g{};
    g.SA = reinterpret_cast<const int8_t*>(ws + L.off_sa[plane_a]);
    g.SB = reinterpret_cast<const int8_t*>(ws + L.off_sb[plane_b]);
    g.a_slice_stride = L.m_pad * L.k_pad;
    g.b_slice_stride = L.n_pad * L.k_pad;
    g.kslabs = (int)(L.k_pad / kSlab);
    g.t_begin = 0;
    g.t_end = g.kslabs;
    g.tiles_m = L.tiles_m;
    g.tiles_n = L.tiles_n;
    g.tile_cols = L.tile_cols;
    g.m = (int)m;
    g.n = (int)n;
    g.block_steps = L.wide ? block_steps_for(s) : 0;
    g.D = L.wide ? reinterpret_cast<long long*>(ws + L.off_d) : nullptr;
    g.EA = reinterpret_cast<const int32_t*>(ws + L.off_ea[plane_a]);
    g.EB = reinterpret_cast<const int32_t*>(ws + L.off_eb[plane_b]);
    g.C = C;
    g.ldc = ldc;
    g.c_mode = c_mode;
    g.alpha = alpha;
    g.beta = beta;
    g.C_lo = C_lo;
    g.Zr = Zr;
    g.Cz = Cz;
    g.ldcz = ldcz;
    return launch_slice_gemm(g, s, C_lo ? 1 : 0, st);
}

// The four real products of a complex one from the split planes (0 = real, 1 = imaginary):
// Cr = G(Ar,Br) - G(Ai,Bi);  Ci = G(Ar,Bi) + G(Ai,Br). The two parts are formed in two m x n planes of
// the workspace (contiguous FP64: every update there is a full-line access), the second product of
// each part combined with the first by one rounded FP64 operation in the kernel's epilogue; the
// epilogue of the last product writes C, once, as (re, im) pairs.
hipError_t run_complex_products(const Layout& L, int64_t m, int64_t n, int s, unsigned char* ws, double* C,
                                int64_t ldc, hipStream_t st) {
    double* Pr = reinterpret_cast<double*>(ws + L.off_z);
    double* Pi = Pr + (size_t)m * n;
    // one launch: every workgroup walks the four products of its tile one after the other (the walk runs
    // three steps ahead of the matrix cores: shorter products and k-blocked ones take four launches;
    // make_layout has chosen the tiles accordingly)
    if (!L.wide && L.k_pad / kSlab >= 3) {
        GemmArgs g{};
        g.SA = reinterpret_cast<const int8_t*>(ws + L.off_sa[0]);
        g.SA2 = reinterpret_cast<const int8_t*>(ws + L.off_sa[1]);
        g.SB = reinterpret_cast<const int8_t*>(ws + L.off_sb[0]);
        g.SB2 = reinterpret_cast<const int8_t*>(ws + L.off_sb[1]);
        g.EA = reinterpret_cast<const int32_t*>(ws + L.off_ea[0]);
        g.EA2 = reinterpret_cast<const int32_t*>(ws + L.off_ea[1]);
        g.EB = reinterpret_cast<const int32_t*>(ws + L.off_eb[0]);
        g.EB2 = reinterpret_cast<const int32_t*>(ws + L.off_eb[1]);
        g.a_slice_stride = L.m_pad * L.k_pad;
        g.b_slice_stride = L.n_pad * L.k_pad;
        g.kslabs = (int)(L.k_pad / kSlab);
        g.t_begin = 0;
        g.t_end = g.kslabs;
        g.tiles_m = L.tiles_m;
        g.tiles_n = L.tiles_n;
        g.tile_cols = L.tile_cols;
        g.m = (int)m;
        g.n = (int)n;
        g.Zr = Pr;
        g.C = Pi;
        g.ldc = n;
        g.Cz = C;
        g.ldcz = ldc;
        g.alpha = 1.0;
        return launch_slice_gemm(g, s, 2, st);
    }
    hipError_t e = run_product(L, m, n, s, ws, 0, 0, Pr, n, 0, st);
    if (e == hipSuccess) e = run_product(L, m, n, s, ws, 1, 1, Pr, n, 2, st);
    if (e == hipSuccess) e = run_product(L, m, n, s, ws, 0, 1, Pi, n, 0, st);
    if (e == hipSuccess) e = run_product(L, m, n, s, ws, 1, 0, Pi, n, 4, st, 1.0, 0.0, nullptr, Pr, C, ldc);
    return e;
}

// 'N' -> 0, 'T' -> 1, 'C' -> 2, anything else -> -1
int parse_trans(char c) {
    switch (c) {
        case 'N': case 'n': return 0;
        case 'T': case 't': return 1;
        case 'C': case 'c': return 2;
    }
    return -1;
}

// One operand of the automatic slice-count choice: a row-major rows x cols array whose groups
// (the vectors that share an exponent) are its rows, or its columns if by_cols.
struct ScanOperand {
    const double* ptr;
    int64_t ld, rows, cols;
    bool by_cols;
};

// The slice-count sums of operand o (0: first, 1: second) into sums[(o * parts + plane) * 16 ..].
hipError_t scan_operand(const ScanOperand& z, int o, int is_complex, unsigned long long* sums, unsigned long long* colmax,
                        hipStream_t st) {
    const int parts = is_complex ? 2 : 1, inc = is_complex ? 2 : 1;
    unsigned long long* dst = sums + o * parts * OZIMMU_MAX_SLICES;
    if (is_complex && !z.by_cols && complex_scan_in_one_pass(z.ptr, z.cols))   // both planes of short rows at once
        return launch_loss_scan_rows_complex(z.ptr, z.ld, z.rows, z.cols, dst, dst + OZIMMU_MAX_SLICES, st);
    if (is_complex && z.by_cols && complex_cols_scan_in_one_launch(z.ptr, z.rows, z.cols))   // a small gate: one launch
        return launch_loss_scan_cols_complex_small(z.ptr, z.ld, z.rows, z.cols, dst, dst + OZIMMU_MAX_SLICES, st);
    if (is_complex && z.by_cols)   // both planes in one set of launches
        return launch_loss_scan_cols_complex(z.ptr, z.ld, z.rows, z.cols, colmax, dst, dst + OZIMMU_MAX_SLICES, st);
    hipError_t e = hipSuccess;
    for (int pl = 0; pl < parts && e == hipSuccess; ++pl) {
        if (z.by_cols) e = launch_loss_scan_cols(z.ptr + pl, z.ld, inc, z.rows, z.cols, colmax, dst + pl * OZIMMU_MAX_SLICES, st);
        else e = launch_loss_scan_rows(z.ptr + pl, z.ld, inc, z.rows, z.cols, dst + pl * OZIMMU_MAX_SLICES, st);
    }
    return e;
}

// 4 x 16 sums in host memory that kernels of any device can write (one buffer per calling thread, kept until the process ends)
unsigned long long* mapped_sums() {
    thread_local unsigned long long* p = nullptr;
    if (!p) {
        void* q = nullptr;
        if (hipHostMalloc(&q, 4 * OZIMMU_MAX_SLICES * sizeof(unsigned long long), hipHostMallocMapped | hipHostMallocPortable) == hipSuccess)
            p = static_cast<unsigned long long*>(q);
    }
    return p;
}

bool scratch_ok(const void* scratch, size_t scratch_bytes, int64_t scratch_cols) {
    size_t need = 0;
    ozimmu_auto_scratch_bytes(scratch_cols, &need);
    return scratch && (reinterpret_cast<uintptr_t>(scratch) % OZIMMU_WORKSPACE_ALIGN) == 0 && scratch_bytes >= need;
}

// The scans of both operands and the copy of the 4 x 16 sums to `host`, all on the stream; nothing waits.
hipError_t enqueue_scans(const ScanOperand& a, const ScanOperand& b, int is_complex, void* scratch, unsigned long long* host,
                         hipStream_t st) {
    unsigned long long* sums = static_cast<unsigned long long*>(scratch);          // [4][16]
    unsigned long long* colmax = sums + 4 * OZIMMU_MAX_SLICES;
    hipError_t e = launch_fill_u64(sums, 4 * OZIMMU_MAX_SLICES, 0ull, st);
    if (e == hipSuccess) e = scan_operand(a, 0, is_complex, sums, colmax, st);
    if (e == hipSuccess) e = scan_operand(b, 1, is_complex, sums, colmax, st);
    if (e == hipSuccess)
        e = hipMemcpyAsync(host, sums, 4 * OZIMMU_MAX_SLICES * sizeof(unsigned long long), hipMemcpyDeviceToHost, st);
    return e;
}

// The smallest count whose sums of lost bits are within the threshold for every plane; max_slices if none.
int pick_slices(const unsigned long long* host, int is_complex, double count_a, double count_b, double threshold,
                int max_slices) {
    const int parts = is_complex ? 2 : 1;
    for (int s = 1; s <= max_slices; ++s) {
        bool ok = true;
        for (int p = 0; p < 2 * parts; ++p)
            ok = ok && (double)host[p * OZIMMU_MAX_SLICES + (s - 1)] <= threshold * (p < parts ? count_a : count_b);
        if (ok) return s;
    }
    return max_slices;
}

// Whether `guess` is the count pick_slices would return, given only the sums for guess and guess - 1 slices (host: [planes][16],
// the first operand's planes first): the loss does not grow with the slice count, so guess is the choice iff every plane
// is within the threshold with it (or it is the largest count allowed) and some plane is not with one slice less.
bool guess_holds(const unsigned long long* host, int planes, double count_a, double count_b, double threshold, int guess,
                 int max_slices) {
    auto within = [&](int s) {
        bool ok = true;
        for (int p = 0; p < planes; ++p)
            ok = ok && (double)host[p * OZIMMU_MAX_SLICES + (s - 1)] <= threshold * (p < planes / 2 ? count_a : count_b);
        return ok;
    };
    return (within(guess) || guess == max_slices) && (guess == 1 || !within(guess - 1));
}

ozimmu_status_t auto_select(const ScanOperand& a, const ScanOperand& b, int64_t scratch_cols, int is_complex,
                            double threshold, int max_slices, void* scratch, size_t scratch_bytes, int* num_slices,
                            uint64_t* loss_sums, void* stream) {
    if (max_slices < 1 || max_slices > OZIMMU_MAX_SLICES || !(threshold >= 0.0)) return OZIMMU_ERR_BAD_SLICES;
    if (!num_slices) return OZIMMU_ERR_NULL;
    if ((a.rows > 0 && a.cols > 0 && !a.ptr) || (b.rows > 0 && b.cols > 0 && !b.ptr)) return OZIMMU_ERR_NULL;
    if (!scratch_ok(scratch, scratch_bytes, scratch_cols)) return OZIMMU_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned long long pageable[4 * OZIMMU_MAX_SLICES];
    unsigned long long* host = mapped_sums();
    if (!host) host = pageable;
    hipError_t e = enqueue_scans(a, b, is_complex, scratch, host, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return OZIMMU_ERR_HIP;

    *num_slices = pick_slices(host, is_complex, (double)a.rows * (double)a.cols, (double)b.rows * (double)b.cols, threshold,
                              max_slices);
    if (loss_sums)
        for (int i = 0; i < (is_complex ? 4 : 2) * OZIMMU_MAX_SLICES; ++i) loss_sums[i] = host[i];
    return OZIMMU_OK;
}

// The splits of a product that also count for the check of num_slices as the automatic slice count (Section 4.4), and
// the two small kernels that leave the bits lost with num_slices and num_slices - 1 slices in `sums` ([planes][16],
// device or mapped host memory; first operand's planes first). Arguments already validated.
hipError_t counting_splits(bool cplx, const Layout& L, int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                           const double* B, int64_t ldb, int s, unsigned char* ws, unsigned long long* sums, hipStream_t st) {
    const int planes = cplx ? 2 : 1;
    unsigned long long* slots_a = reinterpret_cast<unsigned long long*>(ws + L.off_scan);
    unsigned long long* slots_b = slots_a + scan_slots_bytes(planes) / sizeof(unsigned long long);
    unsigned long long* colmax = reinterpret_cast<unsigned long long*>(ws + L.off_colmax);
    hipError_t e = launch_fill_u64(slots_a, (int64_t)(2 * scan_slots_bytes(planes) / sizeof(unsigned long long)), 0ull, st);
    if (e != hipSuccess) return e;
    if (cplx) {
        e = split_complex_rows(A, lda, m, k, s, ws, L.off_sa, L.off_ea, L.m_pad, L.k_pad, st, false, slots_a);
        if (e == hipSuccess)
            e = launch_split_cols_complex(B, ldb, k, n, s, reinterpret_cast<int8_t*>(ws + L.off_sb[0]),
                                          reinterpret_cast<int8_t*>(ws + L.off_sb[1]), L.n_pad, L.k_pad,
                                          reinterpret_cast<int32_t*>(ws + L.off_eb[0]), reinterpret_cast<int32_t*>(ws + L.off_eb[1]),
                                          colmax, st, false, slots_b);
    } else {
        e = launch_split_rows(A, lda, 1, m, k, s, reinterpret_cast<int8_t*>(ws + L.off_sa[0]), L.m_pad, L.k_pad,
                              reinterpret_cast<int32_t*>(ws + L.off_ea[0]), st, false, slots_a, 5);
        if (e == hipSuccess)
            e = launch_split_cols(B, ldb, 1, k, n, s, reinterpret_cast<int8_t*>(ws + L.off_sb[0]), L.n_pad, L.k_pad,
                                  reinterpret_cast<int32_t*>(ws + L.off_eb[0]), colmax, st, false, slots_b, 5);
    }
    if (e == hipSuccess) e = launch_scan_reduce(slots_a, planes, s, sums, st);
    if (e == hipSuccess) e = launch_scan_reduce(slots_b, planes, s, sums + planes * OZIMMU_MAX_SLICES, st);
    return e;
}

// Slice count and product in one call (see ozimmu_dgemm_auto / ozimmu_zgemm_auto in ozimmu.h).
ozimmu_status_t gemm_auto(bool cplx, int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B,
                          int64_t ldb, double* C, int64_t ldc, double threshold, int max_slices, int guess, void* workspace,
                          size_t workspace_bytes, void* scratch, size_t scratch_bytes, int* num_slices,
                          int* guess_confirmed, void* stream) {
    if (max_slices < 1 || max_slices > OZIMMU_MAX_SLICES || !(threshold >= 0.0)) return OZIMMU_ERR_BAD_SLICES;
    if (!num_slices) return OZIMMU_ERR_NULL;
    if (guess_confirmed) *guess_confirmed = 0;
    // the workspace must serve whichever slice count comes out
    Layout L{};
    for (int s = 1; s <= max_slices; ++s) {
        ozimmu_status_t rc = check_gemm_args(m, n, k, A, lda, B, ldb, C, ldc, s, workspace, workspace_bytes, cplx, &L);
        if (rc != OZIMMU_OK) return rc;
    }
    if (!scratch_ok(scratch, scratch_bytes, n)) return OZIMMU_ERR_WORKSPACE;
    auto product = [&](int s) {
        return cplx ? ozimmu_zgemm(m, n, k, A, lda, B, ldb, C, ldc, s, workspace, workspace_bytes, stream)
                    : ozimmu_dgemm(m, n, k, A, lda, B, ldb, C, ldc, s, workspace, workspace_bytes, stream);
    };
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool have_guess = guess >= 1 && guess <= max_slices && m > 0 && n > 0 && k > 0;
    const double count_a = (double)m * (double)k, count_b = (double)k * (double)n;
    unsigned long long* host = have_guess ? mapped_sums() : nullptr;                   // [4][16]
    if (host && cplx && gate_product_applies(A, B, C, n, k, guess)) {
        // Multiply with the guessed count; the kernels that split B and that walk over A count, on their way, what the
        // check of the guess needs (the bits each plane loses with `guess` and with `guess - 1` slices) and a last small
        // kernel writes the eight sums into mapped host memory: no pass of its own over A, no copy.
        L = make_layout(m, n, k, guess, true);
        if (gate_scan_bytes(m) > L.sa_bytes) return OZIMMU_ERR_WORKSPACE;
        unsigned char* ws = static_cast<unsigned char*>(workspace);
        // the per-tile counters wait where the slices of A would be (that region is not used on this path)
        hipError_t e = launch_gate_product(A, lda, m, k, n, B, ldb, guess, ws + L.off_gate, C, ldc, st,
                                           reinterpret_cast<unsigned*>(ws + L.off_sa[0]), host);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return OZIMMU_ERR_HIP;
        if (guess_holds(host, 4, count_a, count_b, threshold, guess, max_slices)) {
            *num_slices = guess;
            if (guess_confirmed) *guess_confirmed = 1;
            return OZIMMU_OK;
        }
    } else if (host) {
        // Any other shape: the splitters of the general path count while they split, two small kernels leave the
        // sums for `guess` and `guess - 1` in the mapped buffer, and the product follows at once; one wait at the end.
        L = make_layout(m, n, k, guess, cplx);
        unsigned char* ws = static_cast<unsigned char*>(workspace);
        hipError_t e = counting_splits(cplx, L, m, n, k, A, lda, B, ldb, guess, ws, host, st);
        if (e == hipSuccess)
            e = cplx ? run_complex_products(L, m, n, guess, ws, C, ldc, st) : run_product(L, m, n, guess, ws, 0, 0, C, ldc, 0, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return OZIMMU_ERR_HIP;
        if (guess_holds(host, cplx ? 4 : 2, count_a, count_b, threshold, guess, max_slices)) {
            *num_slices = guess;
            if (guess_confirmed) *guess_confirmed = 1;
            return OZIMMU_OK;
        }
    }
    int s = 0;
    ozimmu_status_t rc = ozimmu_auto_num_slices(m, n, k, A, lda, B, ldb, cplx, threshold, max_slices, scratch, scratch_bytes,
                                                &s, nullptr, stream);
    if (rc != OZIMMU_OK) return rc;
    rc = product(s);
    if (rc == OZIMMU_OK) *num_slices = s;
    return rc;
}

}  // namespace

extern "C" {

const char* ozimmu_status_string(ozimmu_status_t status) {
    switch (status) {
        case OZIMMU_OK: return "ok";
        case OZIMMU_ERR_BAD_DIM: return "bad dimension or k-range";
        case OZIMMU_ERR_BAD_LD: return "leading dimension too small";
        case OZIMMU_ERR_BAD_SLICES: return "bad slice count or slice index";
        case OZIMMU_ERR_NULL: return "null pointer";
        case OZIMMU_ERR_WORKSPACE: return "workspace null, misaligned or too small";
        case OZIMMU_ERR_HIP: return "HIP error";
        case OZIMMU_ERR_NOT_IMPLEMENTED: return "not implemented";
        case OZIMMU_ERR_TOO_LARGE: return "product too large for the built-in scratch (use a workspace)";
    }
    return "unknown status";
}

ozimmu_status_t ozimmu_slice_geometry(int64_t rows, int64_t k, int64_t* rows_padded, int64_t* k_padded) {
    if (rows < 0 || k < 0 || rows > kMaxDim || k > kMaxDim) return OZIMMU_ERR_BAD_DIM;
    if (!rows_padded || !k_padded) return OZIMMU_ERR_NULL;
    *rows_padded = round_up(rows, kRowAlign);
    *k_padded = round_up(k, kSlab);
    return OZIMMU_OK;
}

int64_t ozimmu_slice_offset(int64_t rows_padded, int64_t k_padded, int slice, int64_t row, int64_t l) {
    if (slice < 0 || row < 0 || l < 0 || row >= rows_padded || l >= k_padded) return -1;
    const int64_t rr = row % kFragRows, h = (l % kSlab) / 16;
    return (int64_t)slice * rows_padded * k_padded + ((row / kFragRows) * (k_padded / kSlab) + l / kSlab) * kFragBytes +
           rr * kSlab + ((h ^ ((rr >> 3) & 1)) << 4) + l % 16;
}

ozimmu_status_t ozimmu_split_rows(int64_t m, int64_t k, const double* A, int64_t lda, int num_slices,
                                  int8_t* slices, int32_t* exps, void* stream) {
    if (!dims_ok(m, k, 0)) return OZIMMU_ERR_BAD_DIM;
    if (num_slices < 1 || num_slices > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    if (m == 0) return OZIMMU_OK;
    if (lda < k) return OZIMMU_ERR_BAD_LD;
    if (!exps || (k > 0 && (!A || !slices))) return OZIMMU_ERR_NULL;
    return hip_status(launch_split_rows(A, lda, 1, m, k, num_slices, slices, round_up(m, kRowAlign),
                                        round_up(k, kSlab), exps, static_cast<hipStream_t>(stream)));
}

ozimmu_status_t ozimmu_split_cols(int64_t k, int64_t n, const double* B, int64_t ldb, int num_slices,
                                  int8_t* slices, int32_t* exps, void* col_scratch, void* stream) {
    if (!dims_ok(n, k, 0)) return OZIMMU_ERR_BAD_DIM;
    if (num_slices < 1 || num_slices > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    if (n == 0) return OZIMMU_OK;
    if (ldb < n) return OZIMMU_ERR_BAD_LD;
    if (!exps || !col_scratch || (k > 0 && (!B || !slices))) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(col_scratch) % 8 != 0) return OZIMMU_ERR_WORKSPACE;
    return hip_status(launch_split_cols(B, ldb, 1, k, n, num_slices, slices, round_up(n, kRowAlign),
                                        round_up(k, kSlab), exps,
                                        static_cast<unsigned long long*>(col_scratch),
                                        static_cast<hipStream_t>(stream)));
}

ozimmu_status_t ozimmu_slice_gemm(int64_t m, int64_t n, int64_t k, const int8_t* SA, const int8_t* SB, int p,
                                  int q, int64_t k0, int64_t klen, int32_t* P, int64_t ldp, void* stream) {
    if (!dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    if (p < 1 || q < 1 || p > OZIMMU_MAX_SLICES || q > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    if (k0 < 0 || klen < 0 || k0 + klen > k || klen > OZIMMU_INT32_BLOCK || k0 % kSlab != 0)
        return OZIMMU_ERR_BAD_DIM;
    if (klen % kSlab != 0 && k0 + klen != k) return OZIMMU_ERR_BAD_DIM;
    if (m == 0 || n == 0) return OZIMMU_OK;
    if (ldp < n) return OZIMMU_ERR_BAD_LD;
    if (!P || (klen > 0 && (!SA || !SB))) return OZIMMU_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (klen == 0) return hip_status(launch_fill_i32(P, ldp, m, n, 0, st));
    const Layout L = make_layout(m, n, k, 1, false);   // the one-slice problem of slices p and q
    GemmArgs g{};
    g.a_slice_stride = L.m_pad * L.k_pad;
    g.b_slice_stride = L.n_pad * L.k_pad;
    g.SA = SA + (int64_t)(p - 1) * g.a_slice_stride;
    g.SB = SB + (int64_t)(q - 1) * g.b_slice_stride;
    g.kslabs = (int)(L.k_pad / kSlab);
    g.t_begin = (int)(k0 / kSlab);
    g.t_end = (int)(round_up(k0 + klen, kSlab) / kSlab);
    g.tiles_m = L.tiles_m;
    g.tiles_n = L.tiles_n;
    g.tile_cols = L.tile_cols;
    g.m = (int)m;
    g.n = (int)n;
    g.P = P;
    g.ldp = ldp;
    return hip_status(launch_slice_gemm(g, 1, 0, st));
}

ozimmu_status_t ozimmu_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_slices, int is_complex,
                                       size_t* bytes) {
    if (!dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    if (num_slices < 1 || num_slices > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    if (!bytes) return OZIMMU_ERR_NULL;
    *bytes = make_layout(m, n, k, num_slices, is_complex != 0).total;
    return OZIMMU_OK;
}

ozimmu_status_t ozimmu_dgemm_stage(int stage, int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                   const double* B, int64_t ldb, double* C, int64_t ldc, int num_slices,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    Layout L{};
    ozimmu_status_t rc = check_gemm_args(m, n, k, A, lda, B, ldb, C, ldc, num_slices, workspace, workspace_bytes,
                                         false, &L);
    if (rc != OZIMMU_OK || m == 0 || n == 0) return rc;
    if (stage < 0 || stage > 2) return OZIMMU_ERR_BAD_DIM;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (k == 0) return stage == 2 ? hip_status(launch_fill_f64(C, ldc, 1, m, n, 0.0, st)) : OZIMMU_OK;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    switch (stage) {
        case 0:
            return hip_status(launch_split_rows(A, lda, 1, m, k, num_slices,
                                                reinterpret_cast<int8_t*>(ws + L.off_sa[0]), L.m_pad, L.k_pad,
                                                reinterpret_cast<int32_t*>(ws + L.off_ea[0]), st));
        case 1:
            return hip_status(launch_split_cols(B, ldb, 1, k, n, num_slices,
                                                reinterpret_cast<int8_t*>(ws + L.off_sb[0]), L.n_pad, L.k_pad,
                                                reinterpret_cast<int32_t*>(ws + L.off_eb[0]),
                                                reinterpret_cast<unsigned long long*>(ws + L.off_colmax), st));
        default:
            return hip_status(run_product(L, m, n, num_slices, ws, 0, 0, C, ldc, 0, st));
    }
}

ozimmu_status_t ozimmu_dgemm(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B,
                             int64_t ldb, double* C, int64_t ldc, int num_slices, void* workspace,
                             size_t workspace_bytes, void* stream) {
    for (int stage = 0; stage < 3; ++stage) {
        ozimmu_status_t rc = ozimmu_dgemm_stage(stage, m, n, k, A, lda, B, ldb, C, ldc, num_slices, workspace,
                                                workspace_bytes, stream);
        if (rc != OZIMMU_OK) return rc;
    }
    return OZIMMU_OK;
}

ozimmu_status_t ozimmu_zgemm(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B,
                             int64_t ldb, double* C, int64_t ldc, int num_slices, void* workspace,
                             size_t workspace_bytes, void* stream) {
    Layout L{};
    ozimmu_status_t rc = check_gemm_args(m, n, k, A, lda, B, ldb, C, ldc, num_slices, workspace, workspace_bytes,
                                         true, &L);
    if (rc != OZIMMU_OK || m == 0 || n == 0) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (k == 0) {
        hipError_t e = launch_fill_f64(C, 2 * ldc, 2, m, n, 0.0, st);
        if (e == hipSuccess) e = launch_fill_f64(C + 1, 2 * ldc, 2, m, n, 0.0, st);
        return hip_status(e);
    }
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const int s = num_slices;
    hipError_t e = hipSuccess;
    // a small B on a tall A (a gate on a state vector): one kernel that splits A on the fly and reads it once
    if (gate_product_applies(A, B, C, n, k, s)) return hip_status(launch_gate_product(A, lda, m, k, n, B, ldb, s, ws + L.off_gate, C, ldc, st));
    // the real and imaginary planes are separated while splitting (element stride 2)
    e = split_complex_rows(A, lda, m, k, s, ws, L.off_sa, L.off_ea, L.m_pad, L.k_pad, st, false);
    if (e == hipSuccess)
        e = launch_split_cols_complex(B, ldb, k, n, s, reinterpret_cast<int8_t*>(ws + L.off_sb[0]),
                                      reinterpret_cast<int8_t*>(ws + L.off_sb[1]), L.n_pad, L.k_pad,
                                      reinterpret_cast<int32_t*>(ws + L.off_eb[0]), reinterpret_cast<int32_t*>(ws + L.off_eb[1]),
                                      reinterpret_cast<unsigned long long*>(ws + L.off_colmax), st);
    if (e == hipSuccess) e = run_complex_products(L, m, n, s, ws, C, ldc, st);
    return hip_status(e);
}

ozimmu_status_t ozimmu_auto_scratch_bytes(int64_t n, size_t* bytes) {
    if (n < 0 || n > kMaxDim) return OZIMMU_ERR_BAD_DIM;
    if (!bytes) return OZIMMU_ERR_NULL;
    *bytes = 512 + 2 * sizeof(unsigned long long) * (size_t)round_up(n, kRowAlign);   // the sums, then column maxima of two planes
    return OZIMMU_OK;
}

ozimmu_status_t ozimmu_auto_num_slices(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                       const double* B, int64_t ldb, int is_complex, double threshold,
                                       int max_slices, void* scratch, size_t scratch_bytes,
                                       int* num_slices, uint64_t* loss_sums, void* stream) {
    if (!dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    if ((m > 0 && lda < k) || (k > 0 && ldb < n)) return OZIMMU_ERR_BAD_LD;
    // row-major A (m x k): rows as stored; row-major B (k x n): columns of the stored array
    const ScanOperand a{A, lda, m, k, false}, b{B, ldb, k, n, true};
    return auto_select(a, b, n, is_complex, threshold, max_slices, scratch, scratch_bytes, num_slices, loss_sums,
                       stream);
}

ozimmu_status_t ozimmu_dgemm_auto(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B,
                                  int64_t ldb, double* C, int64_t ldc, double threshold, int max_slices, int guess,
                                  void* workspace, size_t workspace_bytes, void* scratch, size_t scratch_bytes,
                                  int* num_slices, int* guess_confirmed, void* stream) {
    return gemm_auto(false, m, n, k, A, lda, B, ldb, C, ldc, threshold, max_slices, guess, workspace, workspace_bytes,
                     scratch, scratch_bytes, num_slices, guess_confirmed, stream);
}

ozimmu_status_t ozimmu_zgemm_auto(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B,
                                  int64_t ldb, double* C, int64_t ldc, double threshold, int max_slices, int guess,
                                  void* workspace, size_t workspace_bytes, void* scratch, size_t scratch_bytes,
                                  int* num_slices, int* guess_confirmed, void* stream) {
    return gemm_auto(true, m, n, k, A, lda, B, ldb, C, ldc, threshold, max_slices, guess, workspace, workspace_bytes,
                     scratch, scratch_bytes, num_slices, guess_confirmed, stream);
}

ozimmu_status_t ozimmu_auto_num_slices_blas(char transa, char transb, int64_t m, int64_t n, int64_t k,
                                            const double* A, int64_t lda, const double* B, int64_t ldb,
                                            int is_complex, double threshold, int max_slices, void* scratch,
                                            size_t scratch_bytes, int* num_slices, uint64_t* loss_sums,
                                            void* stream) {
    const int ta = parse_trans(transa), tb = parse_trans(transb);
    if (ta < 0 || tb < 0 || !dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    const int64_t one = 1;
    if (lda < std::max(one, ta ? k : m) || ldb < std::max(one, tb ? n : k)) return OZIMMU_ERR_BAD_LD;
    // A column-major r x c array is the row-major c x r array with the same leading dimension.
    // Exponents go with the rows of op(A) and the columns of op(B): those are rows of the stored
    // row-major array when the operand is transposed (A) or not transposed (B).
    const ScanOperand a = ta ? ScanOperand{A, lda, m, k, false} : ScanOperand{A, lda, k, m, true};
    const ScanOperand b = tb ? ScanOperand{B, ldb, k, n, true} : ScanOperand{B, ldb, n, k, false};
    return auto_select(a, b, std::max(m, n), is_complex, threshold, max_slices, scratch, scratch_bytes, num_slices,
                       loss_sums, stream);
}

// count_sums (device or mapped host memory, [2][16]; or null): the splitters also count for the check of num_slices as
// the automatic slice count, and the bits op(A) and op(B) lose with num_slices and num_slices - 1 slices arrive there.
static ozimmu_status_t dgemm_blas_impl(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha,
                                       const double* A, int64_t lda, const double* B, int64_t ldb, double beta, double* C,
                                       int64_t ldc, int num_slices, void* workspace, size_t workspace_bytes,
                                       void* stream, unsigned long long* count_sums) {
    const int pa = parse_trans(transa), pb = parse_trans(transb);
    if (pa < 0 || pb < 0 || !dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    const bool ta = pa != 0, tb = pb != 0;
    if (num_slices < 1 || num_slices > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    const int64_t one = 1;
    if (lda < std::max(one, ta ? k : m) || ldb < std::max(one, tb ? n : k) || ldc < std::max(one, m))
        return OZIMMU_ERR_BAD_LD;
    if (m == 0 || n == 0) return OZIMMU_OK;
    if (!C) return OZIMMU_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Column-major C (m x n) is the row-major n x m array C^T = op(B)^T op(A)^T: the operands swap
    // roles, and an operand is split along whichever of its two storage directions runs along k.
    if (k == 0 || alpha == 0.0) return hip_status(launch_scale_f64(C, ldc, n, m, beta, st));
    if (!A || !B) return OZIMMU_ERR_NULL;
    const Layout L = make_layout(n, m, k, num_slices, false);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % OZIMMU_WORKSPACE_ALIGN) != 0 || workspace_bytes < L.total)
        return OZIMMU_ERR_WORKSPACE;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    int8_t* SR = reinterpret_cast<int8_t*>(ws + L.off_sa[0]);      // slices of op(B)^T: n rows of length k
    int8_t* SC = reinterpret_cast<int8_t*>(ws + L.off_sb[0]);      // slices of op(A): m rows of length k
    int32_t* ER = reinterpret_cast<int32_t*>(ws + L.off_ea[0]);
    int32_t* EC = reinterpret_cast<int32_t*>(ws + L.off_eb[0]);
    unsigned long long* colmax = reinterpret_cast<unsigned long long*>(ws + L.off_colmax);
    hipError_t e = hipSuccess;
    unsigned long long* slots_a = count_sums ? reinterpret_cast<unsigned long long*>(ws + L.off_scan) : nullptr;
    unsigned long long* slots_b = count_sums ? slots_a + scan_slots_bytes(1) / sizeof(unsigned long long) : nullptr;
    if (count_sums) e = launch_fill_u64(slots_a, (int64_t)(2 * scan_slots_bytes(1) / sizeof(unsigned long long)), 0ull, st);
    if (e == hipSuccess) {
        if (!tb) e = launch_split_rows(B, ldb, 1, n, k, num_slices, SR, L.m_pad, L.k_pad, ER, st, false, slots_b, 5);   // B: k x n, column j contiguous
        else e = launch_split_cols(B, ldb, 1, k, n, num_slices, SR, L.m_pad, L.k_pad, ER, colmax, st, false, slots_b, 5);  // B: n x k
    }
    if (e == hipSuccess) {
        if (!ta) e = launch_split_cols(A, lda, 1, k, m, num_slices, SC, L.n_pad, L.k_pad, EC, colmax, st, false, slots_a, 5);  // A: m x k
        else e = launch_split_rows(A, lda, 1, m, k, num_slices, SC, L.n_pad, L.k_pad, EC, st, false, slots_a, 5);              // A: k x m
    }
    if (e == hipSuccess && count_sums) e = launch_scan_reduce(slots_a, 1, num_slices, count_sums, st);
    if (e == hipSuccess && count_sums) e = launch_scan_reduce(slots_b, 1, num_slices, count_sums + OZIMMU_MAX_SLICES, st);
    if (e == hipSuccess) e = run_product(L, n, m, num_slices, ws, 0, 0, C, ldc, 3, st, alpha, beta);
    return hip_status(e);
}

ozimmu_status_t ozimmu_dgemm_blas(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha,
                                  const double* A, int64_t lda, const double* B, int64_t ldb, double beta, double* C,
                                  int64_t ldc, int num_slices, void* workspace, size_t workspace_bytes,
                                  void* stream) {
    return dgemm_blas_impl(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_slices, workspace,
                           workspace_bytes, stream, nullptr);
}

ozimmu_status_t ozimmu_zgemm_blas_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_slices, int beta_is_zero,
                                                  size_t* bytes) {
    if (!dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    if (num_slices < 1 || num_slices > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    if (!bytes) return OZIMMU_ERR_NULL;
    size_t total = make_layout(n, m, k, num_slices, true).total;
    if (!beta_is_zero) total = align_up(total + 2 * sizeof(double) * (size_t)m * (size_t)n);   // the product before the update
    *bytes = total;
    return OZIMMU_OK;
}

// count_sums ([4][16]: op(A) re, im, op(B) re, im; or null): as for dgemm_blas_impl; with counting the general path is
// taken whatever the shape.
static ozimmu_status_t zgemm_blas_impl(char transa, char transb, int64_t m, int64_t n, int64_t k, const double* alpha,
                                       const double* A, int64_t lda, const double* B, int64_t ldb, const double* beta,
                                       double* C, int64_t ldc, int num_slices, void* workspace, size_t workspace_bytes,
                                       void* stream, unsigned long long* count_sums) {
    const int ta = parse_trans(transa), tb = parse_trans(transb);
    if (ta < 0 || tb < 0 || !dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    if (num_slices < 1 || num_slices > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    const int64_t one = 1;
    if (lda < std::max(one, ta ? k : m) || ldb < std::max(one, tb ? n : k) || ldc < std::max(one, m))
        return OZIMMU_ERR_BAD_LD;
    if (!alpha || !beta) return OZIMMU_ERR_NULL;
    if (m == 0 || n == 0) return OZIMMU_OK;
    if (!C) return OZIMMU_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const double ar = alpha[0], ai = alpha[1], br = beta[0], bi = beta[1];
    const bool beta_zero = br == 0.0 && bi == 0.0;
    // As in ozimmu_dgemm_blas the column-major m x n result is the row-major n x m array
    // C^T = op(B)^T op(A)^T (a complex product commutes element by element, so the parts are the same).
    if (k == 0 || (ar == 0.0 && ai == 0.0)) return hip_status(launch_zaxpby(nullptr, 0, C, ldc, n, m, 0.0, 0.0, br, bi, st));
    if (!A || !B) return OZIMMU_ERR_NULL;
    size_t need = 0;
    ozimmu_zgemm_blas_workspace_bytes(m, n, k, num_slices, beta_zero, &need);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % OZIMMU_WORKSPACE_ALIGN) != 0 || workspace_bytes < need)
        return OZIMMU_ERR_WORKSPACE;
    const Layout L = make_layout(n, m, k, num_slices, true);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    unsigned long long* colmax = reinterpret_cast<unsigned long long*>(ws + L.off_colmax);
    hipError_t e = hipSuccess;
    const bool alpha_one = ar == 1.0 && ai == 0.0;
    // The product goes straight into C when C's old values are not needed, else beside the slices.
    double* G = beta_zero ? C : reinterpret_cast<double*>(ws + align_up(L.total));
    const int64_t ldg = beta_zero ? ldc : m;
    // Neither operand transposed, a small A on a wide B (a gate on a state vector whose amplitudes are the columns'
    // entries): the row-major product B^T A^T has the state as its tall operand and takes the one-kernel path.
    if (!count_sums && !ta && !tb && gate_product_applies(B, A, G, m, k, num_slices)) {
        e = launch_gate_product(B, ldb, n, k, m, A, lda, num_slices, ws + L.off_gate, G, ldg, st);
        if (e == hipSuccess && !(beta_zero && alpha_one)) e = launch_zaxpby(G, ldg, C, ldc, n, m, ar, ai, br, bi, st);
        return hip_status(e);
    }
    unsigned long long* slots_a = count_sums ? reinterpret_cast<unsigned long long*>(ws + L.off_scan) : nullptr;
    unsigned long long* slots_b = count_sums ? slots_a + scan_slots_bytes(2) / sizeof(unsigned long long) : nullptr;
    if (count_sums) e = launch_fill_u64(slots_a, (int64_t)(2 * scan_slots_bytes(2) / sizeof(unsigned long long)), 0ull, st);
    // planes: real, then imaginary (negated while splitting if the operand is conjugated)
    if (e == hipSuccess) {
        if (!tb) e = split_complex_rows(B, ldb, n, k, num_slices, ws, L.off_sa, L.off_ea, L.m_pad, L.k_pad, st, false, slots_b);   // op(B)^T: n rows of length k
        else
            e = launch_split_cols_complex(B, ldb, k, n, num_slices, reinterpret_cast<int8_t*>(ws + L.off_sa[0]),
                                          reinterpret_cast<int8_t*>(ws + L.off_sa[1]), L.m_pad, L.k_pad,
                                          reinterpret_cast<int32_t*>(ws + L.off_ea[0]), reinterpret_cast<int32_t*>(ws + L.off_ea[1]),
                                          colmax, st, tb == 2, slots_b);
    }
    if (e == hipSuccess) {
        if (ta) e = split_complex_rows(A, lda, m, k, num_slices, ws, L.off_sb, L.off_eb, L.n_pad, L.k_pad, st, ta == 2, slots_a);   // op(A): m rows of length k
        else
            e = launch_split_cols_complex(A, lda, k, m, num_slices, reinterpret_cast<int8_t*>(ws + L.off_sb[0]),
                                          reinterpret_cast<int8_t*>(ws + L.off_sb[1]), L.n_pad, L.k_pad,
                                          reinterpret_cast<int32_t*>(ws + L.off_eb[0]), reinterpret_cast<int32_t*>(ws + L.off_eb[1]),
                                          colmax, st, false, slots_a);
    }
    if (e == hipSuccess && count_sums) e = launch_scan_reduce(slots_a, 2, num_slices, count_sums, st);
    if (e == hipSuccess && count_sums) e = launch_scan_reduce(slots_b, 2, num_slices, count_sums + 2 * OZIMMU_MAX_SLICES, st);
    if (e == hipSuccess) e = run_complex_products(L, n, m, num_slices, ws, G, ldg, st);
    if (e == hipSuccess && !(beta_zero && alpha_one)) e = launch_zaxpby(G, ldg, C, ldc, n, m, ar, ai, br, bi, st);
    return hip_status(e);
}

ozimmu_status_t ozimmu_zgemm_blas(char transa, char transb, int64_t m, int64_t n, int64_t k, const double* alpha,
                                  const double* A, int64_t lda, const double* B, int64_t ldb, const double* beta,
                                  double* C, int64_t ldc, int num_slices, void* workspace, size_t workspace_bytes,
                                  void* stream) {
    return zgemm_blas_impl(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_slices, workspace,
                           workspace_bytes, stream, nullptr);
}

// ozimmu_auto_num_slices_blas followed by ozimmu_dgemm_blas / ozimmu_zgemm_blas, as one call (see ozimmu.h).
static ozimmu_status_t gemm_blas_auto(bool cplx, char transa, char transb, int64_t m, int64_t n, int64_t k,
                                      const double* alpha, const double* A, int64_t lda, const double* B, int64_t ldb,
                                      const double* beta, double* C, int64_t ldc, double threshold, int max_slices,
                                      int guess, void* workspace, size_t workspace_bytes, void* scratch,
                                      size_t scratch_bytes, int* num_slices, int* guess_confirmed, void* stream) {
    if (max_slices < 1 || max_slices > OZIMMU_MAX_SLICES || !(threshold >= 0.0)) return OZIMMU_ERR_BAD_SLICES;
    if (!num_slices || !alpha || !beta) return OZIMMU_ERR_NULL;
    if (guess_confirmed) *guess_confirmed = 0;
    if (parse_trans(transa) < 0 || parse_trans(transb) < 0 || !dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    const bool beta_zero = beta[0] == 0.0 && (!cplx || beta[1] == 0.0);
    const bool alpha_zero = alpha[0] == 0.0 && (!cplx || alpha[1] == 0.0);
    // the workspace must serve whichever slice count comes out
    for (int s = 1; s <= max_slices; ++s) {
        size_t need = 0;
        const ozimmu_status_t rc = cplx ? ozimmu_zgemm_blas_workspace_bytes(m, n, k, s, beta_zero, &need)
                                        : ozimmu_workspace_bytes(n, m, k, s, 0, &need);
        if (rc != OZIMMU_OK) return rc;
        if (m > 0 && n > 0 && k > 0 && !alpha_zero && workspace_bytes < need) return OZIMMU_ERR_WORKSPACE;
    }
    if (!scratch_ok(scratch, scratch_bytes, std::max(m, n))) return OZIMMU_ERR_WORKSPACE;
    auto product = [&](int s, unsigned long long* count_sums) {
        return cplx ? zgemm_blas_impl(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, s, workspace,
                                      workspace_bytes, stream, count_sums)
                    : dgemm_blas_impl(transa, transb, m, n, k, alpha[0], A, lda, B, ldb, beta[0], C, ldc, s, workspace,
                                      workspace_bytes, stream, count_sums);
    };
    // Only a product that overwrites C can be formed on a guess: with beta != 0 a wrong guess would have used up C's old values.
    const bool speculate = guess >= 1 && guess <= max_slices && beta_zero && !alpha_zero && m > 0 && n > 0 && k > 0;
    unsigned long long* host = speculate ? mapped_sums() : nullptr;
    if (host) {
        const ozimmu_status_t rc = product(guess, host);
        if (rc != OZIMMU_OK) return rc;
        if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return OZIMMU_ERR_HIP;
        if (guess_holds(host, cplx ? 4 : 2, (double)m * (double)k, (double)k * (double)n, threshold, guess, max_slices)) {
            *num_slices = guess;
            if (guess_confirmed) *guess_confirmed = 1;
            return OZIMMU_OK;
        }
    }
    int s = 0;
    ozimmu_status_t rc = ozimmu_auto_num_slices_blas(transa, transb, m, n, k, A, lda, B, ldb, cplx, threshold, max_slices,
                                                     scratch, scratch_bytes, &s, nullptr, stream);
    if (rc != OZIMMU_OK) return rc;
    rc = product(s, nullptr);
    if (rc == OZIMMU_OK) *num_slices = s;
    return rc;
}

ozimmu_status_t ozimmu_dgemm_blas_auto(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha,
                                       const double* A, int64_t lda, const double* B, int64_t ldb, double beta, double* C,
                                       int64_t ldc, double threshold, int max_slices, int guess, void* workspace,
                                       size_t workspace_bytes, void* scratch, size_t scratch_bytes, int* num_slices,
                                       int* guess_confirmed, void* stream) {
    return gemm_blas_auto(false, transa, transb, m, n, k, &alpha, A, lda, B, ldb, &beta, C, ldc, threshold, max_slices,
                          guess, workspace, workspace_bytes, scratch, scratch_bytes, num_slices, guess_confirmed, stream);
}

ozimmu_status_t ozimmu_zgemm_blas_auto(char transa, char transb, int64_t m, int64_t n, int64_t k, const double* alpha,
                                       const double* A, int64_t lda, const double* B, int64_t ldb, const double* beta,
                                       double* C, int64_t ldc, double threshold, int max_slices, int guess,
                                       void* workspace, size_t workspace_bytes, void* scratch, size_t scratch_bytes,
                                       int* num_slices, int* guess_confirmed, void* stream) {
    // a small gate on a wide state, plain product: the one-kernel path, which counts on its way over the state
    if (alpha && beta && alpha[0] == 1.0 && alpha[1] == 0.0 && beta[0] == 0.0 && beta[1] == 0.0 &&
        parse_trans(transa) == 0 && parse_trans(transb) == 0 && m > 0 && n > 0 && k > 0 && guess >= 1 &&
        guess <= OZIMMU_MAX_SLICES && lda >= m && ldb >= k && ldc >= m && gate_product_applies(B, A, C, m, k, guess))
        return gemm_auto(true, n, m, k, B, ldb, A, lda, C, ldc, threshold, max_slices, guess, workspace, workspace_bytes,
                         scratch, scratch_bytes, num_slices, guess_confirmed, stream);
    return gemm_blas_auto(true, transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, threshold, max_slices,
                          guess, workspace, workspace_bytes, scratch, scratch_bytes, num_slices, guess_confirmed, stream);
}

ozimmu_status_t ozimmu_dgemm_dd(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B,
                                int64_t ldb, double* C_hi, double* C_lo, int64_t ldc, int num_slices,
                                void* workspace, size_t workspace_bytes, void* stream) {
    Layout L{};
    ozimmu_status_t rc = check_gemm_args(m, n, k, A, lda, B, ldb, C_hi, ldc, num_slices, workspace, workspace_bytes,
                                         false, &L);
    if (rc != OZIMMU_OK || m == 0 || n == 0) return rc;
    if (!C_lo) return OZIMMU_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (k == 0) {
        hipError_t e0 = launch_fill_f64(C_hi, ldc, 1, m, n, 0.0, st);
        if (e0 == hipSuccess) e0 = launch_fill_f64(C_lo, ldc, 1, m, n, 0.0, st);
        return hip_status(e0);
    }
    for (int stage = 0; stage < 2; ++stage) {   // the two splits are those of ozimmu_dgemm
        rc = ozimmu_dgemm_stage(stage, m, n, k, A, lda, B, ldb, C_hi, ldc, num_slices, workspace, workspace_bytes, stream);
        if (rc != OZIMMU_OK) return rc;
    }
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    set_tiles(L, m, n, num_slices, false);   // the double-double kernels exist for the large tiles only
    return hip_status(run_product(L, m, n, num_slices, ws, 0, 0, C_hi, ldc, 0, st, 1.0, 0.0, C_lo));
}

ozimmu_status_t ozimmu_launch_plan(int64_t m, int64_t n, int64_t k, int num_slices, ozimmu_plan_t* plan) {
    if (!dims_ok(m, n, k)) return OZIMMU_ERR_BAD_DIM;
    if (num_slices < 1 || num_slices > OZIMMU_MAX_SLICES) return OZIMMU_ERR_BAD_SLICES;
    if (!plan) return OZIMMU_ERR_NULL;
    const Layout L = make_layout(m, n, k, num_slices, false);
    plan->tile_rows = L.tile_rows;
    plan->tile_cols = L.tile_cols;
    plan->workgroups = (int64_t)L.tiles_m * L.tiles_n;
    plan->bands = num_slices > kBand ? 2 : 1;
    plan->int32_block_steps = L.wide ? block_steps_for(num_slices) : 0;
    return OZIMMU_OK;
}

}  // extern "C"
