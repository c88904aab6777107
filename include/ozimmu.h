/*
 * ozimmu -- FP64 matrix product by the Ozaki scheme on the INT8 -> INT32 matrix cores of
 * one MI355X (gfx950). C ABI: plain pointers and sizes, no framework types.
 *
 * What is computed (Section 3.1 of the paper, "Matrix multiplication by the Ozaki scheme
 * on IMMU" and "SplitInt"):
 *   1. every row of A and every column of B gets one power-of-two exponent, and its
 *      elements are cut into num_slices signed 7-bit chunks below that exponent;
 *   2. the slice pairs (p, q) with p + q <= num_slices + 1 are multiplied as INT8 matrices
 *      with exact INT32 accumulation (blocked so that no INT32 sum can overflow);
 *   3. the integer products are scaled by 2^(-7 (p + q)) e_A e_B^T and summed in FP64.
 * Order of the FP64 sum (fixed, part of the contract): the products of one anti-diagonal
 * d = p + q are first added as integers (exact), then
 *     acc = 0;  for d = num_slices + 1 down to 2:  acc = RN(acc + S_d 2^(-7 d));
 *     C_ij = acc * 2^(EA_i + EB_j)      (one ldexp).
 *
 * General rules for every entry point
 *   - All matrix pointers are DEVICE pointers owned by the caller; all matrices are
 *     row-major; leading dimensions count elements (complex: complex elements).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). All work is
 *     enqueued on it; no entry point synchronises, allocates or frees device memory, or
 *     keeps state between calls (exceptions, stated where they are declared:
 *     ozimmu_auto_num_slices and the *_auto products return a value to the host and wait for the stream;
 *     ozimmu_dgemm_static uses the library's own scratch array; the library remembers per
 *     device that it has raised a kernel's dynamic LDS limit). Calls that share a workspace must
 *     be stream-ordered.
 *   - Only kernels are enqueued (no memsets or copies), so the calls can be captured into
 *     a HIP graph. The first launch of a kernel on a device raises that kernel's dynamic
 *     LDS limit (a host-side driver call, once): make one ordinary call before capturing.
 *   - Arguments are validated on the host before anything is launched; on an argument
 *     error nothing is enqueued and outputs are untouched.
 *   - Inputs must be finite; the result for NaN/Inf inputs is unspecified. -0.0 is zero.
 *   - Return value: OZIMMU_OK or an error code; ozimmu_status_string() names it.
 */
#ifndef OZIMMU_H
#define OZIMMU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OZIMMU_OK = 0,
    OZIMMU_ERR_BAD_DIM = 1,        /* negative size, or a k-range that breaks the block rules */
    OZIMMU_ERR_BAD_LD = 2,         /* leading dimension smaller than the row length */
    OZIMMU_ERR_BAD_SLICES = 3,     /* num_slices outside [1, OZIMMU_MAX_SLICES], or bad (p, q) */
    OZIMMU_ERR_NULL = 4,           /* null pointer where data is required */
    OZIMMU_ERR_WORKSPACE = 5,      /* workspace null, misaligned or too small */
    OZIMMU_ERR_HIP = 6,            /* a HIP call or kernel launch failed */
    OZIMMU_ERR_NOT_IMPLEMENTED = 7,
    OZIMMU_ERR_TOO_LARGE = 8       /* the product needs more scratch than ozimmu_dgemm_static holds */
} ozimmu_status_t;

#define OZIMMU_MAX_SLICES 16
#define OZIMMU_SLICE_BITS 7          /* Table 2: INT8-INT32 keeps 7 magnitude bits per slice */
#define OZIMMU_ROW_ALIGN 128         /* slice rows are padded to a multiple of this */
#define OZIMMU_K_ALIGN 32            /* slice row length is padded to a multiple of this: the k-extent of
                                        one MFMA operand fragment (32 rows x 32 bytes = 1 KiB) */
#define OZIMMU_MAX_DIM 4194304       /* largest m, n or k accepted (2^22); beyond: OZIMMU_ERR_BAD_DIM */
#define OZIMMU_INT32_BLOCK 131072    /* at most 2^17 INT8 products go into one INT32 sum:
                                        2^17 * 127^2 < 2^31 (the exact limit is 133144) */
#define OZIMMU_WORKSPACE_ALIGN 256
#define OZIMMU_STATIC_SCRATCH_BYTES 67108864   /* 64 MiB: the built-in scratch of ozimmu_dgemm_static */

const char* ozimmu_status_string(ozimmu_status_t status);

/*
 * Slice tensors. The slices of `rows` rows of length k (A: rows = m; B^T: rows = n, so that both
 * operands of a slice product are "rows of length k", SplitInt header: M = A or B^T) are padded
 * to rows_padded = roundup(rows, OZIMMU_ROW_ALIGN) and k_padded = roundup(k, OZIMMU_K_ALIGN),
 * zero-filled outside [0,rows) x [0,k), and stored as the MFMA operand fragments the
 * slice-product kernel copies unchanged into LDS: a fragment = 32 rows x 32 positions of one slice,
 * 1 KiB contiguous, fragments ordered [slice][row / 32][l / 32]; inside a fragment row rr = r % 32
 * occupies bytes [32 rr, 32 rr + 32), its two 16-byte halves swapped when bit 3 of rr is set.
 * Element (slice s, row r, position l), with rr = r % 32, h = (l % 32) / 16, lives at byte offset
 *     s * rows_padded * k_padded
 *   + ((r / 32) * (k_padded / 32) + l / 32) * 1024
 *   + rr * 32 + ((h ^ ((rr / 8) % 2)) * 16) + l % 16
 * (ozimmu_slice_offset computes it). Size: num_slices * rows_padded * k_padded bytes.
 */
ozimmu_status_t ozimmu_slice_geometry(int64_t rows, int64_t k, int64_t* rows_padded,
                                      int64_t* k_padded);
/* Byte offset of element (slice, row, l) in a slice tensor of the given padded geometry
 * (host-side index arithmetic only); -1 if an index is out of range. */
int64_t ozimmu_slice_offset(int64_t rows_padded, int64_t k_padded, int slice, int64_t row, int64_t l);

/*
 * SplitInt on the rows of A (m x k, lda >= k).
 *   exps   [out] int32[m]: EA_i with 2^(EA_i - 1) <= max_l |A_il| < 2^(EA_i); 0 for a zero row.
 *   slices [out] slice tensor (layout above): element (p-1, i, l) = sign(A_il) * chunk p of
 *                |A_il| 2^(-EA_i), each chunk in [0, 127] (truncation, no rounding).
 * split_cols does the same for the columns of B (k x n, ldb >= n), i.e. for M = B^T:
 * exps int32[n], element (q-1, j, l) from B_lj. `col_scratch` is device memory of at least
 * 8 * roundup(n, OZIMMU_ROW_ALIGN) bytes, 8-byte aligned: the column maxima are reduced there with
 * atomics by one kernel and read by the next (an argument the algorithm itself does not have; it
 * keeps the library free of allocations).
 */
ozimmu_status_t ozimmu_split_rows(int64_t m, int64_t k, const double* A, int64_t lda,
                                  int num_slices, int8_t* slices, int32_t* exps, void* stream);
ozimmu_status_t ozimmu_split_cols(int64_t k, int64_t n, const double* B, int64_t ldb,
                                  int num_slices, int8_t* slices, int32_t* exps,
                                  void* col_scratch, void* stream);

/*
 * One slice product on the matrix cores (the product step of the IMMU algorithm), exposed so that
 * the raw INT32 accumulators can be checked:
 *     P[i][j] = sum_{l = k0}^{k0 + klen - 1} SA(p-1, i, l) * SB(q-1, j, l)     (INT32, exact)
 * SA, SB: slice tensors for m and n rows of length k holding at least p resp. q
 * slices. P: int32, m x n, row-major, ldp >= n. Rules: 1 <= p, q <= OZIMMU_MAX_SLICES;
 * klen <= OZIMMU_INT32_BLOCK; the range must consist of whole fragments: k0 a multiple of
 * OZIMMU_K_ALIGN (32), and klen too unless k0 + klen == k (the kernel has no masking inside a
 * fragment; beyond k the slices hold zeros). klen == 0 gives P = 0.
 */
ozimmu_status_t ozimmu_slice_gemm(int64_t m, int64_t n, int64_t k, const int8_t* SA,
                                  const int8_t* SB, int p, int q, int64_t k0, int64_t klen,
                                  int32_t* P, int64_t ldp, void* stream);

/*
 * Workspace size for ozimmu_dgemm / ozimmu_zgemm: slices of A and B, exponents, column maxima, and
 * -- only when num_slices * k_padded > OZIMMU_INT32_BLOCK (k-blocking) -- num_slices INT64 sums per
 * element of C. Otherwise every integer sum stays in registers. A complex product adds two m x n FP64
 * planes in which its real and imaginary parts are formed before C is written, once, interleaved,
 * and, with k and n small enough, room for B's slices in the form the kernel wants that splits A on
 * the fly (see ozimmu_zgemm).
 */
ozimmu_status_t ozimmu_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_slices,
                                       int is_complex, size_t* bytes);

/*
 * C = A . B (overwrite; the paper's problem statement has no alpha, beta or transposes).
 *   A: m x k, lda >= k.  B: k x n, ldb >= n.  C: m x n, ldc >= n, must not alias A or B.
 *   workspace: device memory, OZIMMU_WORKSPACE_ALIGN-aligned, at least
 *   ozimmu_workspace_bytes(...) bytes; contents are scratch.
 * m == 0 or n == 0: nothing to do. k == 0: C is set to +0.0.
 * ozimmu_zgemm: A, B, C hold interleaved (re, im) doubles (Section 4.4: the real and
 * imaginary parts are separated while splitting; four real products, each plane with its own
 * exponents; Cr = RN(G(Ar,Br) - G(Ai,Bi)), Ci = RN(G(Ar,Bi) + G(Ai,Br))).
 * With k <= 128 and n <= 128 (256 each with num_slices <= 8: a gate of up to eight qubits applied
 * to a state vector) and A, B, C 16-byte aligned, A is split inside the product kernel and read once; the
 * result is the same bit for bit, and of the workspace only the part set aside for B's slices is used.
 */
ozimmu_status_t ozimmu_dgemm(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                             const double* B, int64_t ldb, double* C, int64_t ldc,
                             int num_slices, void* workspace, size_t workspace_bytes,
                             void* stream);
ozimmu_status_t ozimmu_zgemm(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                             const double* B, int64_t ldb, double* C, int64_t ldc,
                             int num_slices, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * ozimmu_dgemm for callers that cannot allocate device memory or carry a workspace around: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments and
 * result as ozimmu_dgemm (bit for bit) without the workspace: the library's own scratch, a device
 * array of OZIMMU_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process
 * ends, takes its place. The call allocates and frees nothing and only enqueues kernels. A product
 * whose ozimmu_workspace_bytes(m, n, k, num_slices, 0) exceeds OZIMMU_STATIC_SCRATCH_BYTES is
 * refused with OZIMMU_ERR_TOO_LARGE before anything is enqueued (use ozimmu_dgemm with a
 * workspace of your own). All calls on one GPU share that GPU's scratch: calls that overlap on one
 * GPU (different streams without ordering between them, or several host threads) race; calls on one
 * stream, or ordered by events, are safe. The first call on a device looks the array's address up
 * (hipGetSymbolAddress, no allocation).
 */
ozimmu_status_t ozimmu_dgemm_static(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                    const double* B, int64_t ldb, double* C, int64_t ldc,
                                    int num_slices, void* stream);

/*
 * The stages of ozimmu_dgemm run one at a time, for per-stage timing and profiling
 * (the time breakdown of Section 4.3): stage 0 = split A, 1 = split B, 2 = slice products
 * with the fused FP64 sum. Stages must be run in order with the same arguments.
 */
ozimmu_status_t ozimmu_dgemm_stage(int stage, int64_t m, int64_t n, int64_t k, const double* A,
                                   int64_t lda, const double* B, int64_t ldb, double* C,
                                   int64_t ldc, int num_slices, void* workspace,
                                   size_t workspace_bytes, void* stream);

/*
 * How ozimmu_dgemm runs a shape, on the host only (nothing is launched; for tests and for callers
 * who want to know): the tile of C one workgroup owns (64 x 128; 64 x 64 from fourteen slices on, and up to
 * nine slices when k <= 512 or fewer than 256 of the larger tiles exist), the number of workgroups, the number of bands
 * the anti-diagonals are walked in (a wavefront holds the INT32 sums of at most eight diagonals at a
 * time: 2 bands beyond eight slices), and int32_block_steps = the number of steps of
 * OZIMMU_K_ALIGN positions after which the INT32 sums are moved into INT64 sums (k-blocking),
 * 0 if a whole diagonal fits one INT32 sum.
 */
typedef struct {
    int tile_rows, tile_cols;
    int64_t workgroups;
    int bands;
    int int32_block_steps;
} ozimmu_plan_t;
ozimmu_status_t ozimmu_launch_plan(int64_t m, int64_t n, int64_t k, int num_slices, ozimmu_plan_t* plan);

/*
 * Product with the summing-up in double-double (Section 2.3.4, first advantage of the scheme: its
 * precision can be raised above FP64 by more slices and a more accurate summing-up). Same splits and
 * slice products as ozimmu_dgemm; the diagonal sums are added, least significant first, in
 * double-double arithmetic (TwoSum of the running high part and the exact term S_d 2^(-7d), error added
 * to the low part, FastTwoSum renormalisation after every term) and both parts are scaled by
 * 2^(EA_i + EB_j): C = C_hi + C_lo as an unevaluated sum, C_hi being the FP64-rounded value. C_hi and
 * C_lo are m x n row-major with the same leading dimension ldc. Workspace and errors as ozimmu_dgemm.
 */
ozimmu_status_t ozimmu_dgemm_dd(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                const double* B, int64_t ldb, double* C_hi, double* C_lo, int64_t ldc,
                                int num_slices, void* workspace, size_t workspace_bytes, void* stream);

/*
 * BLAS-style call (Section 4.4: the library stands in for the vendor DGEMM): COLUMN-MAJOR storage,
 * C <- alpha op(A) op(B) + beta C, op(X) = X ('N') or X^T ('T', 'C'); op(A) is m x k, op(B) is
 * k x n, C is m x n; leading dimensions as in the reference BLAS. G = the Ozaki product of op(A) and
 * op(B) as in ozimmu_dgemm (exponents per row of op(A) and per column of op(B)); then per element
 * C = RN(alpha G) if beta == 0 (C is not read), else C = RN(RN(alpha G) + RN(beta C)); if
 * alpha == 0 or k == 0 the product is not formed (A, B, workspace may be null): C = +0 or
 * RN(beta C). alpha and beta are host scalars. Workspace: ozimmu_workspace_bytes(n, m, k, ...)
 * (note the order: the operands swap roles internally). Errors: an unknown transpose letter gives
 * OZIMMU_ERR_BAD_DIM, the rest as for ozimmu_dgemm.
 */
ozimmu_status_t ozimmu_dgemm_blas(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha,
                                  const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
                                  double* C, int64_t ldc, int num_slices, void* workspace,
                                  size_t workspace_bytes, void* stream);

/*
 * Complex BLAS-style call (Section 4.4: complex GEMM from separated real and imaginary parts,
 * standing in for the vendor ZGEMM): COLUMN-MAJOR storage of interleaved (re, im) doubles, leading
 * dimensions in complex elements, C <- alpha op(A) op(B) + beta C, op(X) = X ('N'), X^T ('T') or
 * X^H ('C'); op(A) is m x k, op(B) is k x n, C is m x n. alpha and beta point to two host doubles
 * (re, im) each. G = the complex Ozaki product of op(A) and op(B) as in ozimmu_zgemm, the imaginary
 * plane of a conjugated operand being negated while it is split (exact). Then per element, every
 * operation one rounded FP64 operation:
 *     t = ( RN(RN(ar Gr) - RN(ai Gi)),  RN(RN(ar Gi) + RN(ai Gr)) )
 *     C = t                                         if beta == 0 (C is not read),
 *     u = beta C formed like t,  C = ( RN(tr + ur), RN(ti + ui) )   otherwise;
 * if alpha == 0 or k == 0 the product is not formed (A, B, workspace may be null): C = +0 or u.
 * With alpha == 1 and beta == 0 the product is written straight into C; with beta != 0 it is held in
 * the workspace until the update (16 m n bytes more). Workspace:
 * ozimmu_zgemm_blas_workspace_bytes(m, n, k, num_slices, beta_is_zero, &bytes). Errors as for
 * ozimmu_dgemm_blas; null alpha or beta gives OZIMMU_ERR_NULL.
 */
ozimmu_status_t ozimmu_zgemm_blas_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_slices,
                                                  int beta_is_zero, size_t* bytes);
ozimmu_status_t ozimmu_zgemm_blas(char transa, char transb, int64_t m, int64_t n, int64_t k,
                                  const double* alpha, const double* A, int64_t lda, const double* B,
                                  int64_t ldb, const double* beta, double* C, int64_t ldc, int num_slices,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Automatic choice of the number of slices (Section 4.4, "INT8-AUTO": all elements of the inputs
 * are inspected and the number of slices is taken so that the average mantissa loss of the split
 * stays within a threshold; threshold 0 means a lossless split).
 *
 * Definition used (the paper gives no formula): an element x != 0 whose row (A) or column (B) has
 * exponent E has its leading bit z + 1 places after the binary point of |x| 2^-E and stores L
 * significant bits (53; fewer if subnormal); s slices keep 7 s places, so the element loses
 * min(L, max(0, z + L - 7 s)) bits, counted by position. Zeros lose nothing and count in the
 * average. The average is taken per input matrix (per real plane if is_complex) over all its
 * elements. *num_slices = the smallest s in 1 .. max_slices for which every plane's sum of lost
 * bits is <= threshold * (number of elements), compared in double precision; max_slices if none.
 *
 * A, B: device pointers, row-major as for ozimmu_dgemm / ozimmu_zgemm (interleaved complex if
 * is_complex). scratch: device memory, 256-byte aligned, at least ozimmu_auto_scratch_bytes(n).
 * num_slices: HOST pointer. loss_sums: optional HOST array of planes * 16 uint64 (planes = 2, or
 * 4 if is_complex: A re, A im, B re, B im / A, B), receives the sums of lost bits for
 * s = 1 .. 16. Unlike the other entry points this one returns a result to the host: it
 * enqueues its kernels on `stream`, copies 512 bytes back and waits for the stream
 * (it cannot be captured into a graph). Errors as for ozimmu_dgemm; a negative or NaN threshold
 * or max_slices outside 1 .. 16 give OZIMMU_ERR_BAD_SLICES.
 */
ozimmu_status_t ozimmu_auto_scratch_bytes(int64_t n, size_t* bytes);
ozimmu_status_t ozimmu_auto_num_slices(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                       const double* B, int64_t ldb, int is_complex, double threshold,
                                       int max_slices, void* scratch, size_t scratch_bytes,
                                       int* num_slices, uint64_t* loss_sums, void* stream);

/*
 * ozimmu_auto_num_slices followed by ozimmu_dgemm / ozimmu_zgemm with the count it chose, as one call:
 * *num_slices receives the count, C the product; both are exactly what the two calls give. `guess` is
 * the caller's expectation of the count (say, the one the previous product of this shape took; 0: none).
 * With a guess the product is formed with it at once:
 *   - where ozimmu_zgemm runs as the kernel that splits A on the fly (see there), that kernel and the
 *     splitter of B count on their way what the check of the guess needs: a right guess means A has
 *     been read once instead of twice;
 *   - for every other shape the splitters count the same while they cut the slices, and the product
 *     follows at once: a right guess means no scan pass over either operand and a single wait.
 * A right guess sets *guess_confirmed = 1 (optional HOST pointer). A wrong one is followed by the
 * product with the count chosen, so it costs one product; without a guess the count is chosen first.
 * workspace: at least the largest ozimmu_workspace_bytes(m, n, k, s, is_complex) over
 * s = 1 .. max_slices; scratch: as for ozimmu_auto_num_slices. Waits for the stream like
 * ozimmu_auto_num_slices; errors as there and as for ozimmu_dgemm. These calls and
 * ozimmu_auto_num_slices receive their sums in 512 bytes of mapped host memory that the first such
 * call of a thread allocates and that is kept until the process ends.
 */
ozimmu_status_t ozimmu_dgemm_auto(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                  const double* B, int64_t ldb, double* C, int64_t ldc, double threshold,
                                  int max_slices, int guess, void* workspace, size_t workspace_bytes,
                                  void* scratch, size_t scratch_bytes, int* num_slices,
                                  int* guess_confirmed, void* stream);
ozimmu_status_t ozimmu_zgemm_auto(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                  const double* B, int64_t ldb, double* C, int64_t ldc, double threshold,
                                  int max_slices, int guess, void* workspace, size_t workspace_bytes,
                                  void* scratch, size_t scratch_bytes, int* num_slices,
                                  int* guess_confirmed, void* stream);

/*
 * The same choice for the operands of a BLAS-style call (ozimmu_dgemm_blas / ozimmu_zgemm_blas):
 * column-major A and B with transposes as there; the exponents go with the rows of op(A) and the
 * columns of op(B). scratch: at least ozimmu_auto_scratch_bytes(max(m, n)). Everything else as
 * ozimmu_auto_num_slices.
 */
ozimmu_status_t ozimmu_auto_num_slices_blas(char transa, char transb, int64_t m, int64_t n, int64_t k,
                                            const double* A, int64_t lda, const double* B, int64_t ldb,
                                            int is_complex, double threshold, int max_slices, void* scratch,
                                            size_t scratch_bytes, int* num_slices, uint64_t* loss_sums,
                                            void* stream);

/*
 * ozimmu_auto_num_slices_blas followed by ozimmu_dgemm_blas / ozimmu_zgemm_blas with the count it chose, as
 * one call, with `guess` as for ozimmu_dgemm_auto. The product is formed on the guess only when it
 * overwrites C (beta = 0: with another beta a wrong guess would have used up C's old values); then the
 * splitters count while they split (a small complex gate on a wide state, untransposed, with alpha = 1:
 * the one-kernel path of ozimmu_zgemm_auto). Otherwise the count is chosen first. workspace: at least
 * the largest ozimmu_workspace_bytes(n, m, k, s, 0) / ozimmu_zgemm_blas_workspace_bytes(m, n, k, s,
 * beta == 0) over s = 1 .. max_slices; scratch: at least ozimmu_auto_scratch_bytes(max(m, n)).
 * Everything else as for the calls it stands for and for ozimmu_dgemm_auto.
 */
ozimmu_status_t ozimmu_dgemm_blas_auto(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha,
                                       const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
                                       double* C, int64_t ldc, double threshold, int max_slices, int guess,
                                       void* workspace, size_t workspace_bytes, void* scratch,
                                       size_t scratch_bytes, int* num_slices, int* guess_confirmed, void* stream);
ozimmu_status_t ozimmu_zgemm_blas_auto(char transa, char transb, int64_t m, int64_t n, int64_t k,
                                       const double* alpha, const double* A, int64_t lda, const double* B,
                                       int64_t ldb, const double* beta, double* C, int64_t ldc, double threshold,
                                       int max_slices, int guess, void* workspace, size_t workspace_bytes,
                                       void* scratch, size_t scratch_bytes, int* num_slices,
                                       int* guess_confirmed, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* OZIMMU_H */
