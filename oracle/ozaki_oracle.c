/*
 * CPU oracle for the Ozaki-scheme DGEMM on an INT8 -> INT32 integer matrix unit.
 *
 * THIS IS TEST INFRASTRUCTURE. It is a plain, slow, step-by-step restatement of the
 * method ("Matrix multiplication by the Ozaki scheme on IMMU" and its "SplitInt"
 * splitting algorithm, Section 3.1 of the paper) that exists only so that the GPU
 * library can be checked against it. Nothing in the product path may call it, and it
 * shares no code, header, table or helper with the HIP kernels.
 *
 * Conventions (each function cites the passage it follows):
 *   - matrices are row-major doubles with a leading dimension;
 *   - W = 7 magnitude bits per slice (Table 2, INT8-INT32: l_in = 7; Eq. (5) BPS);
 *   - slices are stored as M = A or B^T ("SplitInt" header), i.e. both operands are
 *     "rows of length k": SA[p][i][l] and SB[q][j][l], slice index first, 0-based in
 *     memory (slice p of the paper is index p-1);
 *   - exponents are plain integers E with e = 2^E (the paper's exponent offset vector).
 *
 * Parity unpinned: the paper's error curves, its Table 3 figures and the slice counts
 * its automatic mode picked for its circuits (only in figures that are not available).
 *
 * No blocking, no fusion, no reordering beyond what is stated in each comment.
 * Compile with -ffp-contract=off (no fused multiply-add may be formed by the compiler;
 * the only FMA used is the explicit fma() of the double-double reference).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define OZ_W 7 /* magnitude bits kept per INT8 slice */

int oz_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------------------
 * Closed forms of Section 3.2.
 * ------------------------------------------------------------------------------- */

/* Eq. (4): alpha = floor((l_acc - log2 k) / 2). */
int oz_alpha(int l_acc, double k) { return (int)floor(((double)l_acc - log2(k)) / 2.0); }

/* Eq. (5): BPS = min(alpha, l_in). */
int oz_bps(int l_in, int l_acc, double k) {
    int a = oz_alpha(l_acc, k);
    return a < l_in ? a : l_in;
}

/* Number of slice products kept: the pairs with i + j <= s + 1, (s + 1) s / 2 of them
 * (Section 3.2.4, and the double loop of the IMMU algorithm). Counted, not computed
 * from the formula, so that the formula can be tested against it. */
int oz_num_pairs(int s) {
    int c = 0;
    for (int i = 1; i <= s; ++i)
        for (int j = 1; j <= s - i + 1; ++j) ++c;
    return c;
}

/* ---------------------------------------------------------------------------------
 * SplitInt, exponent step: one exponent per row of M.
 *
 * The paper takes the smallest power of two not below the row maximum. Reading used
 * here: E is the frexp exponent of mu = max_l |M_il|, i.e. mu = f * 2^E with
 * 0.5 <= f < 1, so |x| * 2^-E < 1 for every element of the row (at an exact power of
 * two this is one more than the ceiling of log2, which keeps the first chunk below
 * 128). A zero row gets E = 0.
 * ------------------------------------------------------------------------------- */
static int row_exponent(const double *row, int64_t len, int64_t stride) {
    double mu = 0.0;
    for (int64_t l = 0; l < len; ++l) {
        double a = fabs(row[l * stride]);
        if (a > mu) mu = a;
    }
    if (mu == 0.0) return 0;
    int E;
    (void)frexp(mu, &E);
    return E;
}

/* SplitInt, slice-extraction loop, for one element: the magnitude r = |x| 2^-E in [0,1) is cut
 * into consecutive 7-bit chunks below the row's leading place (truncation: the chunk
 * is floor of the shifted remainder), and each chunk carries the sign of x. */
static void split_element(double x, int E, int s, int8_t *out, int64_t slice_stride) {
    double r = ldexp(fabs(x), -E);
    int neg = signbit(x) != 0;
    for (int p = 0; p < s; ++p) {
        r = r * 128.0;         /* exact: power-of-two scaling, r stays below 128 */
        double q = floor(r);   /* 0 .. 127 */
        r = r - q;             /* exact: only leading bits are removed */
        int v = (int)q;
        out[(int64_t)p * slice_stride] = (int8_t)(neg ? -v : v);
    }
}

/* Split the rows of A (m x k, row-major, lda): exponents EA[m], slices SA[s][m][k]. */
void oz_split_rows(int64_t m, int64_t k, const double *A, int64_t lda, int s, int32_t *EA,
                   int8_t *SA) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        int E = row_exponent(A + i * lda, k, 1);
        EA[i] = E;
        for (int64_t l = 0; l < k; ++l)
            split_element(A[i * lda + l], E, s, SA + i * k + l, m * k);
    }
}

/* Split the columns of B (k x n, row-major, ldb), i.e. the rows of M = B^T:
 * exponents EB[n], slices SB[s][n][k] (column j of B becomes row j of the slice). */
void oz_split_cols(int64_t k, int64_t n, const double *B, int64_t ldb, int s, int32_t *EB,
                   int8_t *SB) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        int E = row_exponent(B + j, k, ldb);
        EB[j] = E;
        for (int64_t l = 0; l < k; ++l)
            split_element(B[l * ldb + j], E, s, SB + j * k + l, n * k);
    }
}

/* ---------------------------------------------------------------------------------
 * Product step of the IMMU algorithm: C_tmp = A^(p) . B^(q), exactly, for one pair and for
 * the k-range [k0, k0 + klen). P is m x n INT64, row-major, ld = n.
 * This is the definition (a triple loop); INT64 cannot overflow for any admissible k.
 * ------------------------------------------------------------------------------- */
void oz_pair_product(int64_t m, int64_t n, int64_t k, const int8_t *SAp, const int8_t *SBq,
                     int64_t k0, int64_t klen, int64_t *P) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            int64_t acc = 0;
            const int8_t *a = SAp + i * k + k0;
            const int8_t *b = SBq + j * k + k0;
            for (int64_t l = 0; l < klen; ++l) acc += (int64_t)a[l] * (int64_t)b[l];
            P[i * n + j] = acc;
        }
}

/* Sum of the products of one anti-diagonal d = p + q (2 <= d <= s + 1), in INT64:
 * S_d = sum_{p=1}^{d-1} A^(p) . B^(d-p). All pairs of a diagonal share the scale
 * 2^(-7 d) of the summing-up step, and integer addition is exact, so summing them before the
 * conversion to FP64 changes no mathematics. S is [s][m][n], S[d-2] = S_d. */
void oz_diagonal_sums(int64_t m, int64_t n, int64_t k, int s, const int8_t *SA,
                      const int8_t *SB, int64_t *S) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j)
            for (int d = 2; d <= s + 1; ++d) {
                int64_t acc = 0;
                for (int p = 1; p <= d - 1; ++p) {
                    int q = d - p;
                    const int8_t *a = SA + ((int64_t)(p - 1) * m + i) * k;
                    const int8_t *b = SB + ((int64_t)(q - 1) * n + j) * k;
                    for (int64_t l = 0; l < k; ++l) acc += (int64_t)a[l] * (int64_t)b[l];
                }
                S[((int64_t)(d - 2) * m + i) * n + j] = acc;
            }
}

/* ---------------------------------------------------------------------------------
 * Summing-up step of the IMMU algorithm: C = sum over the kept products of
 * C_tmp (.) 2^(-(i+j) W) e_A e_B^T, in FP64.
 *
 * Fixed order used as the definition of the result: the per-diagonal integer sums
 * are converted (exactly: |S_d| < 2^53) and added least significant diagonal first,
 *     acc = 0;  for d = s+1 down to 2:  acc = RN(acc + S_d * 2^(-7 d))
 * and the row/column scale 2^(EA_i + EB_j) is applied once at the end by ldexp
 * (identical to scaling every term unless the result leaves the normal range).
 * ------------------------------------------------------------------------------- */
void oz_accumulate(int64_t m, int64_t n, int s, const int64_t *S, const int32_t *EA,
                   const int32_t *EB, double *C, int64_t ldc) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int d = s + 1; d >= 2; --d) {
                double t = ldexp((double)S[((int64_t)(d - 2) * m + i) * n + j], -OZ_W * d);
                acc = acc + t;
            }
            C[i * ldc + j] = ldexp(acc, EA[i] + EB[j]);
        }
}

/* The whole method: split A, split B, integer products, FP64 sum. Returns 0, or 1
 * when memory for the slices could not be obtained. */
int oz_dgemm(int64_t m, int64_t n, int64_t k, const double *A, int64_t lda, const double *B,
             int64_t ldb, double *C, int64_t ldc, int s) {
    if (m == 0 || n == 0) return 0;
    int32_t *EA = malloc(sizeof(int32_t) * (size_t)m);
    int32_t *EB = malloc(sizeof(int32_t) * (size_t)n);
    int8_t *SA = malloc((size_t)s * (size_t)m * (size_t)(k ? k : 1));
    int8_t *SB = malloc((size_t)s * (size_t)n * (size_t)(k ? k : 1));
    int64_t *S = malloc(sizeof(int64_t) * (size_t)s * (size_t)m * (size_t)n);
    int rc = 1;
    if (EA && EB && SA && SB && S) {
        oz_split_rows(m, k, A, lda, s, EA, SA);
        oz_split_cols(k, n, B, ldb, s, EB, SB);
        oz_diagonal_sums(m, n, k, s, SA, SB, S);
        oz_accumulate(m, n, s, S, EA, EB, C, ldc);
        rc = 0;
    }
    free(EA); free(EB); free(SA); free(SB); free(S);
    return rc;
}

/* Cross-check only: the literal loop order of the IMMU algorithm (i outer, j inner,
 * one FP64 update of C per pair, every term scaled by 2^(-(i+j) W) e_A e_B^T).
 * It differs from oz_dgemm only in the order and number of FP64 roundings. */
int oz_dgemm_pairwise_order(int64_t m, int64_t n, int64_t k, const double *A, int64_t lda,
                            const double *B, int64_t ldb, double *C, int64_t ldc, int s) {
    if (m == 0 || n == 0) return 0;
    int32_t *EA = malloc(sizeof(int32_t) * (size_t)m);
    int32_t *EB = malloc(sizeof(int32_t) * (size_t)n);
    int8_t *SA = malloc((size_t)s * (size_t)m * (size_t)(k ? k : 1));
    int8_t *SB = malloc((size_t)s * (size_t)n * (size_t)(k ? k : 1));
    int64_t *P = malloc(sizeof(int64_t) * (size_t)m * (size_t)n);
    int rc = 1;
    if (EA && EB && SA && SB && P) {
        oz_split_rows(m, k, A, lda, s, EA, SA);
        oz_split_cols(k, n, B, ldb, s, EB, SB);
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) C[i * ldc + j] = 0.0;
        for (int i = 1; i <= s; ++i)
            for (int j = 1; j <= s - i + 1; ++j) {
                oz_pair_product(m, n, k, SA + (int64_t)(i - 1) * m * k,
                                SB + (int64_t)(j - 1) * n * k, 0, k, P);
                for (int64_t r = 0; r < m; ++r)
                    for (int64_t c = 0; c < n; ++c) {
                        double t = ldexp((double)P[r * n + c], -OZ_W * (i + j) + EA[r] + EB[c]);
                        C[r * ldc + c] = C[r * ldc + c] + t;
                    }
            }
        rc = 0;
    }
    free(EA); free(EB); free(SA); free(SB); free(P);
    return rc;
}

/* ---------------------------------------------------------------------------------
 * Complex product by separating real and imaginary parts during the split
 * (Section 4.4, first extension). A, B, C hold interleaved (re, im) doubles; ld counts
 * complex elements. Four real Ozaki products G(X, Y), each plane split with its own
 * exponents:  Cr = RN(G(Ar,Br) - G(Ai,Bi)),  Ci = RN(G(Ar,Bi) + G(Ai,Br)).
 * ------------------------------------------------------------------------------- */
int oz_zgemm(int64_t m, int64_t n, int64_t k, const double *A, int64_t lda, const double *B,
             int64_t ldb, double *C, int64_t ldc, int s) {
    if (m == 0 || n == 0) return 0;
    size_t ak = (size_t)m * (size_t)(k ? k : 1), bk = (size_t)(k ? k : 1) * (size_t)n;
    double *Ar = malloc(sizeof(double) * ak), *Ai = malloc(sizeof(double) * ak);
    double *Br = malloc(sizeof(double) * bk), *Bi = malloc(sizeof(double) * bk);
    double *G[4];
    for (int t = 0; t < 4; ++t) G[t] = malloc(sizeof(double) * (size_t)m * (size_t)n);
    int rc = 1;
    if (Ar && Ai && Br && Bi && G[0] && G[1] && G[2] && G[3]) {
        for (int64_t i = 0; i < m; ++i)
            for (int64_t l = 0; l < k; ++l) {
                Ar[i * k + l] = A[2 * (i * lda + l)];
                Ai[i * k + l] = A[2 * (i * lda + l) + 1];
            }
        for (int64_t l = 0; l < k; ++l)
            for (int64_t j = 0; j < n; ++j) {
                Br[l * n + j] = B[2 * (l * ldb + j)];
                Bi[l * n + j] = B[2 * (l * ldb + j) + 1];
            }
        rc = oz_dgemm(m, n, k, Ar, k, Br, n, G[0], n, s) |
             oz_dgemm(m, n, k, Ai, k, Bi, n, G[1], n, s) |
             oz_dgemm(m, n, k, Ar, k, Bi, n, G[2], n, s) |
             oz_dgemm(m, n, k, Ai, k, Br, n, G[3], n, s);
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) {
                C[2 * (i * ldc + j)] = G[0][i * n + j] - G[1][i * n + j];
                C[2 * (i * ldc + j) + 1] = G[2][i * n + j] + G[3][i * n + j];
            }
    }
    free(Ar); free(Ai); free(Br); free(Bi);
    for (int t = 0; t < 4; ++t) free(G[t]);
    return rc;
}

/* ---------------------------------------------------------------------------------
 * Reference the accuracy is measured against (Section 4.2, Eq. (7)): the product in
 * double-double arithmetic. Each a*b is taken exactly as (p, e) with an explicit fma
 * (TwoProd), added into the (hi, lo) pair with Knuth's TwoSum, and renormalised.
 * Outputs hi and lo with hi + lo the double-double value. Also |A||B| in FP64.
 * ------------------------------------------------------------------------------- */
void oz_dd_gemm(int64_t m, int64_t n, int64_t k, const double *A, int64_t lda, const double *B,
                int64_t ldb, double *Chi, double *Clo) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double hi = 0.0, lo = 0.0;
            for (int64_t l = 0; l < k; ++l) {
                double a = A[i * lda + l], b = B[l * ldb + j];
                double p = a * b;
                double e = fma(a, b, -p);      /* a*b = p + e exactly */
                double sum = hi + p;           /* TwoSum(hi, p) */
                double bb = sum - hi;
                double err = (hi - (sum - bb)) + (p - bb);
                lo = lo + (err + e);
                hi = sum + lo;                 /* FastTwoSum(sum, lo) */
                lo = lo - (hi - sum);
            }
            Chi[i * n + j] = hi;
            Clo[i * n + j] = lo;
        }
}

void oz_abs_gemm(int64_t m, int64_t n, int64_t k, const double *A, int64_t lda, const double *B,
                 int64_t ldb, double *G) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int64_t l = 0; l < k; ++l) acc = acc + fabs(A[i * lda + l]) * fabs(B[l * ldb + j]);
            G[i * n + j] = acc;
        }
}

/* ---------------------------------------------------------------------------------
 * Automatic choice of the number of slices (Section 4.4, "INT8-AUTO"): every element
 * of both inputs is inspected and the smallest number of slices is taken for which
 * the average number of mantissa bits lost in the splitting is at most a threshold T
 * (T = 0: the split loses nothing).
 *
 * Reading used here (the paper gives no formula). An element x != 0 of a row with
 * exponent E has its leading bit at fraction position z + 1 after the binary point of
 * |x| 2^-E (z = E - frexp exponent of x) and its lowest stored mantissa bit at
 * position z + L, where L = 53 for a normal number and the number of stored
 * significant bits for a subnormal one. s slices keep positions 1 .. 7 s, so
 *     lost(x, s) = number of the L mantissa positions beyond 7 s
 *                = min(L, max(0, z + L - 7 s)),
 * counted by position, whatever the value of the bits there. Zeros lose nothing but
 * count in the average. The average is taken per input matrix (per real plane of a
 * complex one) over all its elements, and every matrix must meet the threshold.
 * ------------------------------------------------------------------------------- */

/* loss_sums[s - 1] = sum over the elements of M of lost(x, s), s = 1 .. s_max, for the
 * rows of M (by_columns = 0: rows x cols with leading dimension ld and element stride
 * inc) or its columns (by_columns = 1: the exponent is per column). */
void oz_auto_loss_sums(int64_t rows, int64_t cols, const double *M, int64_t ld, int64_t inc,
                       int by_columns, int s_max, uint64_t *loss_sums) {
    for (int s = 1; s <= s_max; ++s) loss_sums[s - 1] = 0;
    int64_t outer = by_columns ? cols : rows, inner = by_columns ? rows : cols;
    for (int64_t o = 0; o < outer; ++o) {
        const double *vec = by_columns ? M + o * inc : M + o * ld * 1;
        int64_t stride = by_columns ? ld : inc;
        int E = row_exponent(vec, inner, stride);
        for (int64_t l = 0; l < inner; ++l) {
            double x = vec[l * stride];
            if (x == 0.0) continue;
            int ex;
            (void)frexp(fabs(x), &ex);
            int z = E - ex;
            int L = ex + 1074 < 53 ? ex + 1074 : 53; /* subnormals store fewer bits */
            for (int s = 1; s <= s_max; ++s) {
                int beyond = z + L - OZ_W * s;
                if (beyond < 0) beyond = 0;
                if (beyond > L) beyond = L;
                loss_sums[s - 1] += (uint64_t)beyond;
            }
        }
    }
}

/* The smallest s in 1 .. s_max for which every plane's average loss is <= T; s_max if
 * none is. sums is [planes][s_max], counts[planes] the number of elements of each
 * plane. The comparison is sum <= T * count in double precision. */
int oz_auto_num_slices(int planes, int s_max, const uint64_t *sums, const int64_t *counts, double T) {
    for (int s = 1; s <= s_max; ++s) {
        int ok = 1;
        for (int p = 0; p < planes; ++p)
            if (!((double)sums[(int64_t)p * s_max + (s - 1)] <= T * (double)counts[p])) ok = 0;
        if (ok) return s;
    }
    return s_max;
}

/* ---------------------------------------------------------------------------------
 * BLAS-style call (Section 4.4: the method stands in for the vendor DGEMM routine):
 * column-major storage, C <- alpha op(A) op(B) + beta C with op(X) = X or X^T.
 *
 * op(A) (m x k) and op(B) (k x n) are first written out as plain row-major matrices,
 * G = their Ozaki product as above (exponents per row of op(A) and per column of
 * op(B)), and then, element by element,
 *     C = RN(alpha G)                        if beta == 0 (C is not read),
 *     C = RN( RN(alpha G) + RN(beta C) )     otherwise;
 * if alpha == 0 or k == 0 the product is not formed: C = +0 if beta == 0, else RN(beta C).
 * (The paper does not discuss alpha and beta; this is the reference BLAS order of operations.)
 * ------------------------------------------------------------------------------- */
int oz_dgemm_blas(int transa, int transb, int64_t m, int64_t n, int64_t k, double alpha,
                  const double *A, int64_t lda, const double *B, int64_t ldb, double beta, double *C,
                  int64_t ldc, int s) {
    if (m == 0 || n == 0) return 0;
    if (alpha == 0.0 || k == 0) {
        for (int64_t j = 0; j < n; ++j)
            for (int64_t i = 0; i < m; ++i) C[i + j * ldc] = beta == 0.0 ? 0.0 : beta * C[i + j * ldc];
        return 0;
    }
    double *opA = (double *)malloc(sizeof(double) * (size_t)(m * k));
    double *opB = (double *)malloc(sizeof(double) * (size_t)(k * n));
    double *G = (double *)malloc(sizeof(double) * (size_t)(m * n));
    if (!opA || !opB || !G) { free(opA); free(opB); free(G); return 1; }
    for (int64_t i = 0; i < m; ++i)
        for (int64_t l = 0; l < k; ++l) opA[i * k + l] = transa ? A[l + i * lda] : A[i + l * lda];
    for (int64_t l = 0; l < k; ++l)
        for (int64_t j = 0; j < n; ++j) opB[l * n + j] = transb ? B[j + l * ldb] : B[l + j * ldb];
    int rc = oz_dgemm(m, n, k, opA, k, opB, n, G, n, s);
    if (rc == 0) {
        for (int64_t j = 0; j < n; ++j)
            for (int64_t i = 0; i < m; ++i) {
                double v = alpha * G[i * n + j];
                if (beta != 0.0) v = v + beta * C[i + j * ldc];
                C[i + j * ldc] = v;
            }
    }
    free(opA); free(opB); free(G);
    return rc;
}

/* ---------------------------------------------------------------------------------
 * BLAS-style complex call (Section 4.4: complex GEMM by separated real and imaginary
 * parts, standing in for the vendor ZGEMM routine): column-major storage of
 * interleaved (re, im) doubles, leading dimensions in complex elements,
 * C <- alpha op(A) op(B) + beta C with op(X) = X (0), X^T (1) or X^H (2).
 *
 * op(A) (m x k) and op(B) (k x n) are written out as plain row-major complex matrices,
 * a conjugation negating the imaginary part (exact). G = their complex Ozaki product as
 * in oz_zgemm (four real products, one rounded combination per part). Then per element,
 * with alpha = (ar, ai), beta = (br, bi), every operation a rounded FP64 one:
 *     t = ( RN(RN(ar Gr) - RN(ai Gi)),  RN(RN(ar Gi) + RN(ai Gr)) )
 *     C = t                                                   if beta == 0 (C is not read),
 *     u = ( RN(RN(br Cr) - RN(bi Ci)),  RN(RN(br Ci) + RN(bi Cr)) )
 *     C = ( RN(tr + ur), RN(ti + ui) )                        otherwise;
 * if alpha == 0 or k == 0 the product is not formed: C = +0 if beta == 0, else u.
 * (The paper does not discuss alpha, beta or transposes; the order above is the plain
 * textbook complex multiply-add.)
 * ------------------------------------------------------------------------------- */
int oz_zgemm_blas(int transa, int transb, int64_t m, int64_t n, int64_t k, const double *alpha,
                  const double *A, int64_t lda, const double *B, int64_t ldb, const double *beta,
                  double *C, int64_t ldc, int s) {
    if (m == 0 || n == 0) return 0;
    const double ar = alpha[0], ai = alpha[1], br = beta[0], bi = beta[1];
    const int beta_zero = br == 0.0 && bi == 0.0;
    const int no_product = (ar == 0.0 && ai == 0.0) || k == 0;
    double *opA = NULL, *opB = NULL, *G = NULL;
    int rc = 0;
    if (!no_product) {
        opA = (double *)malloc(sizeof(double) * 2 * (size_t)(m * k));
        opB = (double *)malloc(sizeof(double) * 2 * (size_t)(k * n));
        G = (double *)malloc(sizeof(double) * 2 * (size_t)(m * n));
        if (!opA || !opB || !G) { free(opA); free(opB); free(G); return 1; }
        for (int64_t i = 0; i < m; ++i)
            for (int64_t l = 0; l < k; ++l) {
                const double *src = A + 2 * (transa ? l + i * lda : i + l * lda);
                opA[2 * (i * k + l)] = src[0];
                opA[2 * (i * k + l) + 1] = transa == 2 ? -src[1] : src[1];
            }
        for (int64_t l = 0; l < k; ++l)
            for (int64_t j = 0; j < n; ++j) {
                const double *src = B + 2 * (transb ? j + l * ldb : l + j * ldb);
                opB[2 * (l * n + j)] = src[0];
                opB[2 * (l * n + j) + 1] = transb == 2 ? -src[1] : src[1];
            }
        rc = oz_zgemm(m, n, k, opA, k, opB, n, G, n, s);
    }
    if (rc == 0) {
        for (int64_t j = 0; j < n; ++j)
            for (int64_t i = 0; i < m; ++i) {
                double *c = C + 2 * (i + j * ldc);
                double tr = 0.0, ti = 0.0;
                if (!no_product) {
                    const double gr = G[2 * (i * n + j)], gi = G[2 * (i * n + j) + 1];
                    const double x0 = ar * gr, x1 = ai * gi, y0 = ar * gi, y1 = ai * gr;
                    tr = x0 - x1;
                    ti = y0 + y1;
                }
                if (beta_zero) {
                    c[0] = tr;
                    c[1] = ti;
                } else {
                    const double x0 = br * c[0], x1 = bi * c[1], y0 = br * c[1], y1 = bi * c[0];
                    const double ur = x0 - x1, ui = y0 + y1;
                    c[0] = no_product ? ur : tr + ur;
                    c[1] = no_product ? ui : ti + ui;
                }
            }
    }
    free(opA); free(opB); free(G);
    return rc;
}

/* ---------------------------------------------------------------------------------
 * Summing-up in higher precision (Section 2.3.4, first advantage: the precision of the
 * scheme can be raised above FP64 by more slices and a more accurate summing-up of the
 * products). Here the per-diagonal integer sums are added in double-double arithmetic
 * and the result is returned as an unevaluated pair (hi, lo), C = hi + lo.
 *
 * Steps per element, least significant diagonal first (t = S_d 2^(-7 d) is exact):
 *     (h, l) = (0, 0)
 *     for d = s+1 down to 2:
 *         sh = RN(h + t);  bb = RN(sh - h)                    -- TwoSum of h and t:
 *         e  = RN( RN(h - RN(sh - bb)) + RN(t - bb) )         -- h + t = sh + e exactly
 *         l2 = RN(l + e)
 *         h  = RN(sh + l2);  l = RN(l2 - RN(h - sh))          -- FastTwoSum renormalisation
 *     hi = ldexp(h, EA_i + EB_j),  lo = ldexp(l, EA_i + EB_j)
 * ------------------------------------------------------------------------------- */
void oz_accumulate_dd(int64_t m, int64_t n, int s, const int64_t *S, const int32_t *EA,
                      const int32_t *EB, double *Chi, double *Clo, int64_t ldc) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double h = 0.0, l = 0.0;
            for (int d = s + 1; d >= 2; --d) {
                double t = ldexp((double)S[((int64_t)(d - 2) * m + i) * n + j], -OZ_W * d);
                double sh = h + t;
                double bb = sh - h;
                double e = (h - (sh - bb)) + (t - bb);
                double l2 = l + e;
                double hn = sh + l2;
                l = l2 - (hn - sh);
                h = hn;
            }
            Chi[i * ldc + j] = ldexp(h, EA[i] + EB[j]);
            Clo[i * ldc + j] = ldexp(l, EA[i] + EB[j]);
        }
}

/* The whole method with the double-double summing-up. */
int oz_dgemm_dd(int64_t m, int64_t n, int64_t k, const double *A, int64_t lda, const double *B,
                int64_t ldb, double *Chi, double *Clo, int64_t ldc, int s) {
    if (m == 0 || n == 0) return 0;
    int32_t *EA = malloc(sizeof(int32_t) * (size_t)m);
    int32_t *EB = malloc(sizeof(int32_t) * (size_t)n);
    int8_t *SA = malloc((size_t)s * (size_t)m * (size_t)(k ? k : 1));
    int8_t *SB = malloc((size_t)s * (size_t)n * (size_t)(k ? k : 1));
    int64_t *S = malloc(sizeof(int64_t) * (size_t)s * (size_t)m * (size_t)n);
    int rc = 1;
    if (EA && EB && SA && SB && S) {
        oz_split_rows(m, k, A, lda, s, EA, SA);
        oz_split_cols(k, n, B, ldb, s, EB, SB);
        oz_diagonal_sums(m, n, k, s, SA, SB, S);
        oz_accumulate_dd(m, n, s, S, EA, EB, Chi, Clo, ldc);
        rc = 0;
    }
    free(EA); free(EB); free(SA); free(SB); free(S);
    return rc;
}
