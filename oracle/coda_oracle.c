/*
 * coda_oracle.c -- CPU oracle for the GEMM-plus-epilogue hot path.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the
 * GPU library is checked against.  Only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg may call it; the product path never does.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * Arithmetic: every bf16 / fp32 input is widened exactly to double, every sum
 * is a plain left-to-right sum over the contraction index in double, and no
 * intermediate is ever rounded to a narrower type.  There is no tiling and no
 * fusion: each function below is the operator chain of the cited definition
 * written out as loops.  The only deviations from the textbook "for i, for j,
 * for k" nest are (1) the operands are first copied into dense row-major
 * double arrays (an exact widening that also resolves the transpose flags) and
 * (2) the nest runs in i, k, j order so that the innermost loop is contiguous;
 * each output element still receives its K products in ascending k.
 *
 * Row selection: every function takes `rows` (int64 indices into 0..M-1) and
 * `nrows`.  rows == NULL means "all M rows in order" (nrows is then ignored).
 * Outputs are dense [nrows x width] row-major doubles in the order of `rows`.
 * Every epilogue on the path is row-local, so a row subset is exact; this is
 * how full-size workloads are checked on a sample.
 *
 * Pins (see tests/test_oracle_pins.py): contraction vs a brute-force Python
 * triple loop and vs an independent fp64 library matmul; rstd vs closed form and
 * vs a library RMSNorm; the reparameterised forms vs the canonical operator
 * chain (Section 3.2.1 identity); SwiGLU backward vs its closed-form derivative,
 * central finite differences and reverse-mode autodiff of the forward
 * definition; the row statistic vs sum(Z * dZ); the weight gradient vs finite
 * differences of <dY, H W>; RoPE vs complex multiplication by a library, norm preservation, the
 * relative-position property; the RMSNorm-backward kernel vs reverse-mode autodiff of a library RMSNorm;
 * the log-sum-exp kernel vs a library logsumexp / cross-entropy, shift invariance and the uniform case; the 8-bit
 * operand decoder vs the values the OFP8 specification names and vs a library's conversion of all 256 codes.
 * No function here is "parity unpinned".
 *
 * Naming: "row scale" multiplies row i by r[i]; "column scale" multiplies
 * column j by gamma[j]; a "row reduction" sums over columns and yields one
 * value per row.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG 1
#define ORACLE_ERR_NOMEM 2

/* ---- exact widenings ---------------------------------------------------- */

/* bf16 is the upper 16 bits of an IEEE binary32. */
static double bf16_widen(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int64_t sel_row(const int64_t *rows, int64_t r)
{
    return rows ? rows[r] : r;
}

static int64_t sel_count(const int64_t *rows, int64_t nrows, int64_t M)
{
    return rows ? nrows : M;
}

/*
 * Dense double copy of the selected rows of op(X), shape [R x cols].
 * trans == 0: X is stored [rows x cols] row-major with leading dimension ld,
 *             op(X)[i][j] = X[i*ld + j].
 * trans != 0: X is stored [cols x rows] row-major with leading dimension ld,
 *             op(X)[i][j] = X[j*ld + i].
 */
static double *widen_rows(const uint16_t *X, int64_t ld, int trans, int64_t cols,
                          const int64_t *rows, int64_t R)
{
    double *out = (double *)malloc(sizeof(double) * (size_t)(R > 0 ? R : 1) *
                                   (size_t)(cols > 0 ? cols : 1));
    if (!out)
        return NULL;
    for (int64_t r = 0; r < R; ++r) {
        int64_t i = sel_row(rows, r);
        for (int64_t j = 0; j < cols; ++j)
            out[r * cols + j] = trans ? bf16_widen(X[j * ld + i]) : bf16_widen(X[i * ld + j]);
    }
    return out;
}

/* ---- the contraction ----------------------------------------------------- */

/*
 * D[r][j] = sum_{k=0}^{K-1} A[r][k] * B[k][j]        (GEMM: h = x W)
 * A dense [R x K], B dense [K x N], D dense [R x N]; all double.
 */
static void contract(const double *A, const double *B, int64_t R, int64_t N, int64_t K, double *D)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < R; ++r) {
        double *d = D + r * N;
        for (int64_t j = 0; j < N; ++j)
            d[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = A[r * K + k];
            const double *b = B + k * N;
            for (int64_t j = 0; j < N; ++j)
                d[j] += a * b[j];
        }
    }
}

/* D = op(A)[rows] * op(B) for bf16 operands; returns malloc'd [R x N] or NULL. */
static double *gemm_bf16(const uint16_t *A, int64_t lda, int transA, const uint16_t *B, int64_t ldb,
                         int transB, int64_t N, int64_t K, const int64_t *rows, int64_t R)
{
    double *Ad = widen_rows(A, lda, transA, K, rows, R);
    double *Bd = widen_rows(B, ldb, transB, N, NULL, K);
    double *D = (double *)malloc(sizeof(double) * (size_t)(R > 0 ? R : 1) * (size_t)(N > 0 ? N : 1));
    if (Ad && Bd && D)
        contract(Ad, Bd, R, N, K, D);
    else {
        free(D);
        D = NULL;
    }
    free(Ad);
    free(Bd);
    return D;
}

/* ---- scalar definitions --------------------------------------------------- */

static double sigmoid(double g)
{
    return 1.0 / (1.0 + exp(-g));
}

/* silu(g) = g * sigma(g) */
static double silu(double g)
{
    return g * sigmoid(g);
}

/*
 * Kernel 10's pairwise backward rule for one (gate, up) pair and one incoming
 * gradient d:   dU = d silu(g),   dG = d u ( sigma(g) + silu(g) (1 - sigma(g)) ).
 */
static void swiglu_bwd_pair(double d, double g, double u, double *dG, double *dU)
{
    double sg = sigmoid(g);
    double sl = silu(g);
    *dU = d * sl;
    *dG = d * u * (sg + sl * (1.0 - sg));
}

/* Pointwise entry points so the scalar rules can be pinned on arbitrary doubles. */
int coda_oracle_swiglu_fwd_points(const double *g, const double *u, int64_t n, double *o)
{
    if (!g || !u || !o)
        return ORACLE_ERR_ARG;
    for (int64_t t = 0; t < n; ++t)
        o[t] = silu(g[t]) * u[t];
    return ORACLE_OK;
}

int coda_oracle_swiglu_bwd_points(const double *d, const double *g, const double *u, int64_t n,
                                  double *dG, double *dU)
{
    if (!d || !g || !u || !dG || !dU)
        return ORACLE_ERR_ARG;
    for (int64_t t = 0; t < n; ++t)
        swiglu_bwd_pair(d[t], g[t], u[t], &dG[t], &dU[t]);
    return ORACLE_OK;
}

/* ---- row statistics -------------------------------------------------------- */

/* ss[r] = sum_k X[i][k]^2 for a bf16 matrix X [M x d]. */
int coda_oracle_row_sumsq(const uint16_t *X, int64_t M, int64_t d, int64_t ld, const int64_t *rows,
                          int64_t nrows, double *ss)
{
    if (!X || !ss || M < 0 || d < 0)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    for (int64_t r = 0; r < R; ++r) {
        int64_t i = sel_row(rows, r);
        double s = 0.0;
        for (int64_t k = 0; k < d; ++k) {
            double x = bf16_widen(X[i * ld + k]);
            s += x * x;
        }
        ss[r] = s;
    }
    return ORACLE_OK;
}

/*
 * r[i] = 1 / sqrt( (1/d) * sum_k X[i][k]^2 + eps )
 * Section 3.2.1: r = 1/rms(.), r = 1/sqrt(reduce(partials) + eps), with the
 * standard RMSNorm reading: mean of squares over the full hidden size d.
 */
int coda_oracle_rstd(const uint16_t *X, int64_t M, int64_t d, int64_t ld, double eps,
                     const int64_t *rows, int64_t nrows, double *r)
{
    int rc = coda_oracle_row_sumsq(X, M, d, ld, rows, nrows, r);
    if (rc)
        return rc;
    int64_t R = sel_count(rows, nrows, M);
    for (int64_t q = 0; q < R; ++q)
        r[q] = 1.0 / sqrt(r[q] / (double)d + eps);
    return ORACLE_OK;
}

/* r[i] = 1/sqrt(ss[i]/d + eps): the auxiliary reduction's last step on given sums. */
int coda_oracle_rstd_from_sumsq(const double *ss, int64_t M, int64_t d, double eps, double *r)
{
    if (!ss || !r || d <= 0)
        return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < M; ++i)
        r[i] = 1.0 / sqrt(ss[i] / (double)d + eps);
    return ORACLE_OK;
}

/* ---- GEMM + epilogue definitions (Appendix "List of Kernels") ---------------- */

/*
 * Kernel 5 (and the plain GEMM when r == NULL):
 *   D = A B,  O[i][j] = D[i][j] * r[i].
 * r is indexed by the ORIGINAL row index (length M).
 */
int coda_oracle_gemm_rowscale(const uint16_t *A, int64_t lda, int transA, const uint16_t *B,
                              int64_t ldb, int transB, int64_t M, int64_t N, int64_t K,
                              const double *r, const int64_t *rows, int64_t nrows, double *O)
{
    if (!A || !B || !O)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *D = gemm_bf16(A, lda, transA, B, ldb, transB, N, K, rows, R);
    if (!D)
        return ORACLE_ERR_NOMEM;
    for (int64_t q = 0; q < R; ++q) {
        double ri = r ? r[sel_row(rows, q)] : 1.0;
        for (int64_t j = 0; j < N; ++j)
            O[q * N + j] = D[q * N + j] * ri;
    }
    free(D);
    return ORACLE_OK;
}

/*
 * Kernel 6 (Kernel 2 when r == NULL):
 *   D = A B,  D' = D (.) r,  [G, U] = interleavedSplit(D'),  O = silu(G) (.) U
 * Even column 2j is the gate, odd column 2j+1 the up value.  N must be even.
 * O is [R x N/2]; Dp (optional) receives D' [R x N], the pre-activation that a
 * training run saves for Kernel 10.
 */
int coda_oracle_gemm_rowscale_swiglu(const uint16_t *A, int64_t lda, int transA, const uint16_t *B,
                                     int64_t ldb, int transB, int64_t M, int64_t N, int64_t K,
                                     const double *r, const int64_t *rows, int64_t nrows, double *O,
                                     double *Dp)
{
    if (!A || !B || !O || (N & 1))
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *D = gemm_bf16(A, lda, transA, B, ldb, transB, N, K, rows, R);
    if (!D)
        return ORACLE_ERR_NOMEM;
    for (int64_t q = 0; q < R; ++q) {
        double ri = r ? r[sel_row(rows, q)] : 1.0;
        for (int64_t j = 0; j < N; ++j)
            D[q * N + j] *= ri;
        for (int64_t p = 0; p < N / 2; ++p) {
            double g = D[q * N + 2 * p];
            double u = D[q * N + 2 * p + 1];
            O[q * (N / 2) + p] = silu(g) * u;
        }
        if (Dp)
            memcpy(Dp + q * N, D + q * N, sizeof(double) * (size_t)N);
    }
    free(D);
    return ORACLE_OK;
}

/*
 * Kernels 1 and 7: D = A B,  D' = D (.) r (r == NULL: Kernel 1),  O = RoPE(D').
 * RoPE acts on ADJACENT feature pairs of the output (columns 2p, 2p+1).  Row i has position q = pos[i]; the
 * output is split into heads of head_dim columns and pair p uses frequency index f = p mod (head_dim/2):
 *     O[i][2p]   = x0 * cos[q][f] - x1 * sin[q][f]
 *     O[i][2p+1] = x0 * sin[q][f] + x1 * cos[q][f]          with (x0, x1) = (D'[i][2p], D'[i][2p+1]).
 * Only the first rope_cols columns are rotated (query and key parts of a fused QKV projection); the remaining
 * columns pass through unchanged.  cos / sin are precomputed fp32 tables [T x head_dim/2] given by the caller,
 * so the oracle takes no position on how angles are generated.
 */
int coda_oracle_gemm_rowscale_rope(const uint16_t *A, int64_t lda, int transA, const uint16_t *B,
                                   int64_t ldb, int transB, int64_t M, int64_t N, int64_t K,
                                   const double *r, const float *cos_t, const float *sin_t, int64_t T,
                                   const int32_t *pos, int64_t head_dim, int64_t rope_cols,
                                   const int64_t *rows, int64_t nrows, double *O)
{
    if (!A || !B || !O || !cos_t || !sin_t || !pos || head_dim <= 0 || (head_dim & 1) || (rope_cols & 1) ||
        rope_cols < 0 || rope_cols > N)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    int64_t half = head_dim / 2;
    double *D = gemm_bf16(A, lda, transA, B, ldb, transB, N, K, rows, R);
    if (!D)
        return ORACLE_ERR_NOMEM;
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        double ri = r ? r[i] : 1.0;
        int64_t t = pos[i];
        if (t < 0 || t >= T) {
            free(D);
            return ORACLE_ERR_ARG;
        }
        for (int64_t j = 0; j < N; ++j)
            D[q * N + j] *= ri;
        for (int64_t j = 0; j < N; ++j)
            O[q * N + j] = D[q * N + j];
        for (int64_t p2 = 0; p2 < rope_cols / 2; ++p2) {
            int64_t f = p2 % half;
            double c = (double)cos_t[t * half + f], sn = (double)sin_t[t * half + f];
            double x0 = D[q * N + 2 * p2], x1 = D[q * N + 2 * p2 + 1];
            O[q * N + 2 * p2] = x0 * c - x1 * sn;
            O[q * N + 2 * p2 + 1] = x0 * sn + x1 * c;
        }
    }
    free(D);
    return ORACLE_OK;
}

/*
 * Kernels 3 and 8 (cross-entropy as GEMM + row-wise log-sum-exp):
 *     Z = (A B) (.) r   (r == NULL: Kernel 3),   z_tgt[i] = Z[i][y[i]],   lse[i] = log sum_k exp(Z[i][k]).
 * The per-token loss of Section 3.2.3 is lse[i] - z_tgt[i].  The log-sum-exp is evaluated in its shift-invariant
 * form  m + log sum_k exp(Z[i][k] - m),  m = max_k Z[i][k],  which is the same number without overflow.
 * Zout (optional) receives the logits, which the method materialises for the backward pass.
 */
int coda_oracle_gemm_rowscale_lse(const uint16_t *A, int64_t lda, int transA, const uint16_t *B, int64_t ldb,
                                  int transB, int64_t M, int64_t N, int64_t K, const double *r,
                                  const int32_t *y, const int64_t *rows, int64_t nrows, double *Zout,
                                  double *ztgt, double *lse)
{
    if (!A || !B || !y || !ztgt || !lse || N <= 0)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *D = gemm_bf16(A, lda, transA, B, ldb, transB, N, K, rows, R);
    if (!D)
        return ORACLE_ERR_NOMEM;
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        double ri = r ? r[i] : 1.0;
        if (y[i] < 0 || y[i] >= N) {
            free(D);
            return ORACLE_ERR_ARG;
        }
        double m = -INFINITY;
        for (int64_t j = 0; j < N; ++j) {
            D[q * N + j] *= ri;
            if (D[q * N + j] > m)
                m = D[q * N + j];
        }
        double sum = 0.0;
        for (int64_t j = 0; j < N; ++j)
            sum += exp(D[q * N + j] - m);
        lse[q] = m + log(sum);
        ztgt[q] = D[q * N + y[i]];
        if (Zout)
            memcpy(Zout + q * N, D + q * N, sizeof(double) * (size_t)N);
    }
    free(D);
    return ORACLE_OK;
}

/*
 * Kernel 4, with an optional row scale in front (the tiny configuration's
 * program: row scale, residual add, sum of squares, store):
 *   D = (A B) (.) r + C,   ss[i] = sum_j D[i][j]^2,   O = D (.) gamma
 * r, C, gamma, O may each be NULL (identity / zero / not produced).  The sum of
 * squares is taken on the unrounded D, before the gamma scale.
 */
int coda_oracle_gemm_residual_sumsq(const uint16_t *A, int64_t lda, int transA, const uint16_t *B,
                                    int64_t ldb, int transB, int64_t M, int64_t N, int64_t K,
                                    const double *r, const uint16_t *C, int64_t ldc,
                                    const double *gamma, const int64_t *rows, int64_t nrows,
                                    double *Dout, double *ss, double *O)
{
    if (!A || !B || !Dout)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *D = gemm_bf16(A, lda, transA, B, ldb, transB, N, K, rows, R);
    if (!D)
        return ORACLE_ERR_NOMEM;
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        double ri = r ? r[i] : 1.0;
        double s = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            double v = D[q * N + j] * ri;
            if (C)
                v += bf16_widen(C[i * ldc + j]);
            s += v * v;
            Dout[q * N + j] = v;
            if (O)
                O[q * N + j] = gamma ? v * gamma[j] : v;
        }
        if (ss)
            ss[q] = s;
    }
    free(D);
    return ORACLE_OK;
}

/*
 * Kernel 10.  D = op(A) op(B) has N columns; the saved pre-activation Z is
 * [M x 2N] bf16 with (gate, up) interleaved.
 *   G = Z[:, 2j], U = Z[:, 2j+1]
 *   O      = silu(G) (.) U                                  [R x N]   (optional)
 *   dU     = D (.) silu(G)
 *   dG     = D (.) U (.) ( sigma(G) + silu(G) (.) (1 - sigma(G)) )
 *   dZ     = interleavedConcat(dG, dU)                       [R x 2N]
 *   stat_i = sum_j ( G dG + U dU )                           [R]       (optional)
 */
int coda_oracle_gemm_swiglu_bwd(const uint16_t *A, int64_t lda, int transA, const uint16_t *B,
                                int64_t ldb, int transB, int64_t M, int64_t N, int64_t K,
                                const uint16_t *Z, int64_t ldz, const int64_t *rows, int64_t nrows,
                                double *dZ, double *O, double *stat)
{
    if (!A || !B || !Z || !dZ)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *D = gemm_bf16(A, lda, transA, B, ldb, transB, N, K, rows, R);
    if (!D)
        return ORACLE_ERR_NOMEM;
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        double s = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            double d = D[q * N + j];
            double g = bf16_widen(Z[i * ldz + 2 * j]);
            double u = bf16_widen(Z[i * ldz + 2 * j + 1]);
            double dG, dU;
            swiglu_bwd_pair(d, g, u, &dG, &dU);
            dZ[q * 2 * N + 2 * j] = dG;
            dZ[q * 2 * N + 2 * j + 1] = dU;
            if (O)
                O[q * N + j] = silu(g) * u;
            s += g * dG + u * dU;
        }
        if (stat)
            stat[q] = s;
    }
    free(D);
    return ORACLE_OK;
}

/*
 * Kernel 9 (local part of RMSNorm backward).  D = op(A) op(B) is the gradient w.r.t. the normalised activation;
 * C [M x N] bf16 is the RMSNorm input, r [M] its inverse-RMS factor, gamma [N] the RMSNorm weight and z [M] the
 * row statistic z_i = (1/d) sum_j (grad_h2 * h2)[i][j] delivered by the following pattern's epilogue:
 *     C_norm = C (.) r
 *     O_out  = O_in + ( D (.) gamma - C_norm (.) z ) (.) r          (O_in optional, bf16 [M x N])
 *     C_out  = C_norm (.) gamma                                      (optional: the recomputed normalised activation)
 *     dgamma[j] = sum over the SELECTED rows i of D[i][j] * C_norm[i][j]
 * (with rows == NULL this is the full reduceTile_rows + reduce_rows of the paper; a row subset gives the partial
 * sum over that subset, which is what one tile row contributes).
 */
int coda_oracle_gemm_rmsnorm_bwd(const uint16_t *A, int64_t lda, int transA, const uint16_t *B, int64_t ldb,
                                 int transB, int64_t M, int64_t N, int64_t K, const uint16_t *C, int64_t ldc,
                                 const double *r, const double *z, const double *gamma, const uint16_t *Oin,
                                 int64_t ldo, const int64_t *rows, int64_t nrows, double *Oout, double *Cout,
                                 double *dgamma)
{
    if (!A || !B || !C || !r || !z || !gamma || !Oout)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *D = gemm_bf16(A, lda, transA, B, ldb, transB, N, K, rows, R);
    if (!D)
        return ORACLE_ERR_NOMEM;
    if (dgamma)
        for (int64_t j = 0; j < N; ++j)
            dgamma[j] = 0.0;
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        for (int64_t j = 0; j < N; ++j) {
            double d = D[q * N + j];
            double cn = bf16_widen(C[i * ldc + j]) * r[i];
            double o = (d * gamma[j] - cn * z[i]) * r[i];
            if (Oin)
                o += bf16_widen(Oin[i * ldo + j]);
            Oout[q * N + j] = o;
            if (Cout)
                Cout[q * N + j] = cn * gamma[j];
            if (dgamma)
                dgamma[j] += d * cn;
        }
    }
    free(D);
    return ORACLE_OK;
}

/*
 * Weight gradient of Theorem 1 with accumulation into an existing fp32 buffer:
 *   G_out = G_in + op(A) op(B)       (for dW: op(A) = x^T, op(B) = grad_h)
 * G_in is fp32 [M x N] (ldg); G_out is returned in double.
 */
int coda_oracle_gemm_accumulate(const uint16_t *A, int64_t lda, int transA, const uint16_t *B,
                                int64_t ldb, int transB, int64_t M, int64_t N, int64_t K,
                                const float *Gin, int64_t ldg, const int64_t *rows, int64_t nrows,
                                double *Gout)
{
    if (!A || !B || !Gout)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *D = gemm_bf16(A, lda, transA, B, ldb, transB, N, K, rows, R);
    if (!D)
        return ORACLE_ERR_NOMEM;
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        for (int64_t j = 0; j < N; ++j)
            Gout[q * N + j] = (Gin ? (double)Gin[i * ldg + j] : 0.0) + D[q * N + j];
    }
    free(D);
    return ORACLE_OK;
}

/* ---- canonical (unfused) operator chains and their reparameterised forms ----- */

/*
 * Canonical form of Section 3.2.1:  Y = RMSNorm(X, gamma) W + R
 *   r[i]    = 1/sqrt(mean_k X[i][k]^2 + eps)
 *   Xn[i][k] = X[i][k] * r[i] * gamma[k]          (normalise BEFORE the GEMM)
 *   Y       = Xn W + R,   ss[i] = sum_j Y[i][j]^2
 * X [M x d] bf16, W = op(W) [d x N], R [M x N] bf16 or NULL.
 */
int coda_oracle_rmsnorm_linear_unfused(const uint16_t *X, int64_t ldx, const double *gamma,
                                       double eps, const uint16_t *W, int64_t ldw, int transW,
                                       const uint16_t *Rm, int64_t ldr, int64_t M, int64_t N,
                                       int64_t d, const int64_t *rows, int64_t nrows, double *Y,
                                       double *ss)
{
    if (!X || !gamma || !W || !Y)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *r = (double *)malloc(sizeof(double) * (size_t)(R > 0 ? R : 1));
    double *Xn = widen_rows(X, ldx, 0, d, rows, R);
    double *Wd = widen_rows(W, ldw, transW, N, NULL, d);
    if (!r || !Xn || !Wd) {
        free(r); free(Xn); free(Wd);
        return ORACLE_ERR_NOMEM;
    }
    coda_oracle_rstd(X, M, d, ldx, eps, rows, nrows, r);
    for (int64_t q = 0; q < R; ++q)
        for (int64_t k = 0; k < d; ++k)
            Xn[q * d + k] = Xn[q * d + k] * r[q] * gamma[k];
    contract(Xn, Wd, R, N, d, Y);
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        double s = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            if (Rm)
                Y[q * N + j] += bf16_widen(Rm[i * ldr + j]);
            s += Y[q * N + j] * Y[q * N + j];
        }
        if (ss)
            ss[q] = s;
    }
    free(r); free(Xn); free(Wd);
    return ORACLE_OK;
}

/*
 * Reparameterised form: the row factor commutes with the GEMM and gamma folds
 * into the weight,   Y = diag(r) ( X (diag(gamma) W) ) + R ,
 * with W'[k][j] = gamma[k] * W[k][j] formed exactly in double (no rounding).
 */
int coda_oracle_rmsnorm_linear_reparam(const uint16_t *X, int64_t ldx, const double *gamma,
                                       double eps, const uint16_t *W, int64_t ldw, int transW,
                                       const uint16_t *Rm, int64_t ldr, int64_t M, int64_t N,
                                       int64_t d, const int64_t *rows, int64_t nrows, double *Y,
                                       double *ss)
{
    if (!X || !gamma || !W || !Y)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    double *r = (double *)malloc(sizeof(double) * (size_t)(R > 0 ? R : 1));
    double *Xd = widen_rows(X, ldx, 0, d, rows, R);
    double *Wp = widen_rows(W, ldw, transW, N, NULL, d);
    if (!r || !Xd || !Wp) {
        free(r); free(Xd); free(Wp);
        return ORACLE_ERR_NOMEM;
    }
    coda_oracle_rstd(X, M, d, ldx, eps, rows, nrows, r);
    for (int64_t k = 0; k < d; ++k)
        for (int64_t j = 0; j < N; ++j)
            Wp[k * N + j] *= gamma[k];
    contract(Xd, Wp, R, N, d, Y);
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        double s = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            double v = r[q] * Y[q * N + j];
            if (Rm)
                v += bf16_widen(Rm[i * ldr + j]);
            Y[q * N + j] = v;
            s += v * v;
        }
        if (ss)
            ss[q] = s;
    }
    free(r); free(Xd); free(Wp);
    return ORACLE_OK;
}

/*
 * One MLP sub-layer, canonical operator chain, no intermediate rounding:
 *   Xn = RMSNorm(X, gamma);  Z = Xn W1  ([M x 2F], gate/up interleaved);
 *   H  = silu(Z[:,2j]) * Z[:,2j+1];   Y = H W2 + R;   ss = sum_j Y^2.
 * reparam != 0 evaluates the reparameterised order instead:
 *   Z = diag(r) (X (diag(gamma) W1)), the rest identical.
 * X [M x d], W1 [d x 2F], W2 [F x d2], R [M x d2] (NULL allowed).
 */
int coda_oracle_mlp_block(const uint16_t *X, int64_t ldx, const double *gamma, double eps,
                          const uint16_t *W1, int64_t ldw1, const uint16_t *W2, int64_t ldw2,
                          const uint16_t *Rm, int64_t ldr, int64_t M, int64_t d, int64_t F,
                          int64_t d2, int reparam, const int64_t *rows, int64_t nrows, double *Y,
                          double *ss)
{
    if (!X || !gamma || !W1 || !W2 || !Y)
        return ORACLE_ERR_ARG;
    int64_t R = sel_count(rows, nrows, M);
    size_t Rz = (size_t)(R > 0 ? R : 1);
    double *r = (double *)malloc(sizeof(double) * Rz);
    double *Xd = widen_rows(X, ldx, 0, d, rows, R);
    double *W1d = widen_rows(W1, ldw1, 0, 2 * F, NULL, d);
    double *W2d = widen_rows(W2, ldw2, 0, d2, NULL, F);
    double *Zm = (double *)malloc(sizeof(double) * Rz * (size_t)(2 * F > 0 ? 2 * F : 1));
    double *H = (double *)malloc(sizeof(double) * Rz * (size_t)(F > 0 ? F : 1));
    if (!r || !Xd || !W1d || !W2d || !Zm || !H) {
        free(r); free(Xd); free(W1d); free(W2d); free(Zm); free(H);
        return ORACLE_ERR_NOMEM;
    }
    coda_oracle_rstd(X, M, d, ldx, eps, rows, nrows, r);
    if (!reparam) {
        for (int64_t q = 0; q < R; ++q)
            for (int64_t k = 0; k < d; ++k)
                Xd[q * d + k] = Xd[q * d + k] * r[q] * gamma[k];
        contract(Xd, W1d, R, 2 * F, d, Zm);
    } else {
        for (int64_t k = 0; k < d; ++k)
            for (int64_t j = 0; j < 2 * F; ++j)
                W1d[k * 2 * F + j] *= gamma[k];
        contract(Xd, W1d, R, 2 * F, d, Zm);
        for (int64_t q = 0; q < R; ++q)
            for (int64_t j = 0; j < 2 * F; ++j)
                Zm[q * 2 * F + j] *= r[q];
    }
    for (int64_t q = 0; q < R; ++q)
        for (int64_t p = 0; p < F; ++p)
            H[q * F + p] = silu(Zm[q * 2 * F + 2 * p]) * Zm[q * 2 * F + 2 * p + 1];
    contract(H, W2d, R, d2, F, Y);
    for (int64_t q = 0; q < R; ++q) {
        int64_t i = sel_row(rows, q);
        double s = 0.0;
        for (int64_t j = 0; j < d2; ++j) {
            if (Rm)
                Y[q * d2 + j] += bf16_widen(Rm[i * ldr + j]);
            s += Y[q * d2 + j] * Y[q * d2 + j];
        }
        if (ss)
            ss[q] = s;
    }
    free(r); free(Xd); free(W1d); free(W2d); free(Zm); free(H);
    return ORACLE_OK;
}

/* ---- 8-bit operands ------------------------------------------------------------- */

/* OCP 8-bit floating point, E4M3 (OFP8 specification): 1 sign, 4 exponent (bias 7), 3 mantissa bits; no
   infinities; S.1111.111 is NaN; exponent field 0 is subnormal: (-1)^s * 2^-6 * (m / 8); otherwise
   (-1)^s * 2^(e - 7) * (1 + m / 8).  Every such value is exactly representable in bf16, so 8-bit operands reach
   the GEMM definitions above as the bf16 bit patterns of the same numbers: out[i] = bf16 bits of decode(in[i]). */
int coda_oracle_f8e4m3_to_bf16(const uint8_t *in, int64_t n, uint16_t *out)
{
    if (n < 0 || (n > 0 && (!in || !out))) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        const unsigned b = in[i], sgn = b >> 7, e = (b >> 3) & 15u, m = b & 7u;
        double v;
        if (e == 15u && m == 7u)
            v = NAN;
        else if (e == 0u)
            v = ldexp((double)m / 8.0, -6);
        else
            v = ldexp(1.0 + (double)m / 8.0, (int)e - 7);
        if (sgn) v = -v;
        float f = (float)v;      /* exact: at most 4 significant bits */
        uint32_t u;
        memcpy(&u, &f, sizeof u);
        if (v == v && (u & 0xffffu) != 0u) return ORACLE_ERR_ARG;   /* cannot happen for E4M3 */
        out[i] = (uint16_t)(u >> 16);
    }
    return ORACLE_OK;
}

/* ---- one-time weight preparation (definitions) ----------------------------------- */

/* W'[k][j] = gamma[k] * W[k][j] in double (the GPU helper rounds this to bf16). */
int coda_oracle_fold_gamma(const uint16_t *W, int64_t ldw, const double *gamma, int64_t K, int64_t N,
                           double *Wp)
{
    if (!W || !gamma || !Wp)
        return ORACLE_ERR_ARG;
    for (int64_t k = 0; k < K; ++k)
        for (int64_t j = 0; j < N; ++j)
            Wp[k * N + j] = gamma[k] * bf16_widen(W[k * ldw + j]);
    return ORACLE_OK;
}

/* interleavedConcat of two [K x N] matrices: out[k][2j] = Wa[k][j], out[k][2j+1] = Wb[k][j]. */
int coda_oracle_interleave_pairs(const uint16_t *Wa, int64_t lda, const uint16_t *Wb, int64_t ldb,
                                 int64_t K, int64_t N, uint16_t *out)
{
    if (!Wa || !Wb || !out)
        return ORACLE_ERR_ARG;
    for (int64_t k = 0; k < K; ++k)
        for (int64_t j = 0; j < N; ++j) {
            out[k * 2 * N + 2 * j] = Wa[k * lda + j];
            out[k * 2 * N + 2 * j + 1] = Wb[k * ldb + j];
        }
    return ORACLE_OK;
}
