/*
 * coda.h -- C ABI of the MI355X (gfx950) GEMM-plus-epilogue library.
 *
 * One call, coda_gemm, runs a dense bf16 GEMM with fp32 accumulation and then,
 * while the output tile is still in registers, an ordered list of epilogue
 * primitives ("epilogue program") before anything is written to memory.  The
 * method it implements (Section 3.1) keeps the GEMM mainloop fixed and builds every
 * fused operator out of a few epilogue building blocks -- per-row and per-column
 * scaling, tile loads and stores, row and column reductions, maps over adjacent
 * column pairs, in-place accumulation -- applied in list order, as in the
 * paper's kernel example (Appendix "Epilogue Example").  The remaining entry
 * points are the lightweight auxiliary reduction of Section 3.2.1 and one-time
 * weight preparation.
 *
 * Conventions (all entry points)
 *  - Every pointer is a DEVICE pointer unless the comment says "host".  The
 *    caller owns all buffers; the library allocates nothing, keeps no state
 *    beyond a last-HIP-error slot, never synchronises, and only enqueues work
 *    on the given stream (`stream` is a hipStream_t passed as void*, so that
 *    this header needs no HIP header and stays plain C; NULL is the default
 *    stream).
 *  - Matrices are row-major.  `ld` is the row pitch in ELEMENTS.  bf16 is the
 *    upper half of an IEEE binary32, stored as 16-bit words.
 *  - "row" means a row of the GEMM output (a token): a row scale multiplies
 *    row i by r[i], a row reduction sums over the columns of row i.
 *  - Alignment: every matrix pointer 16-byte aligned, every ld a multiple of 8
 *    elements; vectors 4-byte aligned.  Every ld is at most 4194304 elements
 *    (CODA_ERR_SHAPE beyond that: per-lane offsets are formed in 32 bits).
 *  - Errors are return codes; on any error nothing has been enqueued.
 *  - Outputs must not alias inputs, except the in/out buffer of ACCUM_F32.
 */
#ifndef CODA_H
#define CODA_H

#include <stddef.h>
#include <stdint.h>

/* Entry points are the only symbols the shared objects export (they are built with hidden default visibility). */
#if defined(__GNUC__)
#define CODA_API __attribute__((visibility("default")))
#else
#define CODA_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum coda_status {
    CODA_OK = 0,
    CODA_ERR_NULL = 1,      /* a required pointer is NULL                          */
    CODA_ERR_SHAPE = 2,     /* negative / inconsistent / unsupported sizes         */
    CODA_ERR_ALIGN = 3,     /* pointer or leading dimension not aligned            */
    CODA_ERR_DTYPE = 4,     /* operand dtype not supported in that position        */
    CODA_ERR_PROGRAM = 5,   /* epilogue op list is not a supported program         */
    CODA_ERR_WORKSPACE = 6, /* workspace too small                                 */
    CODA_ERR_LAUNCH = 7     /* HIP reported an error; see coda_last_hip_error()    */
} coda_status;

/* CODA_F8E4M3: OCP 8-bit floating point E4M3 (1-4-3, bias 7, max 448, no infinities), one byte per element. */
typedef enum coda_dtype { CODA_BF16 = 0, CODA_F32 = 1, CODA_F8E4M3 = 2 } coda_dtype;

/*
 * A GEMM operand.  rows/cols/ld describe the matrix AS STORED.
 * trans == 0: the GEMM uses it as stored; trans != 0: the GEMM uses its
 * transpose (no data is moved).  coda_gemm computes op(A)[M x K] * op(B)[K x N];
 * the forms D = A B, D = A B^T and D = A^T B of the paper's kernel list are the
 * trans combinations (0,0), (0,1), (1,0).
 */
typedef struct coda_mat {
    const void *ptr; /* device */
    int64_t rows, cols, ld;
    int32_t trans;
    int32_t dtype; /* coda_dtype; operands are both CODA_BF16 or both CODA_F8E4M3 (see coda_gemm) */
} coda_mat;

/*
 * Epilogue primitives (Section 3.1: elementwise and pairwise maps, vector loads,
 * tile loads and stores, tile reductions; Appendix "List of Kernels").
 * "v" is the running fp32 value of output element (i, j); W is the current
 * width (N until a pairwise op changes it).
 */
typedef enum coda_epi_kind {
    /* v *= r[i].               in: f32[M]            (Kernel 5: O = D (.) r)          */
    CODA_EPI_ROW_SCALE = 0,
    /* side output, v unchanged: out[i][j] = bf16(v * gamma[j]).
       in: f32[N] gamma, out: bf16[M x N] (ld_out)   (Kernel 4: O = D (.) gamma)      */
    CODA_EPI_COL_SCALE_SIDE = 1,
    /* v += float(C[i][j]).     in: bf16[M x N] (ld_in)  (Kernel 4: D = A B + C)      */
    CODA_EPI_ADD_TILE = 2,
    /* Pairwise, width N -> N/2 (Kernels 2, 6): g = v[i][2p], u = v[i][2p+1],
       v'[i][p] = silu(g) * u.  Optional out: bf16[M x N] (ld_out) receives the
       pre-activation v (what Kernel 10 later reads as Z).  N must be even.            */
    CODA_EPI_SWIGLU_FWD = 3,
    /* Pairwise, width N -> 2N (Kernel 10): with d = v[i][j], g = Z[i][2j],
       u = Z[i][2j+1]:  v'[i][2j] = d*u*(sigma(g) + silu(g)*(1 - sigma(g))),
       v'[i][2j+1] = d*silu(g).   in: bf16[M x 2N] Z (ld_in).
       Optional out: bf16[M x N] (ld_out) receives silu(g)*u (the recomputed
       forward activation).  Optional out2: f32 row statistic
       sum_j (g*dG + u*dU), laid out per `flags` like ROW_SUMSQ.                       */
    CODA_EPI_SWIGLU_BWD = 4,
    /* Row reduction of v*v over the columns of this tile, taken on the fp32
       value before any rounding (Kernel 4: reduceTile_cols(D (.) D)).
       out: f32, layout chosen by `flags`:
         CODA_REDUCE_PARTIALS: out is [nblk x M] (block-major: out[b*M + i]),
             nblk = coda_row_partial_blocks(N); every entry is overwritten;
             combine with coda_row_finalize.  Deterministic.
         CODA_REDUCE_ATOMIC:   out is f32[M], pre-zeroed by the caller; tiles add
             into it with fp32 atomics (summation order varies run to run).            */
    CODA_EPI_ROW_SUMSQ = 5,
    /* Final op: round v to `flags & CODA_STORE_F32 ? f32 : bf16` (nearest even)
       and write out[i][j], width W (ld_out).                                          */
    CODA_EPI_STORE = 6,
    /* Final op: out[i][j] += v in fp32, in place (the weight-gradient GEMM of
       Theorem 1 accumulated into an existing gradient buffer). out: f32[M x N].       */
    CODA_EPI_ACCUM_F32 = 7,
    /* Pairwise, width unchanged (Kernels 1, 7: O = RoPE(D)): rotate adjacent column pairs
       (2p, 2p+1) of the first i1 = rope_cols columns by the angle of (position of row i,
       frequency f = p mod (head_dim/2)):  v'[2p] = x0*cos - x1*sin,  v'[2p+1] = x0*sin + x1*cos.
       in: f32 cos table [T x head_dim/2] (dense), in2: f32 sin table (same shape),
       in3: int32 pos[M], i0 = head_dim (multiple of 8), i1 = rope_cols (multiple of 8, <= N),
       ld_in = T, the number of table rows (T * head_dim/2 < 2^31).  A position outside [0, T) is
       clamped to the nearest table row (never read out of bounds).  Columns >= rope_cols pass through.
       The paper pre-broadcasts the tables to [M x N/2]; indexing a [T x head_dim/2] table by
       position gives the same values without that input traffic.                       */
    CODA_EPI_ROPE = 8,
    /* Local part of RMSNorm backward (Kernel 9).  v = D is the gradient w.r.t. the normalised
       activation.  With C the RMSNorm input, r its inverse-rms factor, z the row statistic
       z[i] = (1/d) sum_j (grad_h2 * h2)[i][j] and cn = C (.) r:
           v'[i][j] = ( v*gamma[j] - cn[i][j]*z[i] ) * r[i]
       (follow with ADD_TILE to add the incoming residual gradient O_in, then STORE = O_out).
       in: bf16 C [M x N] (ld_in); in2: f32 r[M]; in3: f32 z[M]; in4: f32 gamma[N] (16-byte aligned).
       i0 = 0: in3 is z itself.  i0 = d > 0: in3 holds the raw row sums sum_j (grad_h2 * h2)[i][j], as the row
       statistic of SWIGLU_BWD leaves them (after coda_row_finalize, or directly with CODA_REDUCE_ATOMIC), and the
       kernel uses z[i] = in3[i] / d -- the chain Kernel 10 -> auxiliary combine -> Kernel 9 needs no scaling pass.
       Optional out: bf16 [M x N] (ld_out) receives C_out = cn (.) gamma (the normalised activation).
       Optional out2: f32 column reduction dgamma[j] = sum_i v[i][j]*cn[i][j] of this tile row, laid
       out per `flags`: CODA_REDUCE_PARTIALS: [nblk x N] block-major (out2[b*N + j]),
       nblk = coda_col_partial_blocks(M), combine with coda_col_finalize; CODA_REDUCE_ATOMIC: f32[N]
       pre-zeroed by the caller.                                                           */
    CODA_EPI_RMSNORM_BWD = 9,
    /* Cross-entropy pieces (Kernels 3, 8): v unchanged (follow with STORE to materialise the logits).
       Per 256-column tile b and row i, on the fp32 value before rounding:
           out [b*M + i] = max_j v[i][j],   out2[b*M + i] = sum_j exp(v[i][j] - max)      (f32 [nblk x M] each,
           nblk = coda_row_partial_blocks(N), every entry overwritten; combine with coda_lse_finalize)
           out3[i] = v[i][y[i]]  (f32[M], the target logit; written by the tile that holds column y[i]).
       in3: int32 y[M] with 0 <= y < N (not checked; an out-of-range y leaves out3[i] unwritten).       */
    CODA_EPI_LSE_PARTIAL = 10
} coda_epi_kind;

#define CODA_REDUCE_PARTIALS 0u
#define CODA_REDUCE_ATOMIC 1u
#define CODA_STORE_F32 2u

typedef struct coda_epi_op {
    int32_t kind;   /* coda_epi_kind */
    uint32_t flags; /* see the op */
    const void *in; /* device */
    void *out;      /* device */
    void *out2;     /* device */
    int64_t ld_in, ld_out;
    const void *in2; /* device; second / third input of ops that take several (ROPE) */
    const void *in3; /* device */
    const void *in4; /* device */
    void *out3;      /* device */
    int64_t i0, i1;  /* integer parameters of the op (ROPE: head_dim, rope_cols; RMSNORM_BWD: i0 = d or 0) */
} coda_epi_op;

/*
 * D = op(A) op(B) (bf16 in, fp32 accumulate), then `prog[0..n_ops)` in order.
 *
 * Supported programs (anything else -> CODA_ERR_PROGRAM): ops must appear in
 * the order
 *     [ROW_SCALE] [ADD_TILE] [ROW_SUMSQ] [COL_SCALE_SIDE] STORE
 *     [ROW_SCALE] ROPE STORE
 *     [ROW_SCALE] LSE_PARTIAL STORE
 *     [ROW_SCALE] SWIGLU_FWD STORE
 *     SWIGLU_BWD STORE
 *     RMSNORM_BWD [ADD_TILE] STORE
 *     ACCUM_F32
 * with bracketed ops optional and each at most once.  These cover Kernels 1 to 10, the plain GEMM (STORE alone) and the accumulating weight gradient.
 *
 * Sizes: M, N, K >= 0 must equal the op() shapes of A and B.  M == 0 or N == 0
 * is a no-op; K == 0 runs the program on D = 0.  K must be a multiple of 8; N a
 * multiple of 8; and M a multiple of 8 when A is used transposed.  No other
 * divisibility is required (edge tiles are predicated).
 *
 * Reproducibility: the order of the fp32 additions behind an output element depends only on the shapes, layouts and the
 * element's position, never on timing; with CODA_REDUCE_PARTIALS every output of a call is bitwise identical from call
 * to call (CODA_REDUCE_ATOMIC sums may differ in their last bits).
 *
 * 8-bit operands: A and B may both be CODA_F8E4M3 (ld in elements = bytes, a multiple of 16), in any of the four
 * trans combinations: forward weights kept [in x out], the backward form A B^T and the weight-gradient form A^T B
 * all run on the fp8 matrix cores.  The contraction accumulates the exact products in fp32, and every epilogue
 * program above applies unchanged (outputs stay bf16 / fp32; quantisation scales of the operands are the caller's
 * and fold into ROW_SCALE).  Operands move in 16-byte chunks along whichever index is contiguous in memory: K must
 * be a multiple of 16; N must be a multiple of 16 when B is stored [K x N] (trans = 0), else of 8; M must be a
 * multiple of 16 when A is stored [K x M] (trans = 1), else it is free.  Mixed operand dtypes are CODA_ERR_DTYPE,
 * sizes that break these rules CODA_ERR_SHAPE.
 *
 * workspace / workspace_bytes (device memory, 16-byte aligned; may be NULL): scratch for sharing output tiles
 * among workgroups (split-K / stream-K).  A shape with fewer than 256 output tiles (256 x 256, counted with a ragged
 * edge) leaves compute units idle, and a shape with more ends with a partly filled round of tiles.  When those
 * tiles (the "tail") number at most 128 and the contraction is long enough (K >= 2048, and every workgroup must be
 * spared at least 64 K-steps of 32 elements), coda_gemm_workspace_bytes returns a non-zero size, and a call that brings
 * that much workspace cuts the K-steps of the tail, laid end to end, into up to 256 equal contiguous ranges, one or two
 * workgroups each (a range may end in one tile and begin in the next): partial tiles go to the workspace in fp32, and
 * the workgroup that reaches a tile last adds its parts up in a fixed order (the result does not depend on arrival
 * order) and runs the epilogue program on the sum.  Without a workspace (NULL) the same shape runs unsplit.  A non-NULL
 * workspace smaller than coda_gemm_workspace_bytes(...) is CODA_ERR_WORKSPACE.  The workspace needs no initialisation
 * and holds nothing between calls; two calls that share one must not overlap in time.
 */
CODA_API coda_status coda_gemm(void *stream, int64_t M, int64_t N, int64_t K, const coda_mat *A,
                      const coda_mat *B, const coda_epi_op *prog /* host */, int32_t n_ops,
                      void *workspace, size_t workspace_bytes);

/*
 * coda_gemm for callers that cannot allocate device memory or hand in a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Identical to coda_gemm -- same arguments, same programs, same
 * results bit for bit -- except that the split-K workspace is a static device array inside the library
 * (CODA_STATIC_WS_BYTES = 32 MiB + 1 KiB per GPU, part of the code object's data, held from library load until the
 * process ends) instead of a caller buffer.  The call allocates nothing and frees nothing.  Shapes that are not planned
 * for split-K do not touch the array.  A shape whose split-K plan needs more than the array holds
 * (coda_gemm_workspace_bytes(...) > CODA_STATIC_WS_BYTES, e.g. 2048 x 2048 x 8192: 64 tiles in 4 parts each) is refused with
 * CODA_ERR_WORKSPACE and nothing is enqueued: run it through coda_gemm with a workspace of the caller's, or with NULL.
 * The array keeps whatever the previous call left in it; the ticket counters are cleared by a small kernel ahead of
 * every split launch (no memset node, so the call can be captured into a HIP graph).  All calls on one GPU share that
 * GPU's array: two calls that overlap in time on one GPU (different streams) race.  The first call on a GPU looks the
 * array's device address up (one symbol query, error code CODA_ERR_LAUNCH if that fails).
 */
#define CODA_STATIC_WS_BYTES ((size_t)32 * 1024 * 1024 + 1024)
CODA_API coda_status coda_gemm_static_ws(void *stream, int64_t M, int64_t N, int64_t K, const coda_mat *A,
                                const coda_mat *B, const coda_epi_op *prog /* host */, int32_t n_ops);

/* Bytes of workspace that enable tile sharing for this shape; 0 when the shape runs unsplit (the program does not matter;
   the figure is sufficient for bf16 and for 8-bit operands alike).  Sharing tiles is this library's answer to the
   tile-count quantisation that the paper leaves to its expert-written mainloop (Section 3.1: the mainloop is taken
   as given); nothing in the method depends on it. */
CODA_API size_t coda_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, const coda_epi_op *prog /* host */,
                                 int32_t n_ops);

/* Number of column blocks nblk of a CODA_REDUCE_PARTIALS buffer for output width N (the partial buffer is
   f32[nblk x M]): one partial per row and output tile, the tile-level partial reduction of Section 3.1
   ("tile reductions") that Section 3.2.1 combines in its auxiliary kernel.  `prog` / `n_ops` name the program
   the buffer is for; every program of this build reduces over the same 256-column tiles, so they may be NULL / 0. */
CODA_API int64_t coda_row_partial_blocks(int64_t N, const coda_epi_op *prog /* host, may be NULL */, int32_t n_ops);

/*
 * Lightweight auxiliary reduction (Section 3.2.1): combine tile partials and
 * optionally form r = 1/sqrt(reduce(partials)/d + eps).
 * partials: f32[nblk x M] (block-major).  sum_out, rstd_out: f32[M], either may
 * be NULL (not both).  d > 0 is the hidden size the mean is taken over.
 */
CODA_API coda_status coda_row_finalize(void *stream, const float *partials, int64_t M, int64_t nblk,
                              float *sum_out, float *rstd_out, int64_t d, float eps);

/* Auxiliary reduction of the log-sum-exp partials (Section 3.2.3: the per-tile maximum and sum-exp statistics are
   combined across tiles by a separate small kernel): lse[i] = M_i + log sum_b psum[b][i] exp(pmax[b][i] - M_i), M_i = max_b pmax[b][i];
   loss[i] = lse[i] - ztgt[i].  pmax, psum: f32[nblk x M]; ztgt f32[M] (needed only for loss_out);
   lse_out, loss_out: f32[M], either may be NULL (not both). */
CODA_API coda_status coda_lse_finalize(void *stream, const float *pmax, const float *psum, int64_t M, int64_t nblk,
                              const float *ztgt, float *lse_out, float *loss_out);

/* Number of row blocks nblk of a column-reduction partial buffer (f32[nblk x N]) for M output rows. */
CODA_API int64_t coda_col_partial_blocks(int64_t M);

/* Auxiliary reduction over column partials (the reduce_rows step of the RMSNorm weight gradient,
   Appendix "GEMM-RMSNorm-GEMM Backward Pass"): out[j] = sum_b partials[b*N + j].  partials f32[nblk x N]. */
CODA_API coda_status coda_col_finalize(void *stream, const float *partials, int64_t N, int64_t nblk, float *out);

/* ss[i] = sum_k X[i][k]^2 in fp32 for a bf16 matrix not produced by coda_gemm (the first layer's input): the
   row statistic behind r = 1/rms(x) of Section 3.2.1, which every later layer gets from the previous GEMM's
   ROW_SUMSQ epilogue instead.  X->trans must be 0.  sum_out: f32[X->rows]. */
CODA_API coda_status coda_row_sumsq(void *stream, const coda_mat *X, float *sum_out);

/* One-time weight preparation: W_out[k][j] = bf16(gamma[k] * W[k][j]) so that
   RMSNorm(x, gamma) W == diag(r) (x W_out): the reparameterisation of Section 3.2.1 (the normalisation's row factor
   commutes with the GEMM and moves into its epilogue) with the column factor gamma moved the other way, into the
   weight.  The paper keeps gamma in the epilogue of the producing GEMM (Kernel 4, available here as COL_SCALE_SIDE);
   folding is this library's default because it costs nothing per step.  One rounding to bf16 per weight element.
   W is [K x N] as stored (trans 0); gamma f32[K]; W_out bf16 [K x N] with row pitch ld_out (elements; lets W_out be
   a column block of a larger fused weight). */
CODA_API coda_status coda_fold_gamma(void *stream, const coda_mat *W, const float *gamma, void *W_out,
                            int64_t ld_out);

/* One-time weight preparation: interleave the columns of two [K x N] bf16
   matrices: W_out[k][2j] = Wa[k][j] (gate), W_out[k][2j+1] = Wb[k][j] (up), the column order that the pairwise
   SwiGLU epilogues split again (Section 3.2.2; interleavedSplit in Kernels 2, 6 and 10).
   W_out is bf16 [K x 2N] with row pitch ld_out (elements). */
CODA_API coda_status coda_interleave_pairs(void *stream, const coda_mat *Wa, const coda_mat *Wb, void *W_out,
                                  int64_t ld_out);

CODA_API const char *coda_status_string(coda_status s);
/* The hipError_t (as int) recorded by the most recent CODA_ERR_LAUNCH on this thread. */
CODA_API int coda_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CODA_H */
