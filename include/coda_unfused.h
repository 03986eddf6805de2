/*
 * coda_unfused.h -- the separate memory-bound kernels of the UNFUSED operator chain.
 *
 * These exist only as the measurement baseline ("speedup vs unfused"): the same GEMM
 * mainloop with a plain store, followed by stand-alone elementwise / reduction kernels
 * that each make their own round trip through HBM -- the canonical formulation that
 * the paper's reparameterisation removes (Section 3.2.2 describes it: the GEMM output is
 * written out, split into pairs and transformed by a separate kernel).
 * Same conventions as coda.h: device pointers, row-major, ld in elements, 16-byte
 * aligned, widths multiples of 8, nothing allocated, work enqueued on `stream`.
 */
#ifndef CODA_UNFUSED_H
#define CODA_UNFUSED_H

#include "coda.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Xn[i][k] = bf16( X[i][k] * r[i] * gamma[k] );  gamma may be NULL (= 1).  X, Xn bf16 [M x K]. */
CODA_API coda_status coda_unfused_rmsnorm_apply(void *stream, const void *X, int64_t ldx, const float *r,
                                       const float *gamma, int64_t M, int64_t K, void *Xn, int64_t ldo);

/* H[i][p] = bf16( silu(Z[i][2p]) * Z[i][2p+1] );  Z bf16 [M x 2F], H bf16 [M x F]. */
CODA_API coda_status coda_unfused_swiglu_fwd(void *stream, const void *Z, int64_t ldz, int64_t M, int64_t F,
                                    void *H, int64_t ldh);

/* Kernel 10's pairwise rule as its own kernel: dH bf16 [M x F], Z bf16 [M x 2F] -> dZ bf16 [M x 2F]. */
CODA_API coda_status coda_unfused_swiglu_bwd(void *stream, const void *dH, int64_t lddh, const void *Z, int64_t ldz,
                                    int64_t M, int64_t F, void *dZ, int64_t lddz);

/* Y = bf16( D + R ), ss[i] = sum_j (D+R)[i][j]^2 in fp32.  D, R, Y bf16 [M x N]; ss f32[M] (may be NULL). */
CODA_API coda_status coda_unfused_add_sumsq(void *stream, const void *D, int64_t ldd, const void *R, int64_t ldr,
                                   int64_t M, int64_t N, void *Y, int64_t ldy, float *ss);

/* G[i][j] += T[i][j] in fp32.  G, T f32 [M x N]. */
CODA_API coda_status coda_unfused_accumulate(void *stream, const float *T, int64_t ldt, int64_t M, int64_t N, float *G,
                                    int64_t ldg);

#ifdef __cplusplus
}
#endif
#endif
