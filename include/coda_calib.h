/*
 * coda_calib.h -- calibration kernel for the measurement harness (not a step of the method).
 *
 * The bf16 MFMA rate an MI355X sustains depends on the operand values: the chip holds its
 * 2.4 GHz clock on all-zero operands and lowers it under its power limit when every
 * multiplier input toggles.  coda_calib_mfma_loop measures that ceiling for given operand
 * data with nothing but MFMA instructions in flight (no LDS, no global traffic inside the
 * loop), so that a GEMM's TFLOP/s can be read against what the matrix cores deliver on
 * the same values as well as against the published peak.
 * Same conventions as coda.h: device pointers, nothing allocated, work enqueued on `stream`.
 */
#ifndef CODA_CALIB_H
#define CODA_CALIB_H

#include "coda.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launches n_blocks workgroups of 512 threads (8 wavefronts, two per SIMD when one workgroup
 * is resident per compute unit).  Thread t of block b loads four 16-byte fragments
 * a_frags[((b*4 + i)*512 + t)*16 .. +16), i < 4, and two fragments b_frags[((b*2 + j)*512 + t)*16 .. +16),
 * j < 2 (8 bf16 each), once, then runs `iters` iterations of 16 v_mfma_f32_32x32x16_bf16
 * (each of the 4 x 2 accumulator tiles twice: acc[i][j] += Bfrag[j] x Afrag[i]^T with the b fragment as
 * the first operand, the operand order of the GEMM kernels).
 * Work: n_blocks * 8 * 16 * 32768 * iters FLOP.
 * out (may be NULL): f32 [8][8][16][64]; block 0 writes its accumulators there as
 * out[((wave*8 + i*2 + j)*16 + reg)*64 + lane].
 * Errors: CODA_ERR_NULL (a_frags / b_frags), CODA_ERR_ALIGN (16-byte alignment),
 * CODA_ERR_SHAPE (n_blocks < 0, iters < 0, n_blocks > 65535 * 16), CODA_ERR_LAUNCH.
 */
CODA_API coda_status coda_calib_mfma_loop(void *stream, const void *a_frags, const void *b_frags, int64_t n_blocks,
                                 int64_t iters, float *out);

/*
 * The same measurement on v_mfma_f32_16x16x32_bf16, the instruction of the bf16 GEMM kernel (it draws less
 * power per FLOP than 32x32x16, so its ceiling on non-trivial operands is higher).  Same fragment inputs and
 * launch shape; each iteration runs 32 MFMAs (each of the 4 x 2 accumulator tiles four times), the same
 * FLOP count per iteration as coda_calib_mfma_loop: n_blocks * 8 * 16 * 32768 * iters FLOP in total.
 * A fragment holds row (lane % 16), k = 8*(lane/16) .. +7 of a [16 x 32] operand.
 * out (may be NULL): f32 [8][8][4][64]; block 0 writes its accumulators there as
 * out[((wave*8 + i*2 + j)*4 + reg)*64 + lane] (lane holds row 4*(lane/16) + reg, column lane % 16 of B x A^T).
 * Errors as above.
 */
CODA_API coda_status coda_calib_mfma_loop16(void *stream, const void *a_frags, const void *b_frags, int64_t n_blocks,
                                   int64_t iters, float *out);

#ifdef __cplusplus
}
#endif
#endif
