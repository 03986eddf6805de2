// aux_kernels.hpp -- host launchers of the small memory-bound kernels around the GEMM:
// the auxiliary reduction over tile partials, the stand-alone row sum of squares and
// the one-time weight preparation.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace coda {

hipError_t launch_row_finalize(hipStream_t s, const float *partials, int64_t M, int64_t nblk, float *sum_out,
                               float *rstd_out, float inv_d, float eps);
hipError_t launch_lse_finalize(hipStream_t s, const float *pmax, const float *psum, int64_t M, int64_t nblk, const float *ztgt,
                               float *lse_out, float *loss_out);
hipError_t launch_col_finalize(hipStream_t s, const float *partials, int64_t N, int64_t nblk, float *out);
hipError_t launch_row_sumsq(hipStream_t s, const uint16_t *X, int64_t M, int64_t K, int64_t ld, float *sum_out);
hipError_t launch_fold_gamma(hipStream_t s, const uint16_t *W, int64_t K, int64_t N, int64_t ld, const float *gamma,
                             uint16_t *out, int64_t ld_out);
hipError_t launch_interleave_pairs(hipStream_t s, const uint16_t *Wa, int64_t lda, const uint16_t *Wb, int64_t ldb,
                                   int64_t K, int64_t N, uint16_t *out, int64_t ld_out);

}  // namespace coda
