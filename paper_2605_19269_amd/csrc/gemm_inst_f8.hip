// Instantiations of the 8-bit-operand kernel (A [M x K], B [N x K], OCP E4M3), one per epilogue mode and kernel kind.
#define CODA_GEMM_INSTANTIATION_UNIT
#include "gemm_launch.hpp"

namespace coda {
template hipError_t launch_gemm_f8<EPI_LINEAR, KIND_WHOLE>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_LINEAR, KIND_RAGGED>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_SWIGLU_FWD, KIND_WHOLE>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_SWIGLU_FWD, KIND_RAGGED>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_SWIGLU_BWD, KIND_WHOLE>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_SWIGLU_BWD, KIND_RAGGED>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_ACCUM, KIND_WHOLE>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_ACCUM, KIND_RAGGED>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_RMSNORM_BWD, KIND_WHOLE>(const GemmParams &, hipStream_t);
template hipError_t launch_gemm_f8<EPI_RMSNORM_BWD, KIND_RAGGED>(const GemmParams &, hipStream_t);
}  // namespace coda
