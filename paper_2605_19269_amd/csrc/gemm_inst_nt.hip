// GEMM+epilogue kernel instantiations for one operand-layout pair:
// A stored [M x K] (K-contiguous), B stored [N x K] (K-contiguous).
#define CODA_GEMM_INSTANTIATION_UNIT
#include "gemm_launch.hpp"
namespace coda {
CODA_INSTANTIATE_LAYOUT(true, true)
}
