// Instantiations of the 8-bit-operand (OCP E4M3) kernel for one operand-layout pair:
// A stored [M x K] (K-contiguous), B stored [N x K] (K-contiguous).
#define CODA_GEMM_INSTANTIATION_UNIT
#include "gemm_launch.hpp"
namespace coda {
CODA_INSTANTIATE_LAYOUT_F8(true, true)
}
