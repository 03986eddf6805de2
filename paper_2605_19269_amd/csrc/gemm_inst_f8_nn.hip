// Instantiations of the 8-bit-operand (OCP E4M3) kernel for one operand-layout pair:
// A stored [M x K] (K-contiguous), B stored [K x N] (N-contiguous).
#define CODA_GEMM_INSTANTIATION_UNIT
#include "gemm_launch.hpp"
namespace coda {
CODA_INSTANTIATE_LAYOUT_F8(true, false)
}
