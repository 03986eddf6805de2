// gemm_launch.hpp -- host launchers for gemm_kernel, instantiated per layout pair.
#pragma once
#include "gemm_kernel.hpp"

namespace coda {

using MainCfg = TileCfg<256, 256, 64, 2, 4>;   // register-staged kernel (edge tiles)
using FastCfg = DlCfg<256, 256, 2, 4, 4>;       // direct-to-LDS ring (whole tiles only)
static_assert(MainCfg::BM == FastCfg::BM && MainCfg::BN == FastCfg::BN, "both kernels share the tile grid");

template <bool AK, bool BKC, int EPI, bool EDGE>
hipError_t launch_gemm(const GemmParams &p, hipStream_t stream)
{
    const dim3 grid((unsigned)(p.tiles_m * p.tiles_n));
    if constexpr (EDGE) {
        using C = MainCfg;
        hipLaunchKernelGGL((gemm_kernel<C, AK, BKC, EPI, true>), grid, dim3(C::NT), 0, stream, p);
    } else {
        using C = FastCfg;
        hipLaunchKernelGGL((gemm_kernel_dl<C, AK, BKC, EPI>), grid, dim3(C::NT), 0, stream, p);
    }
    return hipGetLastError();
}

#define CODA_INSTANTIATE_ONE(AK, BKC, EPI)                                                   \
    template hipError_t launch_gemm<AK, BKC, EPI, false>(const GemmParams &, hipStream_t);   \
    template hipError_t launch_gemm<AK, BKC, EPI, true>(const GemmParams &, hipStream_t);

#define CODA_INSTANTIATE_LAYOUT(AK, BKC)            \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_LINEAR)       \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_SWIGLU_FWD)   \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_SWIGLU_BWD)   \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_ACCUM)

}  // namespace coda
