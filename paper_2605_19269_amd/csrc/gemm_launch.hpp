// gemm_launch.hpp -- host launchers of the GEMM+epilogue kernels, instantiated per layout pair.
#pragma once
#include "gemm_kernel.hpp"

#include <type_traits>

namespace coda {

using FastCfg = DlCfg<256, 256, 2, 4, 4>;       // direct-to-LDS ring of four K-steps of 32; 128x64 wave tiles
constexpr int TILE_M = FastCfg::BM, TILE_N = FastCfg::BN;
constexpr int TILE_K = 64;                      // the kernels walk K-steps of 32 in pairs

// Workgroups of a fast-kernel launch: one per whole tile below split_from, then one per piece of every range of the shared tail.
inline unsigned fast_grid(const GemmParams &p)
{
    const unsigned tiles = (unsigned)(p.tiles_m * p.tiles_n);
    if (p.tail_chunks == 0) return tiles;
    return (unsigned)p.split_from + (unsigned)p.tail_chunks * (unsigned)p.tail_pieces;
}

// `p` arrives without tile counts.
//   KIND_WHOLE:  M, N, K are whole multiples of TILE_M, TILE_N, TILE_K;
//   KIND_RAGGED: anything else (K, N multiples of 8): clamped operand fetches on the edges of M and N, zero-filled K
//                tail, bounds-checked epilogue.
template <bool AK, bool BKC, int EPI, int KIND>
hipError_t launch_gemm(const GemmParams &p_in, hipStream_t stream)
{
    using C = FastCfg;
    GemmParams p = p_in;
    p.tiles_m = (p.M + C::BM - 1) / C::BM;
    p.tiles_n = (p.N + C::BN - 1) / C::BN;
    if (p.tail_chunks > 0)
        hipLaunchKernelGGL((gemm_kernel_dl<C, AK, BKC, EPI, KIND == KIND_RAGGED, true>), dim3(fast_grid(p)), dim3(C::NT), 0, stream, p);
    else
        hipLaunchKernelGGL((gemm_kernel_dl<C, AK, BKC, EPI, KIND == KIND_RAGGED, false>), dim3(fast_grid(p)), dim3(C::NT), 0, stream, p);
    return hipGetLastError();
}

// 8-bit operands.  KIND_WHOLE: M, N multiples of 256 and K a multiple of 128.
template <bool AK, bool BKC, int EPI, int KIND>
hipError_t launch_gemm_f8(const GemmParams &p_in, hipStream_t stream)
{
    using C = FastCfg;
    GemmParams p = p_in;
    p.tiles_m = (p.M + C::BM - 1) / C::BM;
    p.tiles_n = (p.N + C::BN - 1) / C::BN;
    if (p.tail_chunks > 0)
        hipLaunchKernelGGL((gemm_kernel_dl_f8<C, AK, BKC, EPI, KIND == KIND_RAGGED, true>), dim3(fast_grid(p)), dim3(C::NT), 0, stream, p);
    else
        hipLaunchKernelGGL((gemm_kernel_dl_f8<C, AK, BKC, EPI, KIND == KIND_RAGGED, false>), dim3(fast_grid(p)), dim3(C::NT), 0, stream, p);
    return hipGetLastError();
}

#define CODA_INSTANTIATE_ONE(AK, BKC, EPI)                                                   \
    template hipError_t launch_gemm<AK, BKC, EPI, KIND_WHOLE>(const GemmParams &, hipStream_t);   \
    template hipError_t launch_gemm<AK, BKC, EPI, KIND_RAGGED>(const GemmParams &, hipStream_t);

#define CODA_INSTANTIATE_ONE_F8(AK, BKC, EPI)                                                    \
    template hipError_t launch_gemm_f8<AK, BKC, EPI, KIND_WHOLE>(const GemmParams &, hipStream_t);   \
    template hipError_t launch_gemm_f8<AK, BKC, EPI, KIND_RAGGED>(const GemmParams &, hipStream_t);
#define CODA_INSTANTIATE_LAYOUT_F8(AK, BKC)            \
    CODA_INSTANTIATE_ONE_F8(AK, BKC, EPI_LINEAR)       \
    CODA_INSTANTIATE_ONE_F8(AK, BKC, EPI_SWIGLU_FWD)   \
    CODA_INSTANTIATE_ONE_F8(AK, BKC, EPI_SWIGLU_BWD)   \
    CODA_INSTANTIATE_ONE_F8(AK, BKC, EPI_ACCUM)        \
    CODA_INSTANTIATE_ONE_F8(AK, BKC, EPI_RMSNORM_BWD)

#define CODA_INSTANTIATE_LAYOUT(AK, BKC)            \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_LINEAR)       \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_SWIGLU_FWD)   \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_SWIGLU_BWD)   \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_ACCUM)        \
    CODA_INSTANTIATE_ONE(AK, BKC, EPI_RMSNORM_BWD)

// Translation units that only call the launchers (the C ABI) must not instantiate the kernels a second time:
// unless CODA_GEMM_INSTANTIATION_UNIT is defined, every launcher is declared as instantiated elsewhere.
#ifndef CODA_GEMM_INSTANTIATION_UNIT
#define CODA_EXTERN_ONE(AK, BKC, EPI)                                                               \
    extern template hipError_t launch_gemm<AK, BKC, EPI, KIND_WHOLE>(const GemmParams &, hipStream_t);   \
    extern template hipError_t launch_gemm<AK, BKC, EPI, KIND_RAGGED>(const GemmParams &, hipStream_t);
#define CODA_EXTERN_LAYOUT(AK, BKC)            \
    CODA_EXTERN_ONE(AK, BKC, EPI_LINEAR)       \
    CODA_EXTERN_ONE(AK, BKC, EPI_SWIGLU_FWD)   \
    CODA_EXTERN_ONE(AK, BKC, EPI_SWIGLU_BWD)   \
    CODA_EXTERN_ONE(AK, BKC, EPI_ACCUM)        \
    CODA_EXTERN_ONE(AK, BKC, EPI_RMSNORM_BWD)
CODA_EXTERN_LAYOUT(true, false)
CODA_EXTERN_LAYOUT(true, true)
CODA_EXTERN_LAYOUT(false, false)
CODA_EXTERN_LAYOUT(false, true)
#define CODA_EXTERN_ONE_F8(AK, BKC, EPI)                                                                \
    extern template hipError_t launch_gemm_f8<AK, BKC, EPI, KIND_WHOLE>(const GemmParams &, hipStream_t);   \
    extern template hipError_t launch_gemm_f8<AK, BKC, EPI, KIND_RAGGED>(const GemmParams &, hipStream_t);
#define CODA_EXTERN_LAYOUT_F8(AK, BKC)            \
    CODA_EXTERN_ONE_F8(AK, BKC, EPI_LINEAR)       \
    CODA_EXTERN_ONE_F8(AK, BKC, EPI_SWIGLU_FWD)   \
    CODA_EXTERN_ONE_F8(AK, BKC, EPI_SWIGLU_BWD)   \
    CODA_EXTERN_ONE_F8(AK, BKC, EPI_ACCUM)        \
    CODA_EXTERN_ONE_F8(AK, BKC, EPI_RMSNORM_BWD)
CODA_EXTERN_LAYOUT_F8(true, false)
CODA_EXTERN_LAYOUT_F8(true, true)
CODA_EXTERN_LAYOUT_F8(false, false)
CODA_EXTERN_LAYOUT_F8(false, true)
#endif

}  // namespace coda
