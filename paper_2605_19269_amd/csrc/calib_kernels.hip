// calib_kernels.hip -- measurement calibration (include/coda_calib.h): a register-resident bf16 MFMA
// loop on caller-supplied operand fragments.  The sustained rate depends on the operand values
// (power-limited clock), which is why the fragments are an input.
#include "../../include/coda_calib.h"

#include <hip/hip_runtime.h>

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void mfma_loop_kernel(
    const u32x4 *__restrict__ a, const u32x4 *__restrict__ b, int iters, float *__restrict__ out)
{
    const int tid = threadIdx.x;
    bf16x8 fa[4], fb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = __builtin_bit_cast(bf16x8, a[((size_t)blockIdx.x * 4 + i) * 512 + tid]);
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[j] = __builtin_bit_cast(bf16x8, b[((size_t)blockIdx.x * 2 + j) * 512 + tid]);
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    // every wave keeps its accumulators live to the end; only block 0 has somewhere to put them
    if (out != nullptr && blockIdx.x == 0) {
        const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) out[((wave * 8 + i * 2 + j) * 16 + e) * 64 + lane] = acc[i][j][e];
    } else {
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) s += acc[i][j][e];
        asm volatile("" ::"v"(s));
    }
}

// The same loop on v_mfma_f32_16x16x32_bf16, the instruction of the bf16 GEMM kernel: 32 MFMAs per iteration
// (each of the 4 x 2 accumulator tiles four times), the same FLOP count per iteration as above.
typedef __attribute__((ext_vector_type(4))) float f32x4;

__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void mfma_loop16_kernel(
    const u32x4 *__restrict__ a, const u32x4 *__restrict__ b, int iters, float *__restrict__ out)
{
    const int tid = threadIdx.x;
    bf16x8 fa[4], fb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = __builtin_bit_cast(bf16x8, a[((size_t)blockIdx.x * 4 + i) * 512 + tid]);
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[j] = __builtin_bit_cast(bf16x8, b[((size_t)blockIdx.x * 2 + j) * 512 + tid]);
    f32x4 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (out != nullptr && blockIdx.x == 0) {
        const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) out[((wave * 8 + i * 2 + j) * 4 + e) * 64 + lane] = acc[i][j][e];
    } else {
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) s += acc[i][j][e];
        asm volatile("" ::"v"(s));
    }
}

coda_status check_args(const void *a_frags, const void *b_frags, int64_t n_blocks, int64_t iters, const float *out)
{
    if (!a_frags || !b_frags) return CODA_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(a_frags) & 15u) || (reinterpret_cast<uintptr_t>(b_frags) & 15u) ||
        (reinterpret_cast<uintptr_t>(out) & 15u))
        return CODA_ERR_ALIGN;
    if (n_blocks < 0 || iters < 0 || iters > 0x7fffffff || n_blocks > 65535 * 16) return CODA_ERR_SHAPE;
    return CODA_OK;
}

}  // namespace

extern "C" coda_status coda_calib_mfma_loop16(void *stream, const void *a_frags, const void *b_frags, int64_t n_blocks,
                                              int64_t iters, float *out)
{
    const coda_status st = check_args(a_frags, b_frags, n_blocks, iters, out);
    if (st != CODA_OK || n_blocks == 0) return st;
    hipLaunchKernelGGL(mfma_loop16_kernel, dim3((unsigned)n_blocks), dim3(512), 0, (hipStream_t)stream,
                       (const u32x4 *)a_frags, (const u32x4 *)b_frags, (int)iters, out);
    return hipGetLastError() == hipSuccess ? CODA_OK : CODA_ERR_LAUNCH;
}

extern "C" coda_status coda_calib_mfma_loop(void *stream, const void *a_frags, const void *b_frags, int64_t n_blocks,
                                            int64_t iters, float *out)
{
    const coda_status st = check_args(a_frags, b_frags, n_blocks, iters, out);
    if (st != CODA_OK || n_blocks == 0) return st;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3((unsigned)n_blocks), dim3(512), 0, (hipStream_t)stream,
                       (const u32x4 *)a_frags, (const u32x4 *)b_frags, (int)iters, out);
    return hipGetLastError() == hipSuccess ? CODA_OK : CODA_ERR_LAUNCH;
}
