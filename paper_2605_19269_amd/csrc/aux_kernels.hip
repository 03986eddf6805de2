// aux_kernels.hip -- small HBM-bound kernels around the GEMM (gfx950).
//  * row_finalize: the small auxiliary reduction of Section 3.2.1: sums the per-tile
//    partial row reductions and optionally forms r = 1/sqrt(sum/d + eps).
//  * row_sumsq: sum of squares of each row of a bf16 matrix that no GEMM of ours produced.
//  * fold_gamma / interleave_pairs: one-time weight preparation.
// All of them move 16 bytes per lane per access and are bound by HBM bandwidth.
#include "aux_kernels.hpp"

namespace coda {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

static __device__ __forceinline__ float lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
static __device__ __forceinline__ float hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
static __device__ __forceinline__ uint32_t pack(float a, float b)
{
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// The three combine kernels share one shape: a workgroup of four waves owns 64 consecutive rows (columns for the column
// reduction); lane l of every wave reads row l of a block, so a wave-load is 256 contiguous bytes, and wave w takes
// blocks w, w + 4, w + 8, ... with four loads in flight.  The four waves meet in LDS and wave 0 combines them in wave
// order, so the summation order is fixed.  (One thread per row walking all blocks alone keeps 1/8 of the chip busy with
// one dependent load at a time: 83 us for the 128 blocks of a 32768-wide vocabulary instead of a few.)
constexpr int FIN_ROWS = 64, FIN_WAVES = 4;

// partials is [nblk x M]
__global__ __launch_bounds__(256) void row_finalize_kernel(const float *__restrict__ partials, int64_t M, int64_t nblk,
                                                           float *__restrict__ sum_out, float *__restrict__ rstd_out,
                                                           float inv_d, float eps)
{
    __shared__ float part[FIN_WAVES][FIN_ROWS];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * FIN_ROWS + lane;
    float s = 0.0f;
    if (i < M) {
        int64_t b = w;
        for (; b + 3 * FIN_WAVES < nblk; b += 4 * FIN_WAVES) {
            const float v0 = partials[b * M + i], v1 = partials[(b + FIN_WAVES) * M + i];
            const float v2 = partials[(b + 2 * FIN_WAVES) * M + i], v3 = partials[(b + 3 * FIN_WAVES) * M + i];
            s += v0; s += v1; s += v2; s += v3;
        }
        for (; b < nblk; b += FIN_WAVES) s += partials[b * M + i];
    }
    part[w][lane] = s;
    __syncthreads();
    if (w != 0 || i >= M) return;
    s = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
    if (sum_out) sum_out[i] = s;
    if (rstd_out) rstd_out[i] = 1.0f / sqrtf(s * inv_d + eps);
}

// Combine per-tile (max, sum-exp) pairs of each row into the row's log-sum-exp; optionally the per-token loss.
// Each wave keeps a running (max, sum) over its blocks with the usual rescaling rule.
__device__ __forceinline__ void lse_merge(float &m, float &s, float pm, float ps)
{
    const float mn = fmaxf(m, pm);
    if (mn == -__builtin_inff()) return;        // both empty
    s = s * __expf(m - mn) + ps * __expf(pm - mn);
    m = mn;
}
__global__ __launch_bounds__(256) void lse_finalize_kernel(const float *__restrict__ pmax, const float *__restrict__ psum,
                                                           int64_t M, int64_t nblk, const float *__restrict__ ztgt,
                                                           float *__restrict__ lse_out, float *__restrict__ loss_out)
{
    __shared__ float pm_[FIN_WAVES][FIN_ROWS], ps_[FIN_WAVES][FIN_ROWS];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * FIN_ROWS + lane;
    float m = -__builtin_inff(), s = 0.0f;
    if (i < M) {
        int64_t b = w;
        for (; b + 3 * FIN_WAVES < nblk; b += 4 * FIN_WAVES) {
            float vm[4], vs[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                vm[q] = pmax[(b + q * FIN_WAVES) * M + i];
                vs[q] = psum[(b + q * FIN_WAVES) * M + i];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) lse_merge(m, s, vm[q], vs[q]);
        }
        for (; b < nblk; b += FIN_WAVES) lse_merge(m, s, pmax[b * M + i], psum[b * M + i]);
    }
    pm_[w][lane] = m;
    ps_[w][lane] = s;
    __syncthreads();
    if (w != 0 || i >= M) return;
#pragma unroll
    for (int q = 1; q < FIN_WAVES; ++q) lse_merge(m, s, pm_[q][lane], ps_[q][lane]);
    const float lse = m + logf(s);
    if (lse_out) lse_out[i] = lse;
    if (loss_out) loss_out[i] = lse - ztgt[i];
}

// partials is [nblk x N]
__global__ __launch_bounds__(256) void col_finalize_kernel(const float *__restrict__ partials, int64_t N, int64_t nblk,
                                                           float *__restrict__ out)
{
    __shared__ float part[FIN_WAVES][FIN_ROWS];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t j = (int64_t)blockIdx.x * FIN_ROWS + lane;
    float s = 0.0f;
    if (j < N) {
        int64_t b = w;
        for (; b + 3 * FIN_WAVES < nblk; b += 4 * FIN_WAVES) {
            const float v0 = partials[b * N + j], v1 = partials[(b + FIN_WAVES) * N + j];
            const float v2 = partials[(b + 2 * FIN_WAVES) * N + j], v3 = partials[(b + 3 * FIN_WAVES) * N + j];
            s += v0; s += v1; s += v2; s += v3;
        }
        for (; b < nblk; b += FIN_WAVES) s += partials[b * N + j];
    }
    part[w][lane] = s;
    __syncthreads();
    if (w != 0 || j >= N) return;
    out[j] = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
}

// One wavefront per row, 16 bytes per lane per step, butterfly reduction at the end.
__global__ __launch_bounds__(256) void row_sumsq_kernel(const uint16_t *__restrict__ X, int64_t M, int64_t K, int64_t ld,
                                                        float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const uint16_t *x = X + row * ld;
    float s = 0.0f;
    for (int64_t k = lane * 8; k < K; k += 64 * 8) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(x + k);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float a = lo(v[e]), b = hi(v[e]);
            s += a * a + b * b;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) out[row] = s;
}

__global__ __launch_bounds__(256) void fold_gamma_kernel(const uint16_t *__restrict__ W, int64_t K, int64_t N, int64_t ld,
                                                         const float *__restrict__ gamma, uint16_t *__restrict__ out,
                                                         int64_t ld_out)
{
    const int64_t chunks = N / 8;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= K * chunks) return;
    const int64_t k = id / chunks, c = id % chunks;
    const float g = gamma[k];
    const u32x4 v = *reinterpret_cast<const u32x4 *>(W + k * ld + c * 8);
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = pack(g * lo(v[e]), g * hi(v[e]));
    *reinterpret_cast<u32x4 *>(out + k * ld_out + c * 8) = o;
}

__global__ __launch_bounds__(256) void interleave_pairs_kernel(const uint16_t *__restrict__ Wa, int64_t lda,
                                                               const uint16_t *__restrict__ Wb, int64_t ldb, int64_t K,
                                                               int64_t N, uint16_t *__restrict__ out, int64_t ld_out)
{
    const int64_t chunks = N / 8;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= K * chunks) return;
    const int64_t k = id / chunks, c = id % chunks;
    const u32x4 a = *reinterpret_cast<const u32x4 *>(Wa + k * lda + c * 8);
    const u32x4 b = *reinterpret_cast<const u32x4 *>(Wb + k * ldb + c * 8);
    u32x4 o0, o1;  // (a0,b0)(a1,b1)... : low half-word first
    o0[0] = (a[0] & 0xffffu) | (b[0] << 16);
    o0[1] = (a[0] >> 16) | (b[0] & 0xffff0000u);
    o0[2] = (a[1] & 0xffffu) | (b[1] << 16);
    o0[3] = (a[1] >> 16) | (b[1] & 0xffff0000u);
    o1[0] = (a[2] & 0xffffu) | (b[2] << 16);
    o1[1] = (a[2] >> 16) | (b[2] & 0xffff0000u);
    o1[2] = (a[3] & 0xffffu) | (b[3] << 16);
    o1[3] = (a[3] >> 16) | (b[3] & 0xffff0000u);
    u32x4 *dst = reinterpret_cast<u32x4 *>(out + k * ld_out + c * 16);
    dst[0] = o0;
    dst[1] = o1;
}

static inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

hipError_t launch_row_finalize(hipStream_t s, const float *partials, int64_t M, int64_t nblk, float *sum_out,
                               float *rstd_out, float inv_d, float eps)
{
    hipLaunchKernelGGL(row_finalize_kernel, dim3(blocks_for(M, FIN_ROWS)), dim3(256), 0, s, partials, M, nblk, sum_out,
                       rstd_out, inv_d, eps);
    return hipGetLastError();
}

hipError_t launch_lse_finalize(hipStream_t s, const float *pmax, const float *psum, int64_t M, int64_t nblk, const float *ztgt,
                               float *lse_out, float *loss_out)
{
    hipLaunchKernelGGL(lse_finalize_kernel, dim3(blocks_for(M, FIN_ROWS)), dim3(256), 0, s, pmax, psum, M, nblk, ztgt, lse_out,
                       loss_out);
    return hipGetLastError();
}

hipError_t launch_col_finalize(hipStream_t s, const float *partials, int64_t N, int64_t nblk, float *out)
{
    hipLaunchKernelGGL(col_finalize_kernel, dim3(blocks_for(N, FIN_ROWS)), dim3(256), 0, s, partials, N, nblk, out);
    return hipGetLastError();
}

hipError_t launch_row_sumsq(hipStream_t s, const uint16_t *X, int64_t M, int64_t K, int64_t ld, float *sum_out)
{
    hipLaunchKernelGGL(row_sumsq_kernel, dim3(blocks_for(M, 4)), dim3(256), 0, s, X, M, K, ld, sum_out);
    return hipGetLastError();
}

hipError_t launch_fold_gamma(hipStream_t s, const uint16_t *W, int64_t K, int64_t N, int64_t ld, const float *gamma,
                             uint16_t *out, int64_t ld_out)
{
    hipLaunchKernelGGL(fold_gamma_kernel, dim3(blocks_for(K * (N / 8), 256)), dim3(256), 0, s, W, K, N, ld, gamma, out,
                       ld_out);
    return hipGetLastError();
}

hipError_t launch_interleave_pairs(hipStream_t s, const uint16_t *Wa, int64_t lda, const uint16_t *Wb, int64_t ldb,
                                   int64_t K, int64_t N, uint16_t *out, int64_t ld_out)
{
    hipLaunchKernelGGL(interleave_pairs_kernel, dim3(blocks_for(K * (N / 8), 256)), dim3(256), 0, s, Wa, lda, Wb, ldb, K,
                       N, out, ld_out);
    return hipGetLastError();
}

}  // namespace coda
