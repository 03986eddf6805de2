// baseline_kernels.hip -- stand-alone elementwise / reduction kernels of the UNFUSED operator
// chain (include/coda_unfused.h).  Measurement baseline only: each kernel reads its operands
// from HBM and writes its result back, which is exactly the traffic the fused epilogues avoid.
// One wavefront walks one row, 16 bytes per lane per access.
#include "../../include/coda_unfused.h"

#include <hip/hip_runtime.h>

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

__device__ __forceinline__ float lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack(float a, float b)
{
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float sigmoidf_fast(float g) { return __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

#define ROW_SETUP                                                       \
    const int lane = threadIdx.x & 63;                                  \
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   \
    if (row >= M) return;

__global__ __launch_bounds__(256) void rmsnorm_apply_kernel(const uint16_t *__restrict__ X, int64_t ldx,
                                                            const float *__restrict__ r, const float *__restrict__ gamma,
                                                            int64_t M, int64_t K, uint16_t *__restrict__ O, int64_t ldo)
{
    ROW_SETUP
    const float ri = r[row];
    for (int64_t k = lane * 8; k < K; k += 512) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(X + row * ldx + k);
        float g[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] = gamma ? gamma[k + e] : 1.0f;
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = pack(lo(v[e]) * ri * g[2 * e], hi(v[e]) * ri * g[2 * e + 1]);
        *reinterpret_cast<u32x4 *>(O + row * ldo + k) = o;
    }
}

__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const uint16_t *__restrict__ Z, int64_t ldz, int64_t M, int64_t F,
                                                         uint16_t *__restrict__ H, int64_t ldh)
{
    ROW_SETUP
    for (int64_t p = lane * 8; p < F; p += 512) {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(Z + row * ldz + 2 * p);
        const u32x4 b = *reinterpret_cast<const u32x4 *>(Z + row * ldz + 2 * p + 8);
        float h[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h[e] = lo(a[e]) * sigmoidf_fast(lo(a[e])) * hi(a[e]);
            h[4 + e] = lo(b[e]) * sigmoidf_fast(lo(b[e])) * hi(b[e]);
        }
        u32x4 o = {pack(h[0], h[1]), pack(h[2], h[3]), pack(h[4], h[5]), pack(h[6], h[7])};
        *reinterpret_cast<u32x4 *>(H + row * ldh + p) = o;
    }
}

__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const uint16_t *__restrict__ dH, int64_t lddh,
                                                         const uint16_t *__restrict__ Z, int64_t ldz, int64_t M, int64_t F,
                                                         uint16_t *__restrict__ dZ, int64_t lddz)
{
    ROW_SETUP
    for (int64_t p = lane * 8; p < F; p += 512) {
        const u32x4 d = *reinterpret_cast<const u32x4 *>(dH + row * lddh + p);
        const u32x4 z0 = *reinterpret_cast<const u32x4 *>(Z + row * ldz + 2 * p);
        const u32x4 z1 = *reinterpret_cast<const u32x4 *>(Z + row * ldz + 2 * p + 8);
        u32x4 o0, o1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t zw = e < 4 ? z0[e] : z1[e - 4];
            const float dd = (e & 1) ? hi(d[e >> 1]) : lo(d[e >> 1]);
            const float g = lo(zw), u = hi(zw);
            const float sg = sigmoidf_fast(g), sl = g * sg;
            const uint32_t w = pack(dd * u * (sg + sl * (1.0f - sg)), dd * sl);
            if (e < 4) o0[e] = w; else o1[e - 4] = w;
        }
        *reinterpret_cast<u32x4 *>(dZ + row * lddz + 2 * p) = o0;
        *reinterpret_cast<u32x4 *>(dZ + row * lddz + 2 * p + 8) = o1;
    }
}

__global__ __launch_bounds__(256) void add_sumsq_kernel(const uint16_t *__restrict__ D, int64_t ldd,
                                                        const uint16_t *__restrict__ R, int64_t ldr, int64_t M, int64_t N,
                                                        uint16_t *__restrict__ Y, int64_t ldy, float *__restrict__ ss)
{
    ROW_SETUP
    float s = 0.0f;
    for (int64_t j = lane * 8; j < N; j += 512) {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(D + row * ldd + j);
        const u32x4 b = *reinterpret_cast<const u32x4 *>(R + row * ldr + j);
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x = lo(a[e]) + lo(b[e]), y = hi(a[e]) + hi(b[e]);
            s += x * x + y * y;
            o[e] = pack(x, y);
        }
        *reinterpret_cast<u32x4 *>(Y + row * ldy + j) = o;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (ss && lane == 0) ss[row] = s;
}

__global__ __launch_bounds__(256) void accumulate_kernel(const float *__restrict__ T, int64_t ldt, int64_t M, int64_t N,
                                                         float *__restrict__ G, int64_t ldg)
{
    ROW_SETUP
    for (int64_t j = lane * 4; j < N; j += 256) {
        f32x4 g = *reinterpret_cast<const f32x4 *>(G + row * ldg + j);
        g += *reinterpret_cast<const f32x4 *>(T + row * ldt + j);
        *reinterpret_cast<f32x4 *>(G + row * ldg + j) = g;
    }
}

bool al16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
coda_status tile_ok(const void *p, int64_t ld, int64_t w, int64_t ldmask)
{
    if (!p) return CODA_ERR_NULL;
    if (ld < w) return CODA_ERR_SHAPE;
    if (!al16(p) || (ld & ldmask)) return CODA_ERR_ALIGN;
    return CODA_OK;
}
coda_status done(hipError_t e) { return e == hipSuccess ? CODA_OK : CODA_ERR_LAUNCH; }
unsigned row_blocks(int64_t M) { return (unsigned)((M + 3) / 4); }

}  // namespace

#define CHECK(x) do { coda_status st_ = (x); if (st_ != CODA_OK) return st_; } while (0)

extern "C" {

coda_status coda_unfused_rmsnorm_apply(void *stream, const void *X, int64_t ldx, const float *r, const float *gamma,
                                       int64_t M, int64_t K, void *Xn, int64_t ldo)
{
    if (M < 0 || K < 0 || (K & 7)) return CODA_ERR_SHAPE;
    CHECK(tile_ok(X, ldx, K, 7)); CHECK(tile_ok(Xn, ldo, K, 7));
    if (!r) return CODA_ERR_NULL;
    if (M == 0 || K == 0) return CODA_OK;
    hipLaunchKernelGGL(rmsnorm_apply_kernel, dim3(row_blocks(M)), dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t *)X, ldx, r, gamma, M, K, (uint16_t *)Xn, ldo);
    return done(hipGetLastError());
}

coda_status coda_unfused_swiglu_fwd(void *stream, const void *Z, int64_t ldz, int64_t M, int64_t F, void *H, int64_t ldh)
{
    if (M < 0 || F < 0 || (F & 7)) return CODA_ERR_SHAPE;
    CHECK(tile_ok(Z, ldz, 2 * F, 7)); CHECK(tile_ok(H, ldh, F, 7));
    if (M == 0 || F == 0) return CODA_OK;
    hipLaunchKernelGGL(swiglu_fwd_kernel, dim3(row_blocks(M)), dim3(256), 0, (hipStream_t)stream, (const uint16_t *)Z, ldz,
                       M, F, (uint16_t *)H, ldh);
    return done(hipGetLastError());
}

coda_status coda_unfused_swiglu_bwd(void *stream, const void *dH, int64_t lddh, const void *Z, int64_t ldz, int64_t M,
                                    int64_t F, void *dZ, int64_t lddz)
{
    if (M < 0 || F < 0 || (F & 7)) return CODA_ERR_SHAPE;
    CHECK(tile_ok(dH, lddh, F, 7)); CHECK(tile_ok(Z, ldz, 2 * F, 7)); CHECK(tile_ok(dZ, lddz, 2 * F, 7));
    if (M == 0 || F == 0) return CODA_OK;
    hipLaunchKernelGGL(swiglu_bwd_kernel, dim3(row_blocks(M)), dim3(256), 0, (hipStream_t)stream, (const uint16_t *)dH,
                       lddh, (const uint16_t *)Z, ldz, M, F, (uint16_t *)dZ, lddz);
    return done(hipGetLastError());
}

coda_status coda_unfused_add_sumsq(void *stream, const void *D, int64_t ldd, const void *R, int64_t ldr, int64_t M,
                                   int64_t N, void *Y, int64_t ldy, float *ss)
{
    if (M < 0 || N < 0 || (N & 7)) return CODA_ERR_SHAPE;
    CHECK(tile_ok(D, ldd, N, 7)); CHECK(tile_ok(R, ldr, N, 7)); CHECK(tile_ok(Y, ldy, N, 7));
    if (M == 0 || N == 0) return CODA_OK;
    hipLaunchKernelGGL(add_sumsq_kernel, dim3(row_blocks(M)), dim3(256), 0, (hipStream_t)stream, (const uint16_t *)D, ldd,
                       (const uint16_t *)R, ldr, M, N, (uint16_t *)Y, ldy, ss);
    return done(hipGetLastError());
}

coda_status coda_unfused_accumulate(void *stream, const float *T, int64_t ldt, int64_t M, int64_t N, float *G, int64_t ldg)
{
    if (M < 0 || N < 0 || (N & 3)) return CODA_ERR_SHAPE;
    CHECK(tile_ok(T, ldt, N, 3)); CHECK(tile_ok(G, ldg, N, 3));
    if (M == 0 || N == 0) return CODA_OK;
    hipLaunchKernelGGL(accumulate_kernel, dim3(row_blocks(M)), dim3(256), 0, (hipStream_t)stream, T, ldt, M, N, G, ldg);
    return done(hipGetLastError());
}

}  // extern "C"
