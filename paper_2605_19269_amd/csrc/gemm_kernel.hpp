// gemm_kernel.hpp -- bf16 MFMA GEMM mainloop + epilogue program for gfx950 (MI355X).
//
// D = op(A) op(B) with fp32 accumulation in v_mfma_f32_32x32x16_bf16, followed by
// the epilogue primitives of the paper's Section 3.1 applied to the accumulators
// while they are still in registers (kernel forms: Appendix "List of Kernels",
// Kernels 2, 4, 5, 6, 10, plus the accumulating weight gradient of Theorem 1).
//
// Orientation.  The MFMA's first source takes the B-matrix fragment (indexed by
// output column n) and the second the A-matrix fragment (indexed by token row m),
// i.e. each 32x32 block is computed transposed.  The accumulator layout of the
// instruction then gives every lane ONE token row (m = lane % 32) and, in each
// group of four consecutive registers, FOUR CONSECUTIVE output columns
// (n = 8*(reg/4) + 4*(lane/32) + reg%4).  Adjacent (gate, up) column pairs
// therefore sit in adjacent registers of one lane, so the pairwise maps are pure
// register arithmetic, and a row's 32 columns of a block live in just two lanes
// (lane, lane^32), so a row reduction is in-lane adds plus one cross-half exchange.
//
// Operand staging.  Tiles are copied global -> registers -> LDS in 16-byte chunks
// exactly as they lie in memory.  An operand whose contraction index is
// contiguous in memory ("K-contiguous": A as stored [M x K], B stored [N x K]) is
// kept as [rows][BK] and fragments are read with ds_read_b128.  An operand whose
// output index is contiguous ("MN-contiguous": A stored [K x M], B stored
// [K x N]) is kept as [BK][rows] and fragments are read with the transposing
// ds_read_b64_tr_b16, which hands each lane four k-values of one column.  Both
// LDS layouts are XOR-swizzled so that neither the chunk writes nor the fragment
// reads pile onto the same banks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace coda {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

enum EpiMode : int { EPI_LINEAR = 0, EPI_SWIGLU_FWD = 1, EPI_SWIGLU_BWD = 2, EPI_ACCUM = 3 };
enum RowRedMode : int { ROWRED_NONE = 0, ROWRED_PARTIALS = 1, ROWRED_ATOMIC = 2 };

struct GemmParams {
    const uint16_t *A, *B;  // bf16 bits
    int64_t lda, ldb;       // element pitches of the matrices as stored
    int M, N, K;
    int tiles_m, tiles_n;
    // epilogue operands (null = op absent)
    const float *row_scale;              // f32[M]
    const uint16_t *add; int64_t ld_add; // bf16 [M x N]
    const float *col_scale;              // f32[N]   (side output = v * gamma)
    uint16_t *side; int64_t ld_side;     // bf16 [M x N]
    float *rowred; int rowred_mode;      // see RowRedMode; partials are [tiles_n x M]
    void *out; int64_t ld_out; int out_f32;
    const uint16_t *Z; int64_t ldz;      // SWIGLU_BWD saved pre-activation [M x 2N]
    uint16_t *out2; int64_t ld_out2;     // SWIGLU_FWD: pre-activation; SWIGLU_BWD: silu(g)*u
};

// ---------------------------------------------------------------------------------
// LDS layouts
// ---------------------------------------------------------------------------------
// K-contiguous tile [ROWS][BK]: 16-byte chunk c of row r.
template <int BK>
__device__ __forceinline__ uint32_t lds_kc(int r, int c)
{
    return (uint32_t)(r * (BK * 2) + (((c ^ (r >> 1)) & (BK / 8 - 1)) << 4));
}
// MN-contiguous tile [BK][ROWS]: 32-byte granule gr (16 elements) of k-row k.
__device__ __forceinline__ int mn_swz(int k) { return (k & 3) | ((k >> 1) & 4); }
template <int ROWS>
__device__ __forceinline__ uint32_t lds_mn(int k, int gr)
{
    return (uint32_t)(k * (ROWS * 2) + (((gr ^ mn_swz(k)) & (ROWS / 16 - 1)) << 5));
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    f32x2 v = {a, b};
    bf16x2 h = __builtin_convertvector(v, bf16x2);  // round-to-nearest-even
    return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

__device__ __forceinline__ float fast_sigmoid(float g)
{
    return __builtin_amdgcn_rcpf(1.0f + __expf(-g));
}

// ---------------------------------------------------------------------------------
// Tile -> workgroup mapping: workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2.  Give every XCD a contiguous range of tile ids and walk that
// range in column-major order inside groups of GROUP_M tile rows, so the tiles
// resident on one XCD at a time form a compact patch that re-uses A and B panels.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ void tile_coords(int bid, int nb, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int XCDS = 8, GROUP_M = 8;
    const int x = bid % XCDS, q = bid / XCDS;
    const int base = nb / XCDS, rem = nb % XCDS;
    const int id = x * base + (x < rem ? x : rem) + q;
    const int per_group = GROUP_M * tiles_n;
    const int grp = id / per_group;
    const int first_m = grp * GROUP_M;
    const int gm = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
    const int in_grp = id - grp * per_group;
    tm = first_m + in_grp % gm;
    tn = in_grp / gm;
}

// ---------------------------------------------------------------------------------
// The kernel
// ---------------------------------------------------------------------------------
template <int BM_, int BN_, int BK_, int WGM_, int WGN_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
    static constexpr int NT = WGM * WGN * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int FM = WTM / 32, FN = WTN / 32;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int CHA = BM * BK / 8 / NT, CHB = BN * BK / 8 / NT;  // 16-byte chunks per thread
    static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tiles are multiples of 32");
    static_assert(BK % 16 == 0 && (BM * BK / 8) % NT == 0 && (BN * BK / 8) % NT == 0, "chunking");
    static_assert(BM >= 128 && BN >= 128, "granule swizzle needs >= 8 granules per k-row");
};

// Global -> register loads of one operand tile (chunks laid out as in memory).
template <class C, int ROWS, int CH, bool KCONT, bool EDGE>
__device__ __forceinline__ void tile_gload(u32x4 (&r)[CH], const uint16_t *__restrict__ base, int64_t ld,
                                           int row0, int k0, int rows_total, int K, int tid)
{
#pragma unroll
    for (int it = 0; it < CH; ++it) {
        const int ci = tid + it * C::NT;
        int rr, kk;  // row (output index) and k of the chunk's first element
        if (KCONT) {
            rr = ci / (C::BK / 8);
            kk = (ci % (C::BK / 8)) * 8;
        } else {
            kk = ci / (ROWS / 8);
            rr = (ci % (ROWS / 8)) * 8;
        }
        const int gr = row0 + rr, gk = k0 + kk;
        const uint16_t *src = KCONT ? base + (int64_t)gr * ld + gk : base + (int64_t)gk * ld + gr;
        if (EDGE) {
            const bool ok = gr < rows_total && gk < K;
            u32x4 z = {0u, 0u, 0u, 0u};
            r[it] = ok ? *reinterpret_cast<const u32x4 *>(src) : z;
        } else {
            r[it] = *reinterpret_cast<const u32x4 *>(src);
        }
    }
}

// Register -> LDS stores of one operand tile.
template <class C, int ROWS, int CH, bool KCONT>
__device__ __forceinline__ void tile_lstore(const u32x4 (&r)[CH], unsigned char *tile, int tid)
{
#pragma unroll
    for (int it = 0; it < CH; ++it) {
        const int ci = tid + it * C::NT;
        uint32_t off;
        if (KCONT) {
            off = lds_kc<C::BK>(ci / (C::BK / 8), ci % (C::BK / 8));
        } else {
            const int kk = ci / (ROWS / 8), c8 = ci % (ROWS / 8);
            off = lds_mn<ROWS>(kk, c8 >> 1) + ((c8 & 1) << 4);
        }
        *reinterpret_cast<u32x4 *>(tile + off) = r[it];
    }
}

// One MFMA operand fragment (32 rows x 16 k) from an LDS tile.
//   lane l holds row (l % 32), k = 8*(l/32) .. 8*(l/32)+7 of the 16-wide k-slice `ks`.
template <class C, int ROWS, bool KCONT>
__device__ __forceinline__ bf16x8 frag_load(const unsigned char *tile, int row_base, int ks, int lane)
{
    if (KCONT) {
        const int r = row_base + (lane & 31);
        const int c = ks * 2 + (lane >> 5);
        return *reinterpret_cast<const bf16x8 *>(tile + lds_kc<C::BK>(r, c));
    } else {
        // transposing read: within each 16-lane group, lane i supplies the address of k-row
        // (i/4), columns 4*(i%4)..+3 and receives column i of those four k-rows.
        const int i = lane & 15, nh = (lane >> 4) & 1, h = lane >> 5;
        const int gr = (row_base >> 4) + nh;
        const int k_lo = ks * 16 + 8 * h + (i >> 2);
        const uint32_t sub = (uint32_t)((i & 3) << 3);
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const uint32_t o0 = lds_mn<ROWS>(k_lo, gr) + sub;
        const uint32_t o1 = lds_mn<ROWS>(k_lo + 4, gr) + sub;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + o0));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + o1));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    }
}

template <class C, bool AK, bool BKC, int EPI, bool EDGE>
__global__ __launch_bounds__(C::NT) void gemm_kernel(const GemmParams p)
{
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, FM = C::FM, FN = C::FN;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * C::STAGE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % C::WGM, wn = wave / C::WGM;
    int tm, tn;
    tile_coords(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int KT = (p.K + BK - 1) / BK;
    u32x4 ra[C::CHA], rb[C::CHB];

    if (KT > 0) {
        tile_gload<C, BM, C::CHA, AK, EDGE>(ra, p.A, p.lda, m0, 0, p.M, p.K, tid);
        tile_gload<C, BN, C::CHB, BKC, EDGE>(rb, p.B, p.ldb, n0, 0, p.N, p.K, tid);
        tile_lstore<C, BM, C::CHA, AK>(ra, smem, tid);
        tile_lstore<C, BN, C::CHB, BKC>(rb, smem + C::A_BYTES, tid);
    }
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const unsigned char *sa = smem + (kt & 1) * C::STAGE_BYTES;
        const unsigned char *sb = sa + C::A_BYTES;
        const bool more = kt + 1 < KT;
        if (more) {
            tile_gload<C, BM, C::CHA, AK, EDGE>(ra, p.A, p.lda, m0, (kt + 1) * BK, p.M, p.K, tid);
            tile_gload<C, BN, C::CHB, BKC, EDGE>(rb, p.B, p.ldb, n0, (kt + 1) * BK, p.N, p.K, tid);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[FM], fb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                fa[i] = frag_load<C, BM, AK>(sa, wm * C::WTM + i * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                fb[j] = frag_load<C, BN, BKC>(sb, wn * C::WTN + j * 32, ks, lane);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
        if (more) {
            unsigned char *da = smem + ((kt + 1) & 1) * C::STAGE_BYTES;
            tile_lstore<C, BM, C::CHA, AK>(ra, da, tid);
            tile_lstore<C, BN, C::CHB, BKC>(rb, da + C::A_BYTES, tid);
        }
        __syncthreads();
    }

    // ------------------------------------------------------------------ epilogue
    // lane -> (row, column group):  m = mb + (lane & 31);  n = nb + 8*g + 4*(lane >> 5) + e
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int mw = m0 + wm * C::WTM, nw = n0 + wn * C::WTN;
    float *red = reinterpret_cast<float *>(smem);  // [WGN][BM] row-reduction exchange
    const bool want_red = (EPI == EPI_LINEAR || EPI == EPI_SWIGLU_BWD) && p.rowred_mode != ROWRED_NONE;

#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int m = mw + i * 32 + lrow;
        const bool mok = !EDGE || m < p.M;
        float rs = 1.0f;
        if ((EPI == EPI_LINEAR || EPI == EPI_SWIGLU_FWD) && p.row_scale) rs = mok ? p.row_scale[m] : 0.0f;
        float rsum = 0.0f;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = nw + j * 32 + g * 8 + lhalf * 4;
                const bool ok = mok && (!EDGE || n < p.N);
                f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                if (EPI == EPI_LINEAR) {
                    v *= rs;
                    if (p.add && ok) {
                        u32x2 c = *reinterpret_cast<const u32x2 *>(p.add + (int64_t)m * p.ld_add + n);
                        v[0] += bf16_lo(c[0]); v[1] += bf16_hi(c[0]);
                        v[2] += bf16_lo(c[1]); v[3] += bf16_hi(c[1]);
                    }
                    if (ok) rsum += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
                    if (p.side && ok) {
                        f32x4 gm = *reinterpret_cast<const f32x4 *>(p.col_scale + n);
                        u32x2 o = {pack_bf16x2(v[0] * gm[0], v[1] * gm[1]), pack_bf16x2(v[2] * gm[2], v[3] * gm[3])};
                        *reinterpret_cast<u32x2 *>(p.side + (int64_t)m * p.ld_side + n) = o;
                    }
                    if (ok) {
                        if (p.out_f32) {
                            *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(p.out) + (int64_t)m * p.ld_out + n) = v;
                        } else {
                            u32x2 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                            *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(p.out) + (int64_t)m * p.ld_out + n) = o;
                        }
                    }
                } else if (EPI == EPI_SWIGLU_FWD) {
                    v *= rs;
                    if (ok) {
                        if (p.out2) {
                            u32x2 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                            *reinterpret_cast<u32x2 *>(p.out2 + (int64_t)m * p.ld_out2 + n) = o;
                        }
                        const float h0 = v[0] * fast_sigmoid(v[0]) * v[1];
                        const float h1 = v[2] * fast_sigmoid(v[2]) * v[3];
                        *reinterpret_cast<uint32_t *>(reinterpret_cast<uint16_t *>(p.out) + (int64_t)m * p.ld_out + (n >> 1)) =
                            pack_bf16x2(h0, h1);
                    }
                } else if (EPI == EPI_SWIGLU_BWD) {
                    if (ok) {
                        const u32x4 z = *reinterpret_cast<const u32x4 *>(p.Z + (int64_t)m * p.ldz + 2 * n);
                        u32x4 dz;
                        float o[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float gg = bf16_lo(z[e]), uu = bf16_hi(z[e]);
                            const float sg = fast_sigmoid(gg);
                            const float sl = gg * sg;
                            const float dU = v[e] * sl;
                            const float dG = v[e] * uu * (sg + sl * (1.0f - sg));
                            dz[e] = pack_bf16x2(dG, dU);
                            o[e] = sl * uu;
                            rsum += gg * dG + uu * dU;
                        }
                        *reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(p.out) + (int64_t)m * p.ld_out + 2 * n) = dz;
                        if (p.out2) {
                            u32x2 oo = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
                            *reinterpret_cast<u32x2 *>(p.out2 + (int64_t)m * p.ld_out2 + n) = oo;
                        }
                    }
                } else {  // EPI_ACCUM
                    if (ok) {
                        float *gp = reinterpret_cast<float *>(p.out) + (int64_t)m * p.ld_out + n;
                        f32x4 cur = *reinterpret_cast<const f32x4 *>(gp);
                        cur += v;
                        *reinterpret_cast<f32x4 *>(gp) = cur;
                    }
                }
            }
        }
        if (want_red) {
            rsum += __shfl_xor(rsum, 32, 64);
            if (lane < 32) red[wn * BM + wm * C::WTM + i * 32 + lane] = rsum;
        }
    }
    if (want_red) {
        __syncthreads();
        for (int r = tid; r < BM; r += C::NT) {
            const int m = m0 + r;
            if (EDGE && m >= p.M) continue;
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < C::WGN; ++w) s += red[w * BM + r];
            if (p.rowred_mode == ROWRED_PARTIALS)
                p.rowred[(int64_t)tn * p.M + m] = s;
            else
                atomicAdd(p.rowred + m, s);
        }
    }
}

// Host-side launcher, one per (operand layouts, epilogue mode, edge predication).
template <bool AK, bool BKC, int EPI, bool EDGE>
hipError_t launch_gemm(const GemmParams &p, hipStream_t stream);

}  // namespace coda
