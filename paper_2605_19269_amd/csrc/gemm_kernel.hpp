// gemm_kernel.hpp -- bf16 MFMA GEMM mainloop + epilogue program for gfx950 (MI355X).
//
// D = op(A) op(B) with fp32 accumulation on the matrix cores (v_mfma_f32_16x16x32_bf16 for bf16 operands,
// v_mfma_f32_32x32x64_f8f6f4 for 8-bit operands), followed by
// the epilogue primitives of the paper's Section 3.1 applied to the accumulators
// while they are still in registers (kernel forms: Appendix "List of Kernels",
// Kernels 1 - 10, plus the accumulating weight gradient of Theorem 1).
//
// Orientation.  The MFMA's first source takes the B-matrix fragment (indexed by
// output column n) and the second the A-matrix fragment (indexed by token row m),
// i.e. each block is computed transposed.  The accumulator layout of the
// instruction then gives every lane ONE token row per block and, in each
// group of four consecutive registers, FOUR CONSECUTIVE output columns
// (see Acc32 / Acc16 below).  Adjacent (gate, up) column pairs
// therefore sit in adjacent registers of one lane, so the pairwise maps are pure
// register arithmetic, and a row's columns of a block live in just two (four) lanes,
// so a row reduction is in-lane adds plus one (two) cross-lane exchanges.
//
// Operand staging.  Tiles are copied global -> LDS in 16-byte chunks
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
#include <type_traits>

namespace coda {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

enum EpiMode : int { EPI_LINEAR = 0, EPI_SWIGLU_FWD = 1, EPI_SWIGLU_BWD = 2, EPI_ACCUM = 3, EPI_RMSNORM_BWD = 4 };
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
    const float *rope_cos, *rope_sin;    // f32 [T x rope_half] tables (linear mode; null = no rotation)
    const int *rope_pos;                 // int32 [M]; values are clamped to [0, rope_T - 1] where they are read
    int rope_half, rope_cols;            // head_dim / 2 (multiple of 4); leading columns that are rotated
    int rope_T;                          // rows of the tables (rope_T * rope_half fits 31 bits)
    // RMSNORM_BWD: RMSNorm input C [M x N] bf16, inverse rms r[M], row statistic z[M], weight gamma[N];
    // the optional O_in tile travels in `add`, the optional C_out in `out2`
    const uint16_t *rn_c; int64_t ld_rn_c;
    const float *rn_r, *rn_z, *rn_gamma;
    float rn_zscale;                     // z = rn_z[i] * rn_zscale (1, or 1/d when rn_z holds the raw row sums)
    float *colred; int colred_mode;      // dgamma: partials [tiles_m x N] (ROWRED_PARTIALS) or atomics into f32[N]
    // log-sum-exp partials (linear mode): per column tile the row maximum and sum of exp(v - max), both [tiles_n x M];
    // target column y[M] and the selected logit z_tgt[M]
    float *lse_max, *lse_sum, *lse_tgt;
    const int *lse_y;
    // Shared tiles (tail_chunks = 0: none).  Tiles below split_from run whole, one workgroup each.  The K-steps of the
    // tail_tiles tiles from split_from on, laid end to end, are cut into tail_chunks equal contiguous ranges (see
    // locate_workgroup; tail_pieces = 2 when ranges straddle tile boundaries: then two workgroups per range): a tile is then contracted by up to ws_stride workgroups, each of which
    // leaves its fp32 partial in ws_part[(tile - split_from) * ws_stride + part] and takes a ticket from
    // ws_cnt[tile - split_from] (zeroed before the launch); the last one to arrive adds the partials up in part order and
    // runs the epilogue.
    int split_from, tail_tiles, tail_chunks, tail_pieces, ws_stride;
    float *ws_part;
    unsigned *ws_cnt;
};

// ---------------------------------------------------------------------------------
// LDS layouts
// ---------------------------------------------------------------------------------
// MN-contiguous tile [BK][ROWS]: 32-byte granule gr (16 elements) of k-row k.
// The transposing read serves 32 lanes per LDS cycle: four k-rows (k & 3) of two adjacent granules.
// XOR-ing the granule with 2*(k & 3) sends those eight 32-byte pieces to eight different bank groups.
__device__ __forceinline__ int mn_swz(int k) { return ((k & 3) << 1) | ((k >> 3) & 1); }
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
__device__ __host__ __forceinline__ void tile_coords(int bid, int nb, int tiles_m, int tiles_n, int &tm, int &tn)
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
    static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tiles are multiples of 32");
    static_assert(BM >= 128 && BN >= 128, "granule swizzle needs >= 8 granules per k-row");
};

// ---------------------------------------------------------------------------------
// Row staging through LDS (epilogue I/O).
//
// In the accumulator layout a lane owns a few bytes of 32 different rows, so direct
// global accesses touch 32 rows per instruction with 8..32 bytes each.  Instead every
// wave owns a private LDS region (a slice of the operand ring, free after the
// mainloop) holding P rows of RB bytes of its tile: bf16 tiles are moved between
// global memory and the region with row-contiguous 16-byte accesses (full cache
// lines per row), and between the region and the accumulator layout with per-lane
// units.  16-byte chunks are XOR-swizzled with the row index so that both access
// patterns sweep all LDS banks.  Only lanes of one wave touch a region and a wave's
// LDS operations execute in order, so no workgroup barrier is needed; wave_barrier()
// only keeps the compiler from reordering the phases.
// ---------------------------------------------------------------------------------
// Swizzled region layout: row r occupies RB bytes; its 16-byte chunk c is stored at chunk position
// c ^ f(r), f(r) = (r >> SH) mod NCH, with SH chosen so that 256 consecutive bytes' worth of rows see
// different f.  All address arithmetic below is split into a per-lane part (computed once) and a
// compile-time part (XOR-ed / added as immediates), so no per-access address has to stay in a register.
template <int RB>
struct Stage {
    static constexpr int NCH = RB / 16;                             // 16-byte chunks per row
    static constexpr int RPI = 64 / NCH;                            // rows covered by one wave-wide 16-byte access
    static constexpr int SH = RB >= 256 ? 0 : (RB == 128 ? 1 : 2);
    static_assert(RB == 64 || RB == 128 || RB == 256, "row sizes of the staged tiles");
    static_assert(RPI >= (1 << SH), "row-group bits and lane-row bits of f() must not overlap");

    // ---- row-contiguous phase: access `it` covers rows it*RPI .. it*RPI+RPI-1, lane -> (row lane/NCH, chunk lane%NCH)
    __device__ static __forceinline__ uint32_t row_lane(int lane)
    {
        const int lr = lane / NCH, c = lane % NCH;
        return (uint32_t)(lr * RB + ((c ^ ((lr >> SH) & (NCH - 1))) << 4));
    }
    __device__ static __forceinline__ uint32_t row_addr(uint32_t lane_part, int it)
    {
        return (uint32_t)(it * 1024) + (lane_part ^ (uint32_t)((((it * RPI) >> SH) & (NCH - 1)) << 4));
    }
    // ---- unit phase (accumulator layout with LR rows per block, 64 / LR lanes per row): lane -> row (lane % LR) of
    // LR-row block fi, a unit of U bytes at byte column cb + (lane / LR) * U
    template <int U, int LR>
    __device__ static __forceinline__ uint32_t unit_lane(int lane)
    {
        const int lrow = lane % LR, hb = (lane / LR) * U;
        const int f = (lrow >> SH) & (NCH - 1);
        return (uint32_t)(lrow * RB + ((f ^ (hb >> 4)) << 4) + (hb & 15));
    }
    // cb: compile-time byte column of the first lane's unit (a multiple of U * 64 / LR)
    template <int LR>
    __device__ static __forceinline__ uint32_t unit_addr(uint32_t lane_part, int fi, int cb)
    {
        return (uint32_t)(fi * LR * RB + (cb & 15)) + (lane_part ^ (uint32_t)((cb >> 4) << 4));
    }
};

// 16-byte global load, optionally with the non-temporal hint: for epilogue inputs that are read exactly once, so that they
// do not displace operand panels in L2.  Measured: +2 % on the SwiGLU backward (Z), +6 % on the RMSNorm backward (C, O_in);
// the residual of the down-projection (-0.5 %) and the fp32 gradient buffer (-0.6 %) keep ordinary loads.
template <bool STREAM>
__device__ __forceinline__ u32x4 load16(const unsigned char *g)
{
    if (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(g));
    return *reinterpret_cast<const u32x4 *>(g);
}

// P rows x RB bytes: global (row pitch `pitch` bytes) -> region.  rows_ok / bytes_ok bound the valid part.
template <int RB, int P, bool EDGE, bool STREAM = false>
__device__ __forceinline__ void stage_load(unsigned char *reg, const unsigned char *g, int64_t pitch, int rows_ok,
                                           int bytes_ok, int lane)
{
    using St = Stage<RB>;
    constexpr int TOTAL = P / St::RPI, BATCH = TOTAL < 8 ? TOTAL : 8;
    static_assert(P % St::RPI == 0 && TOTAL % BATCH == 0, "whole wave accesses");
    const int lr = lane / St::NCH, lc = (lane % St::NCH) * 16;
    const uint32_t goff = (uint32_t)(lr * (int)pitch + lc);        // 32-bit lane offset; rows advance via the scalar base
    const uint32_t loff = St::row_lane(lane);
#pragma unroll
    for (int b = 0; b < TOTAL / BATCH; ++b) {
        u32x4 t[BATCH];
#pragma unroll
        for (int q = 0; q < BATCH; ++q) {
            const int it = b * BATCH + q;
            const unsigned char *gi = g + (int64_t)(it * St::RPI) * pitch;
            const u32x4 z = {0u, 0u, 0u, 0u};
            const bool ok = !EDGE || (it * St::RPI + lr < rows_ok && lc < bytes_ok);
            t[q] = ok ? load16<STREAM>(gi + goff) : z;
        }
#pragma unroll
        for (int q = 0; q < BATCH; ++q)
            *reinterpret_cast<u32x4 *>(reg + St::row_addr(loff, b * BATCH + q)) = t[q];
        __builtin_amdgcn_sched_barrier(0);   // keep at most one batch of loads live
    }
}

// P rows x RB bytes: region -> global.  STREAM: stores carry the non-temporal hint (the output is not read again by this
// kernel and should not displace operand panels in L2).  Measured on the benchmark shapes: +2.5 % on the down-projection,
// +2 to +6 % on the QKV kernels; the SwiGLU forward (no gain, half-line rows) and the SwiGLU backward, whose 268 MB output
// leaves in chip-wide bursts (-2.4 % with the hint), keep ordinary stores.
template <int RB, int P, bool EDGE, bool STREAM = true>
__device__ __forceinline__ void stage_store(const unsigned char *reg, unsigned char *g, int64_t pitch, int rows_ok,
                                            int bytes_ok, int lane)
{
    auto put16 = [](unsigned char *dst, u32x4 v) {
        if (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(dst));
        else *reinterpret_cast<u32x4 *>(dst) = v;
    };
    using St = Stage<RB>;
    constexpr int TOTAL = P / St::RPI;
    const int lr = lane / St::NCH, lc = (lane % St::NCH) * 16;
    const uint32_t goff = (uint32_t)(lr * (int)pitch + lc);
    const uint32_t loff = St::row_lane(lane);
#pragma unroll
    for (int it = 0; it < TOTAL; ++it) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(reg + St::row_addr(loff, it));
        unsigned char *gi = g + (int64_t)(it * St::RPI) * pitch;
        if (!EDGE) {
            put16(gi + goff, v);
        } else if (it * St::RPI + lr < rows_ok) {
            // valid widths are multiples of 8 bytes (halved widths of the pairwise forward), so the last chunk may be half
            if (lc + 16 <= bytes_ok) put16(gi + goff, v);
            else if (lc < bytes_ok) *reinterpret_cast<u32x2 *>(gi + goff) = u32x2{v[0], v[1]};
        }
        if ((it & 3) == 3) __builtin_amdgcn_sched_barrier(0);
    }
}

// Split form of stage_load: global -> registers now, registers -> region later, so the loads of the next pass can be
// in flight while the current pass is processed.  t holds P / RPI chunks per lane.
template <int RB, int P, bool EDGE, bool STREAM = false>
__device__ __forceinline__ void stage_fetch(u32x4 (&t)[P / Stage<RB>::RPI], const unsigned char *g, int64_t pitch, int rows_ok,
                                            int bytes_ok, int lane)
{
    using St = Stage<RB>;
    const int lr = lane / St::NCH, lc = (lane % St::NCH) * 16;
    const uint32_t goff = (uint32_t)(lr * (int)pitch + lc);
#pragma unroll
    for (int it = 0; it < P / St::RPI; ++it) {
        const unsigned char *gi = g + (int64_t)(it * St::RPI) * pitch;
        const u32x4 z = {0u, 0u, 0u, 0u};
        const bool ok = !EDGE || (it * St::RPI + lr < rows_ok && lc < bytes_ok);
        t[it] = ok ? load16<STREAM>(gi + goff) : z;
    }
}
template <int RB, int P>
__device__ __forceinline__ void stage_put(unsigned char *reg, const u32x4 (&t)[P / Stage<RB>::RPI], int lane)
{
    using St = Stage<RB>;
    const uint32_t loff = St::row_lane(lane);
#pragma unroll
    for (int it = 0; it < P / St::RPI; ++it) *reinterpret_cast<u32x4 *>(reg + St::row_addr(loff, it)) = t[it];
}

// Phase boundary inside a wave: no instruction may be moved across it.
__device__ __forceinline__ void stage_fence()
{
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

// RoPE on the two adjacent pairs held in one unit (columns n..n+3): pair frequencies f and f+1 of position row `trow`.
__device__ __forceinline__ void rope_unit(f32x4 &v, const GemmParams &p, int64_t trow, int f)
{
    const f32x2 c = *reinterpret_cast<const f32x2 *>(p.rope_cos + trow + f);
    const f32x2 s = *reinterpret_cast<const f32x2 *>(p.rope_sin + trow + f);
    const float a0 = v[0] * c[0] - v[1] * s[0], a1 = v[0] * s[0] + v[1] * c[0];
    const float b0 = v[2] * c[1] - v[3] * s[1], b1 = v[2] * s[1] + v[3] * c[1];
    v = f32x4{a0, a1, b0, b1};
}

constexpr int pass_rows(int reg_bytes, int row_bytes, int max_rows)
{
    int p = 32;
    while (p * 2 <= max_rows && p * 2 * row_bytes <= reg_bytes) p *= 2;
    return p;
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// ---------------------------------------------------------------------------------
// Accumulators of one wave's WTM x WTN tile, in the layout of the MFMA that produced them.
// Both instructions are issued with the B fragment as first source, so a lane owns ONE token row per block and
// groups of four consecutive output columns ("units").  With LR rows per block and LQ = 64 / LR lanes per row:
//   row of block i:   i * LR + lane % LR
//   unit u of a row:  columns u * 4 * LQ + 4 * (lane / LR) .. + 3
// Acc32: v_mfma_f32_32x32x64_f8f6f4 and the 32x32 bf16 shapes (LR 32, 2 lanes per row, 4 units per 32x32 block);
// Acc16: v_mfma_f32_16x16x32_bf16 (LR 16, 4 lanes per row, one unit per 16x16 block).
// ---------------------------------------------------------------------------------
template <class C>
struct Acc32 {
    static constexpr int LR = 32, LQ = 2, NB = C::WTM / 32, NU = C::WTN / 8;
    f32x16 a[C::WTM / 32][C::WTN / 32];
    __device__ __forceinline__ f32x4 get(int i, int u) const
    {
        const f32x16 &b = a[i][u >> 2];
        const int g = (u & 3) * 4;
        return f32x4{b[g], b[g + 1], b[g + 2], b[g + 3]};
    }
    __device__ __forceinline__ void set(int i, int u, f32x4 v)
    {
        f32x16 &b = a[i][u >> 2];
        const int g = (u & 3) * 4;
        b[g] = v[0]; b[g + 1] = v[1]; b[g + 2] = v[2]; b[g + 3] = v[3];
    }
};
template <class C>
struct Acc16 {
    static constexpr int LR = 16, LQ = 4, NB = C::WTM / 16, NU = C::WTN / 16;
    f32x4 a[C::WTM / 16][C::WTN / 16];
    __device__ __forceinline__ f32x4 get(int i, int u) const { return a[i][u]; }
    __device__ __forceinline__ void set(int i, int u, f32x4 v) { a[i][u] = v; }
};
template <class ACC>
__device__ __forceinline__ void acc_zero(ACC &acc)
{
#pragma unroll
    for (int i = 0; i < ACC::NB; ++i)
#pragma unroll
        for (int u = 0; u < ACC::NU; ++u) acc.set(i, u, f32x4{0.f, 0.f, 0.f, 0.f});
}

// Sum over the LQ lanes that share a row (lanes lane % LR + k * LR).
template <int LR>
__device__ __forceinline__ float row_lanes_sum(float v)
{
#pragma unroll
    for (int off = LR; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---------------------------------------------------------------------------------
// Epilogue program on the accumulators of one workgroup tile (layout: see Acc32 / Acc16).
// `ring` (RING bytes, 1 KiB aligned) must no longer be read by any wave as an operand
// tile (callers synchronise); `red` is a separate [2][WGN][BM] float exchange buffer.
// ---------------------------------------------------------------------------------
template <class C, class ACC, int EPI, bool EDGE, int RING>
__device__ __forceinline__ void run_epilogue(ACC &acc, const GemmParams &p, int m0, int n0, int tn,
                                             unsigned char *ring, float *red, int tid)
{
    constexpr int BM = C::BM, WTM = C::WTM, WTN = C::WTN;
    constexpr int LR = ACC::LR, LQ = ACC::LQ, NB = ACC::NB, NU = ACC::NU, UC = 4 * LQ;   // UC: column step between units
    constexpr int REG = RING / (C::WGM * C::WGN);   // private staging bytes per wave
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % C::WGM, wn = wave / C::WGM;
    const int lrow = lane % LR, lcol = (lane / LR) * 4;           // the lane's row in a block, first column in a unit step
    const int mw = m0 + wm * WTM, nw = n0 + wn * WTN;
    unsigned char *reg = ring + wave * REG;
    const int rows_ok = EDGE ? clampi(p.M - mw, 0, WTM) : WTM;   // valid rows / columns of this wave's tile
    const int cols_ok = EDGE ? clampi(p.N - nw, 0, WTN) : WTN;
    const bool want_red = (EPI == EPI_LINEAR || EPI == EPI_SWIGLU_BWD) && p.rowred_mode != ROWRED_NONE;
    float rsum[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) rsum[i] = 0.0f;
    // Row scales of the lane's NB rows, all fetched in one go at the head of the program branch that uses them: a load
    // per block inside the passes would sit behind that pass's stores and expose one memory round trip per block.
    // (Fetched per branch, not once up here, so that they are not live across the other branches' code.)
    auto fetch_row_scales = [&](float(&rsv)[NB]) {
#pragma unroll
        for (int i = 0; i < NB; ++i) rsv[i] = 1.0f;
        if (p.row_scale) {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int m = mw + i * LR + lrow;
                rsv[i] = (!EDGE || m < p.M) ? p.row_scale[m] : 0.0f;
            }
        }
    };

    if (EPI == EPI_LINEAR && p.lse_max) {
        // ---- log-sum-exp partials of this 256-column tile (Kernels 3 / 8) on the fp32 values v = acc * r, before rounding:
        // per lane and row the maximum and the sum of exp(v - max) over its values, merged over the lanes that share the
        // row and then over the four column waves with the usual rescaling rule.
        constexpr float NEG_INF = -__builtin_inff();
        float rsv[NB];
        fetch_row_scales(rsv);
        int yv[NB];                                                 // target columns of the lane's rows, fetched in one go
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int m = mw + i * LR + lrow;
            yv[i] = (!EDGE || m < p.M) ? p.lse_y[m] : -1;
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int m = mw + i * LR + lrow;
            const bool mok = !EDGE || m < p.M;
            const float rs = rsv[i];
            const int yy = yv[i];
            // row maximum of v = a * rs without scaling every element: the extreme of the raw accumulators in the direction of
            // rs's sign, scaled once (a monotone map of the same fp32 products, so it is the maximum of the rounded v exactly)
            float hi = NEG_INF, lo = -NEG_INF;
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int n = nw + u * UC + lcol;
                if (mok && (!EDGE || n < p.N)) {
                    const f32x4 a = acc.get(i, u);
                    hi = fmaxf(fmaxf(hi, fmaxf(a[0], a[1])), fmaxf(a[2], a[3]));
                    lo = fminf(fminf(lo, fminf(a[0], a[1])), fminf(a[2], a[3]));
                }
            }
            float mx = rs >= 0.0f ? hi * rs : lo * rs;
            if (hi == NEG_INF) mx = NEG_INF;                          // no valid column in this lane's part of the row
            // maximum over the wave's 64 columns of the row first (the lanes that share the row exchange it), so that all
            // of them take their exponentials against the same reference and the sums simply add up
#pragma unroll
            for (int off = LR; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
            // the target logit: at most one unit of the wave's 64 columns holds column y[i]
            {
                const unsigned e0 = (unsigned)(yy - (nw + lcol));      // distance from the lane's first column
                if (mok && e0 < (unsigned)WTN && (e0 & (UC - 1)) < 4u && (!EDGE || yy < p.N)) {
#pragma unroll
                    for (int u = 0; u < NU; ++u)
                        if ((int)(e0 / UC) == u) {
                            const f32x4 a = acc.get(i, u) * rs;
                            const unsigned e = e0 & 3u;
                            p.lse_tgt[m] = e == 0 ? a[0] : (e == 1 ? a[1] : (e == 2 ? a[2] : a[3]));
                        }
                }
            }
            // exp(a * rs - mx) as one multiply-add and one base-2 exponential per element
            constexpr float LOG2E = 1.4426950408889634f;
            const float c2 = rs * LOG2E, d2 = -mx * LOG2E;
            float sm = 0.0f;
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int n = nw + u * UC + lcol;
                if (mok && (!EDGE || n < p.N)) {
                    const f32x4 a = acc.get(i, u);
#pragma unroll
                    for (int e = 0; e < 4; ++e) sm += __builtin_amdgcn_exp2f(__builtin_fmaf(a[e], c2, d2));
                }
            }
            sm = row_lanes_sum<LR>(sm);
            if (lane < LR) {
                red[wn * BM + wm * WTM + i * LR + lane] = mx;
                red[C::WGN * BM + wn * BM + wm * WTM + i * LR + lane] = sm;
            }
        }
        __syncthreads();
        for (int r = tid; r < BM; r += C::NT) {
            const int m = m0 + r;
            if (EDGE && m >= p.M) continue;
            float mm = NEG_INF;
#pragma unroll
            for (int w = 0; w < C::WGN; ++w) mm = fmaxf(mm, red[w * BM + r]);
            float ss = 0.0f;
#pragma unroll
            for (int w = 0; w < C::WGN; ++w) {
                const float mw_ = red[w * BM + r];
                if (mw_ != NEG_INF) ss += red[C::WGN * BM + w * BM + r] * __expf(mw_ - mm);
            }
            p.lse_max[(int64_t)tn * p.M + m] = mm;
            p.lse_sum[(int64_t)tn * p.M + m] = ss;
        }
        __syncthreads();   // `red` is reused by the row-reduction exchange below
    }

    if constexpr (EPI == EPI_RMSNORM_BWD) {
        // ---- local part of RMSNorm backward: with d the accumulator, cn = C*r:
        //   O_out = O_in + (d*gamma - cn*z)*r,   C_out = cn*gamma,   dgamma partial = column sums of d*cn over this tile.
        // Per 64-row pass the region holds the C rows and the O_in rows side by side; results overwrite them in place.
        constexpr int RB = WTN * 2, P = 64, FPP = P / LR;
        static_assert(WTN == 64 && WTM % P == 0 && 2 * P * RB <= REG, "staging pass");
        static_assert((C::WGM * C::BN + C::WGM * C::WGN * WTN) * 4 <= 2 * C::WGN * C::BM * 4, "gamma strips fit behind the column sums in `red`");
        using St = Stage<RB>;
        const uint32_t ulane = St::template unit_lane<8, LR>(lane);
        unsigned char *rego = reg + P * RB;
        uint16_t *outp = reinterpret_cast<uint16_t *>(p.out);
        f32x4 dg[NU];
#pragma unroll
        for (int u = 0; u < NU; ++u) dg[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        // the wave's 64 gamma values wait in LDS (a private 256-byte strip of `red` behind the part the column reduction
        // uses) instead of in 16 registers that would have to live across both passes
        float *gstrip = red + C::WGM * C::BN + wave * WTN;
        {
            const int n = nw + lane;
            gstrip[lane] = (!EDGE || n < p.N) ? p.rn_gamma[n] : 0.0f;
        }
#pragma unroll
        for (int ps = 0; ps < WTM / P; ++ps) {
            const int r0 = ps * P;
            // the pass's row factors first, so that they travel with the tile loads instead of waiting, block by block,
            // behind the previous pass's stores
            float rrv[FPP], zzv[FPP];
#pragma unroll
            for (int fi = 0; fi < FPP; ++fi) {
                const int m = mw + (ps * FPP + fi) * LR + lrow;
                const bool mok = !EDGE || m < p.M;
                rrv[fi] = mok ? p.rn_r[m] : 0.0f;
                zzv[fi] = mok ? p.rn_z[m] * p.rn_zscale : 0.0f;
            }
            stage_load<RB, P, EDGE, true>(reg, reinterpret_cast<const unsigned char *>(p.rn_c + (int64_t)(mw + r0) * p.ld_rn_c + nw),
                                    p.ld_rn_c * 2, rows_ok - r0, cols_ok * 2, lane);
            if (p.add)
                stage_load<RB, P, EDGE, true>(rego, reinterpret_cast<const unsigned char *>(p.add + (int64_t)(mw + r0) * p.ld_add + nw),
                                        p.ld_add * 2, rows_ok - r0, cols_ok * 2, lane);
            stage_fence();
#pragma unroll
            for (int fi = 0; fi < FPP; ++fi) {
                const int i = ps * FPP + fi, m = mw + i * LR + lrow;
                const bool mok = !EDGE || m < p.M;
                const float rr = rrv[fi], zz = zzv[fi];
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const int nl = u * UC + lcol;
                    const bool ok = mok && (!EDGE || nw + nl < p.N);
                    const uint32_t ua = St::template unit_addr<LR>(ulane, fi, u * UC * 2);
                    const f32x4 gm = *reinterpret_cast<const f32x4 *>(gstrip + nl);
                    const u32x2 cw = *reinterpret_cast<const u32x2 *>(reg + ua);
                    const f32x4 d = acc.get(i, u);
                    const f32x4 cn = f32x4{bf16_lo(cw[0]), bf16_hi(cw[0]), bf16_lo(cw[1]), bf16_hi(cw[1])} * rr;
                    f32x4 o = (d * gm - cn * zz) * rr;
                    if (p.add) {
                        const u32x2 ow = *reinterpret_cast<const u32x2 *>(rego + ua);
                        o += f32x4{bf16_lo(ow[0]), bf16_hi(ow[0]), bf16_lo(ow[1]), bf16_hi(ow[1])};
                    }
                    if (ok) dg[u] += d * cn;
                    // pin the column sums here: otherwise their multiply-add chains are sunk to the point of use behind the
                    // last pass and every cn of the tile has to stay live (spilled) until then
                    asm volatile("" : "+v"(dg[u]));
                    const f32x4 co = cn * gm;
                    *reinterpret_cast<u32x2 *>(rego + ua) = u32x2{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
                    *reinterpret_cast<u32x2 *>(reg + ua) = u32x2{pack_bf16x2(co[0], co[1]), pack_bf16x2(co[2], co[3])};
                    if ((u & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                }
            }
            stage_fence();
            stage_store<RB, P, EDGE>(rego, reinterpret_cast<unsigned char *>(outp + (int64_t)(mw + r0) * p.ld_out + nw), p.ld_out * 2,
                                     rows_ok - r0, cols_ok * 2, lane);
            if (p.out2)
                stage_store<RB, P, EDGE>(reg, reinterpret_cast<unsigned char *>(p.out2 + (int64_t)(mw + r0) * p.ld_out2 + nw),
                                         p.ld_out2 * 2, rows_ok - r0, cols_ok * 2, lane);
            stage_fence();
        }
        if (p.colred_mode != ROWRED_NONE) {
            // column reduction: the lane's partial sums go to the region as an [LR rows][64 columns] f32 tile, lane l
            // then adds up column l over the LR rows; the two row-waves of the workgroup meet in `red`
            using Sf = Stage<256>;
            const uint32_t fl = Sf::template unit_lane<16, LR>(lane);
#pragma unroll
            for (int u = 0; u < NU; ++u) *reinterpret_cast<f32x4 *>(reg + Sf::template unit_addr<LR>(fl, 0, u * UC * 4)) = dg[u];
            stage_fence();
            float cs = 0.0f;
#pragma unroll
            for (int rr = 0; rr < LR; ++rr)
                cs += *reinterpret_cast<const float *>(reg + rr * 256 + ((((lane >> 2) ^ rr) & 15) << 4) + (lane & 3) * 4);
            red[wm * C::BN + wn * WTN + lane] = cs;
            __syncthreads();
            for (int c = tid; c < C::BN; c += C::NT) {
                const int n = n0 + c;
                if (EDGE && n >= p.N) continue;
                float t = 0.0f;
#pragma unroll
                for (int w = 0; w < C::WGM; ++w) t += red[w * C::BN + c];
                const int tm_idx = m0 / BM;
                if (p.colred_mode == ROWRED_PARTIALS)
                    p.colred[(int64_t)tm_idx * p.N + n] = t;
                else
                    atomicAdd(p.colred + n, t);
            }
        }
    } else if constexpr (EPI == EPI_SWIGLU_FWD) {
        // ---- row scale, pairwise SwiGLU (width halves), optional pre-activation side output
        constexpr int RBH = WTN, RBZ = WTN * 2;
        constexpr int P = pass_rows(REG, RBZ, WTM), FPP = P / LR;
        static_assert(P % LR == 0 && WTM % P == 0, "staging pass");
        uint16_t *outp = reinterpret_cast<uint16_t *>(p.out);
        const uint32_t ulane_h = Stage<RBH>::template unit_lane<4, LR>(lane), ulane_z = Stage<RBZ>::template unit_lane<8, LR>(lane);
        float rsv[NB];
        fetch_row_scales(rsv);
#pragma unroll
        for (int ps = 0; ps < WTM / P; ++ps) {
            const int r0 = ps * P;
#pragma unroll
            for (int fi = 0; fi < FPP; ++fi) {
                const int i = ps * FPP + fi;
                const float rs = rsv[i];
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const f32x4 v = acc.get(i, u) * rs;
                    const float h0 = v[0] * fast_sigmoid(v[0]) * v[1], h1 = v[2] * fast_sigmoid(v[2]) * v[3];
                    *reinterpret_cast<uint32_t *>(reg + Stage<RBH>::template unit_addr<LR>(ulane_h, fi, u * UC)) = pack_bf16x2(h0, h1);
                    if ((u & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                }
            }
            stage_fence();
            // ordinary stores: a wave's H rows are 64-byte halves of 128-byte lines, which L2 merges with the neighbouring
            // wave's halves; with the streaming hint the L2 -> fabric write counter reads 10 % above the output bytes
            stage_store<RBH, P, EDGE, false>(reg, reinterpret_cast<unsigned char *>(outp + (int64_t)(mw + r0) * p.ld_out + (nw >> 1)),
                                      p.ld_out * 2, rows_ok - r0, cols_ok, lane);
            if (p.out2) {
                stage_fence();
#pragma unroll
                for (int fi = 0; fi < FPP; ++fi) {
                    const int i = ps * FPP + fi;
                    const float rs = rsv[i];
#pragma unroll
                    for (int u = 0; u < NU; ++u) {
                        const f32x4 v = acc.get(i, u) * rs;
                        *reinterpret_cast<u32x2 *>(reg + Stage<RBZ>::template unit_addr<LR>(ulane_z, fi, u * UC * 2)) =
                            u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                    }
                }
                stage_fence();
                stage_store<RBZ, P, EDGE>(reg, reinterpret_cast<unsigned char *>(p.out2 + (int64_t)(mw + r0) * p.ld_out2 + nw),
                                          p.ld_out2 * 2, rows_ok - r0, cols_ok * 2, lane);
            }
            stage_fence();
        }
    } else if constexpr (EPI == EPI_SWIGLU_BWD) {
        // ---- pairwise SwiGLU backward (width doubles): Z in and dZ out staged; row statistic; the optional
        // recomputed activation silu(g)*u is a second sweep over 32-row passes that re-reads Z.
        constexpr int RB = WTN * 4, RBO = WTN * 2, P = 32, FPP = P / LR, NP = WTM / P;
        static_assert(P * (RB + RBO) <= REG && WTM % P == 0, "staging pass");
        uint16_t *outp = reinterpret_cast<uint16_t *>(p.out);
        const uint32_t ulane = Stage<RB>::template unit_lane<16, LR>(lane), ulane_o = Stage<RBO>::template unit_lane<8, LR>(lane);
        // 32-row passes; the Z rows of the next pass are fetched into registers while this pass is computed and stored
        u32x4 zt[P / Stage<RB>::RPI];
        auto zrows = [&](int ps) { return reinterpret_cast<const unsigned char *>(p.Z + (int64_t)(mw + ps * P) * p.ldz + 2 * nw); };
        stage_fetch<RB, P, EDGE, true>(zt, zrows(0), p.ldz * 2, rows_ok, cols_ok * 4, lane);
#pragma unroll
        for (int ps = 0; ps < NP; ++ps) {
            stage_put<RB, P>(reg, zt, lane);
            stage_fence();
            if (ps + 1 < NP) stage_fetch<RB, P, EDGE, true>(zt, zrows(ps + 1), p.ldz * 2, rows_ok - (ps + 1) * P, cols_ok * 4, lane);
            stage_fence();
#pragma unroll
            for (int fi = 0; fi < FPP; ++fi) {
                const int i = ps * FPP + fi, m = mw + i * LR + lrow;
                const bool mok = !EDGE || m < p.M;
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const bool ok = mok && (!EDGE || nw + u * UC + lcol < p.N);
                    u32x4 *slot = reinterpret_cast<u32x4 *>(reg + Stage<RB>::template unit_addr<LR>(ulane, fi, u * UC * 4));
                    const u32x4 z = *slot;
                    const f32x4 a = acc.get(i, u);
                    u32x4 dz;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float d = a[e];
                        const float gg = bf16_lo(z[e]), uu = bf16_hi(z[e]);
                        const float sg = fast_sigmoid(gg), sl = gg * sg;
                        const float dU = d * sl, dG = d * uu * (sg + sl * (1.0f - sg));
                        dz[e] = pack_bf16x2(dG, dU);
                        if (want_red && ok) rsum[i] += gg * dG + uu * dU;
                    }
                    *slot = dz;
                    asm volatile("" : "+v"(rsum[i]));   // keep the row statistic's add chain in place
                    if (u & 1) __builtin_amdgcn_sched_barrier(0);
                }
            }
            stage_fence();
            stage_store<RB, P, EDGE, false>(reg, reinterpret_cast<unsigned char *>(outp + (int64_t)(mw + ps * P) * p.ld_out + 2 * nw), p.ld_out * 2,
                                     rows_ok - ps * P, cols_ok * 4, lane);
            stage_fence();
        }
        if (p.out2) {
            unsigned char *rego = reg + P * RB;   // activation rows live behind the staged Z rows
#pragma unroll
            for (int ps = 0; ps < NP; ++ps) {
                const int r0 = ps * P;
                stage_load<RB, P, EDGE>(reg, reinterpret_cast<const unsigned char *>(p.Z + (int64_t)(mw + r0) * p.ldz + 2 * nw),
                                        p.ldz * 2, rows_ok - r0, cols_ok * 4, lane);
                stage_fence();
#pragma unroll
                for (int fi = 0; fi < FPP; ++fi)
#pragma unroll
                    for (int u = 0; u < NU; ++u) {
                        const u32x4 z = *reinterpret_cast<const u32x4 *>(reg + Stage<RB>::template unit_addr<LR>(ulane, fi, u * UC * 4));
                        float o[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float gg = bf16_lo(z[e]);
                            o[e] = gg * fast_sigmoid(gg) * bf16_hi(z[e]);
                        }
                        *reinterpret_cast<u32x2 *>(rego + Stage<RBO>::template unit_addr<LR>(ulane_o, fi, u * UC * 2)) =
                            u32x2{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
                    }
                stage_fence();
                stage_store<RBO, P, EDGE, false>(rego, reinterpret_cast<unsigned char *>(p.out2 + (int64_t)(mw + r0) * p.ld_out2 + nw),
                                          p.ld_out2 * 2, rows_ok - r0, cols_ok * 2, lane);
                stage_fence();
            }
        }
    } else if (EPI == EPI_LINEAR && !p.out_f32 && p.rope_cos && WTN == 64 && (p.rope_half & 31) == 0) {
        // ---- row scale, RoPE, bf16 store with the cos / sin rows staged like tiles: per 32-row pass the wave gathers
        // each token's 32 table entries (128 bytes of cos, 128 of sin; the wave's 64 columns are 32 consecutive pairs
        // inside one head because head_dim/2 is a multiple of 32) with row-contiguous 16-byte loads into its region,
        // so the per-unit table reads come from LDS instead of 8-byte gathers from 32 different rows.
        constexpr int RB = 128, P = 32, FPP = P / LR, NP = WTM / P;
        using St = Stage<RB>;
        const uint32_t ulane = St::template unit_lane<8, LR>(lane);
        const uint32_t rlane = St::row_lane(lane);
        const int f0 = (nw >> 1) % p.rope_half;                        // first frequency index of this wave's columns
        float rsv[NB];
        fetch_row_scales(rsv);
        unsigned char *rcos = reg + P * RB, *rsin = reg + 2 * P * RB;
        uint16_t *outp = reinterpret_cast<uint16_t *>(p.out);
        u32x4 tc[4], ts[4];
        auto gather = [&](int ps) {                                    // table slices of 32-row pass ps -> registers
            const int m = mw + ps * P + (lane & 31);
            const int trow = (!EDGE || m < p.M) ? clampi(p.rope_pos[m], 0, p.rope_T - 1) * p.rope_half + f0 : f0;
#pragma unroll
            for (int it = 0; it < 4; ++it) {                           // 8 rows x 128 bytes per access
                const int src = __shfl(trow, it * 8 + (lane >> 3), 64) + (lane & 7) * 4;
                tc[it] = *reinterpret_cast<const u32x4 *>(p.rope_cos + src);
                ts[it] = *reinterpret_cast<const u32x4 *>(p.rope_sin + src);
            }
        };
        gather(0);
#pragma unroll
        for (int ps = 0; ps < NP; ++ps) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                *reinterpret_cast<u32x4 *>(rcos + St::row_addr(rlane, it)) = tc[it];
                *reinterpret_cast<u32x4 *>(rsin + St::row_addr(rlane, it)) = ts[it];
            }
            stage_fence();
            if (ps + 1 < NP) gather(ps + 1);                           // in flight under this pass's math and stores
            stage_fence();
#pragma unroll
            for (int fi = 0; fi < FPP; ++fi) {
                const int i = ps * FPP + fi;
                const float rs = rsv[i];
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const int nl = u * UC + lcol;
                    const uint32_t ua = St::template unit_addr<LR>(ulane, fi, u * UC * 2);
                    f32x4 v = acc.get(i, u) * rs;
                    if (nw + nl < p.rope_cols) {
                        const f32x2 c = *reinterpret_cast<const f32x2 *>(rcos + ua);
                        const f32x2 sn = *reinterpret_cast<const f32x2 *>(rsin + ua);
                        v = f32x4{v[0] * c[0] - v[1] * sn[0], v[0] * sn[0] + v[1] * c[0],
                                  v[2] * c[1] - v[3] * sn[1], v[2] * sn[1] + v[3] * c[1]};
                    }
                    *reinterpret_cast<u32x2 *>(reg + ua) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                }
            }
            stage_fence();
            stage_store<RB, P, EDGE>(reg, reinterpret_cast<unsigned char *>(outp + (int64_t)(mw + ps * P) * p.ld_out + nw), p.ld_out * 2,
                                     rows_ok - ps * P, cols_ok * 2, lane);
            stage_fence();
        }
    } else if (EPI == EPI_LINEAR && !p.out_f32) {
        // ---- row scale, residual add, row sum of squares, bf16 store: all tile I/O staged.  The gamma-scaled side
        // output (when requested) is a second sweep that re-reads the residual and recomputes the value, so that
        // nothing has to stay in registers between the two stores.
        constexpr int RB = WTN * 2, P = pass_rows(REG, RB, WTM), FPP = P / LR;
        static_assert(P % LR == 0 && WTM % P == 0, "staging pass");
        const uint32_t ulane = Stage<RB>::template unit_lane<8, LR>(lane);
        const int sweeps = p.side ? 2 : 1;
        for (int sw = 0; sw < sweeps; ++sw) {
            uint16_t *dst = sw == 0 ? reinterpret_cast<uint16_t *>(p.out) : p.side;
            const int64_t ldd = sw == 0 ? p.ld_out : p.ld_side;
            float rsv[NB];
            fetch_row_scales(rsv);
#pragma unroll
            for (int ps = 0; ps < WTM / P; ++ps) {
                const int r0 = ps * P;
                if (p.add) {
                    stage_load<RB, P, EDGE>(reg, reinterpret_cast<const unsigned char *>(p.add + (int64_t)(mw + r0) * p.ld_add + nw),
                                            p.ld_add * 2, rows_ok - r0, cols_ok * 2, lane);
                    stage_fence();
                }
#pragma unroll
                for (int fi = 0; fi < FPP; ++fi) {
                    const int i = ps * FPP + fi, m = mw + i * LR + lrow;
                    const bool mok = !EDGE || m < p.M;
                    const float rs = rsv[i];
                    // RoPE: table row of this token and the frequency index of the lane's first pair; units follow each
                    // other UC / 2 <= 8 pairs apart and rope_half is a multiple of 4, so the index wraps at most twice per step
                    const int64_t trow = (p.rope_cos && mok) ? (int64_t)clampi(p.rope_pos[m], 0, p.rope_T - 1) * p.rope_half : 0;
                    int rf = p.rope_cos ? ((nw + lcol) >> 1) % p.rope_half : 0;
#pragma unroll
                    for (int u = 0; u < NU; ++u) {
                        const int nl = u * UC + lcol;
                        const bool ok = mok && (!EDGE || nw + nl < p.N);
                        f32x4 v = acc.get(i, u) * rs;
                        if (p.rope_cos) {
                            if (ok && nw + nl < p.rope_cols) rope_unit(v, p, trow, rf);
                            rf += UC / 2;
                            if (rf >= p.rope_half) rf -= p.rope_half;
                            if (rf >= p.rope_half) rf -= p.rope_half;
                        }
                        u32x2 *slot = reinterpret_cast<u32x2 *>(reg + Stage<RB>::template unit_addr<LR>(ulane, fi, u * UC * 2));
                        if (p.add) {
                            const u32x2 c = *slot;
                            v[0] += bf16_lo(c[0]); v[1] += bf16_hi(c[0]);
                            v[2] += bf16_lo(c[1]); v[3] += bf16_hi(c[1]);
                        }
                        if (sw == 0) {
                            if (ok) rsum[i] += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
                        } else {
                            f32x4 gm = {0.f, 0.f, 0.f, 0.f};
                            if (ok) gm = *reinterpret_cast<const f32x4 *>(p.col_scale + nw + nl);
                            v *= gm;
                        }
                        *slot = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                        if ((u & 3) == 3) {
                            // pin the running row sum here: otherwise its whole add chain is sunk to the point of
                            // use after the stores and every addend has to stay live (spilled) until then
                            asm volatile("" : "+v"(rsum[i]));
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
                stage_fence();
                stage_store<RB, P, EDGE>(reg, reinterpret_cast<unsigned char *>(dst + (int64_t)(mw + r0) * ldd + nw), ldd * 2,
                                         rows_ok - r0, cols_ok * 2, lane);
                stage_fence();
            }
        }
    } else if constexpr (EPI == EPI_ACCUM) {
        // ---- in-place fp32 accumulate: 16 bytes per lane, direct.  Loads and stores go through the same pointer, so the
        // compiler cannot move a load above an earlier store on its own, and unit by unit only a handful of loads would
        // be in flight per wave.  The units are walked in batches of QB with the loads of the next batch issued ahead of
        // the adds and stores of the current one (two register buffers).
        constexpr int NQ = NB * NU, QB = 8, NBATCH = NQ / QB;
        static_assert(NQ % QB == 0, "whole batches");
        float *outp = reinterpret_cast<float *>(p.out);
        f32x4 buf[2][QB];
        auto where = [&](int q, bool &ok) -> float * {
            const int i = q / NU, u = q % NU;
            const int m = mw + i * LR + lrow, n = nw + u * UC + lcol;
            ok = !EDGE || (m < p.M && n < p.N);
            return outp + (int64_t)m * p.ld_out + n;
        };
        auto fetch = [&](f32x4(&b)[QB], int batch) {
#pragma unroll
            for (int k = 0; k < QB; ++k) {
                bool ok;
                const float *gp = where(batch * QB + k, ok);
                b[k] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (ok) b[k] = *reinterpret_cast<const f32x4 *>(gp);
            }
        };
        fetch(buf[0], 0);
#pragma unroll
        for (int b = 0; b < NBATCH; ++b) {
            if (b + 1 < NBATCH) fetch(buf[(b + 1) & 1], b + 1);
#pragma unroll
            for (int k = 0; k < QB; ++k) {
                const int q = b * QB + k;
                bool ok;
                float *gp = where(q, ok);
                const f32x4 v = buf[b & 1][k] + acc.get(q / NU, q % NU);
                if (ok) *reinterpret_cast<f32x4 *>(gp) = v;
            }
        }
    } else {
        // ---- fp32 store of the linear program: 16 bytes per lane, direct
        float rsv[NB];
        fetch_row_scales(rsv);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int m = mw + i * LR + lrow;
            const bool mok = !EDGE || m < p.M;
            const float rs = rsv[i];
            const bool rope = EPI == EPI_LINEAR && p.rope_cos;
            const int64_t trow = (rope && mok) ? (int64_t)clampi(p.rope_pos[m], 0, p.rope_T - 1) * p.rope_half : 0;
            int rf = rope ? ((nw + lcol) >> 1) % p.rope_half : 0;
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int n = nw + u * UC + lcol;
                const bool ok = mok && (!EDGE || n < p.N);
                f32x4 v = acc.get(i, u);
                float *gp = reinterpret_cast<float *>(p.out) + (int64_t)m * p.ld_out + n;
                if (EPI == EPI_LINEAR) {
                    v *= rs;
                    if (rope) {
                        if (ok && n < p.rope_cols) rope_unit(v, p, trow, rf);
                        rf += UC / 2;
                        if (rf >= p.rope_half) rf -= p.rope_half;
                        if (rf >= p.rope_half) rf -= p.rope_half;
                    }
                    if (p.add && ok) {
                        const u32x2 c = *reinterpret_cast<const u32x2 *>(p.add + (int64_t)m * p.ld_add + n);
                        v[0] += bf16_lo(c[0]); v[1] += bf16_hi(c[0]);
                        v[2] += bf16_lo(c[1]); v[3] += bf16_hi(c[1]);
                    }
                    if (ok) rsum[i] += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
                    if (p.side && ok) {
                        const f32x4 gm = *reinterpret_cast<const f32x4 *>(p.col_scale + n);
                        *reinterpret_cast<u32x2 *>(p.side + (int64_t)m * p.ld_side + n) =
                            u32x2{pack_bf16x2(v[0] * gm[0], v[1] * gm[1]), pack_bf16x2(v[2] * gm[2], v[3] * gm[3])};
                    }
                    if (ok) *reinterpret_cast<f32x4 *>(gp) = v;
                    asm volatile("" : "+v"(rsum[i]));
                }
            }
        }
    }

    if (want_red) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const float s = row_lanes_sum<LR>(rsum[i]);
            if (lane < LR) red[wn * BM + wm * WTM + i * LR + lane] = s;
        }
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

// ---------------------------------------------------------------------------------
// Mainloops: multi-stage LDS ring filled by direct-to-LDS global loads.
//
// global_load_lds_dwordx4 moves 16 bytes per lane from global memory straight into LDS
// (lane L of the issuing wave lands at M0-base + 16*L), so operand tiles never pass
// through VGPRs and there is no ds_write phase.  The LDS position of a chunk is fixed
// by the lane, so the XOR swizzle is applied on the global side: lane L fetches the
// chunk whose swizzled home is position L.  Per-lane global offsets are loop-invariant
// (32-bit, in VGPRs); only the 64-bit scalar base advances along K.
// The loads are issued from inline asm, invisible to the compiler's waitcnt insertion;
// vmcnt is waited on explicitly (loads retire in order).  The K-step pipelines are
// described at the kernels.
// ---------------------------------------------------------------------------------
template <int BM_, int BN_, int WGM_, int WGN_, int STAGES_, int WPE_ = 2>
struct DlCfg : TileCfg<BM_, BN_, 32, WGM_, WGN_> {
    using Base = TileCfg<BM_, BN_, 32, WGM_, WGN_>;
    static constexpr int STAGES = STAGES_;
    static constexpr int WPE = WPE_;   // waves per SIMD the kernel is compiled for (register budget 512 / WPE)
    static constexpr int NW = WGM_ * WGN_;
    static constexpr int LA = Base::A_BYTES / 1024 / NW, LB = Base::B_BYTES / 1024 / NW;  // wave-loads per wave
    static_assert(Base::A_BYTES % (1024 * NW) == 0 && Base::B_BYTES % (1024 * NW) == 0, "whole wave-loads");
    static_assert(STAGES >= 3 && STAGES * Base::STAGE_BYTES <= 160 * 1024, "LDS ring");
};

// Chunk swizzle of the K-contiguous [ROWS][32] ring tiles (64-byte rows, four 16-byte chunks): chunk c of row r sits
// at chunk position c ^ kc16_swz(r).  The 16-row fragment read (lane -> row lane % 16, chunk lane / 16) is
// bank-conflict-free with row bit 2 folded into chunk bit 1 (timed over all XOR maps of the row bits: folding row
// bits 2..3 into chunk bits 0..1, which is conflict-free for 32-row fragments, takes twice as long here).
__device__ __forceinline__ int kc16_swz(int r) { return ((r >> 2) & 1) << 1; }

// Byte offset (from the tile's first element in global memory) of the chunk that lane `lane`
// of wave-load `j` must fetch so that it lands at its swizzled LDS home.  `valid` (<= ROWS) is the number of rows of
// the operand tile that exist (a tile on the ragged edge of M or N): positions past it fetch the last existing row
// (or 8-element chunk) again, so that no load leaves the matrix; what they feed is masked out by the epilogue.
template <class C, int ROWS, bool KCONT>
__device__ __forceinline__ uint32_t dl_goffset(int j, int lane, int64_t ld, int valid)
{
    if (KCONT) {  // [ROWS][32]: 64-byte rows, 16 rows per wave-load
        const int r = j * 16 + (lane >> 2);
        const int c = (lane & 3) ^ kc16_swz(r);
        const int rg = r < valid ? r : valid - 1;
        return (uint32_t)(((int64_t)rg * ld + c * 8) * 2);
    } else {      // [32][ROWS]: 2 k-rows per wave-load (ROWS = 256) or 4 (ROWS = 128); valid is a multiple of 8
        constexpr int CPR = ROWS / 8;  // chunks per k-row
        const int idx = j * 64 + lane;
        const int k = idx / CPR, pc = idx % CPR;
        const int g = (pc >> 1) ^ mn_swz(k);
        const int col = (g * 2 + (pc & 1)) * 8;
        const int cg = col < valid ? col : valid - 8;
        return (uint32_t)(((int64_t)k * ld + cg) * 2);
    }
}

// First contraction index, within the 32-wide operand tile, of the 8-element chunk (K-contiguous) or of the k-row
// (MN-contiguous) that lane `lane` of wave-load `j` fetches.
template <int ROWS, bool KCONT>
__device__ __forceinline__ int dl_chunk_k(int j, int lane)
{
    if (KCONT) {
        const int r = j * 16 + (lane >> 2);
        return ((lane & 3) ^ kc16_swz(r)) * 8;
    } else {
        return (j * 64 + lane) / (ROWS / 8);
    }
}

// K-contiguous A operand, fetched two K-steps at a time ("pair"): [ROWS][64] tiles with 128-byte rows, so that a wave-load
// covers 8 rows x one whole 128-byte line instead of 16 rows x half a line (half the L1 -> L2 requests for the same bytes:
// +2.4 % up-projection, +3.9 % down-projection, +2 to +3 % on the 8B-shape kernels).  Chunk c (of 8) of row r sits at chunk
// position c ^ (r & 7): conflict-free for the 16-row fragment read (timed over the XOR maps of the row bits).
template <class C, int ROWS>
__device__ __forceinline__ uint32_t dl_goffset_pair(int j, int lane, int64_t ld, int valid)
{
    const int r = j * 8 + (lane >> 3);
    const int c = (lane & 7) ^ (r & 7);
    const int rg = r < valid ? r : valid - 1;
    return (uint32_t)(((int64_t)rg * ld + c * 8) * 2);
}
// first contraction index, within the 64-wide pair, of the chunk that lane `lane` of wave-load `j` fetches
__device__ __forceinline__ int dl_chunk_k_pair(int j, int lane)
{
    const int r = j * 8 + (lane >> 3);
    return ((lane & 7) ^ (r & 7)) * 8;
}
// fragment of K-step h (0 / 1) of the pair: lane -> row row_base + lane % 16, elements 32 h + 8 (lane / 16) .. + 7
__device__ __forceinline__ bf16x8 dl_frag16_pair(const unsigned char *tile, int row_base, int lane, int h)
{
    const int r = row_base + (lane & 15), c = h * 4 + (lane >> 4);
    return *reinterpret_cast<const bf16x8 *>(tile + r * 128 + ((c ^ (r & 7)) << 4));
}

__device__ __forceinline__ void dl_load16(uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    // M0 carries the wave-uniform LDS destination; one wait state between the M0 write and its use.  M0 is declared
    // clobbered, so the compiler never assumes that a value of its own survives this statement.
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory", "m0");
}

// Virtual workgroup -> its work items.  A work item is an output tile, a contiguous range of that tile's K-steps, and --
// when the tile is shared -- which of its `nsplit` parts this is.
//  * Workgroups below split_from (all of them when nothing is shared) own one whole tile each.
//  * The others share the tail: the K-steps of the tail's tiles, laid end to end in units of K-step pairs, are cut into
//    tail_chunks equal contiguous ranges ("stream-K" on the last, partly filled round of tiles, or on all tiles when
//    there are few).  Range c lies in one tile or straddles the boundary between two: it then has two work items
//    (`piece` 0 and 1), the end of one tile and the start of the next, each run by a workgroup of its own.  When the
//    chunk count is a multiple of the tile count every tile is cut into equal parts and no range straddles.
//    `bid` = split_from + c.
// kcnt = 0: there is no such piece.
struct WorkItem {
    int tile, slot, split, nsplit, kbeg, kcnt;    // slot: the tile's index within the tail
};
__device__ __host__ __forceinline__ WorkItem locate_workgroup(int split_from, int tail_tiles, int tail_chunks, int bid, int piece,
                                                              int KT_all)
{
    WorkItem w = {bid, 0, 0, 1, 0, piece == 0 ? KT_all : 0};
    if (tail_chunks == 0 || bid < split_from) return w;
    const int64_t KP = KT_all / 2, total = (int64_t)tail_tiles * KP, c = bid - split_from;
    const int64_t s0 = c * total / tail_chunks, s1 = (c + 1) * total / tail_chunks;    // this chunk: pairs [s0, s1)
    const int64_t a0 = s0 / KP;
    int64_t a, lo, hi;
    if (piece == 0) {
        a = a0;
        lo = s0 - a0 * KP;
        hi = (s1 < (a0 + 1) * KP ? s1 : (a0 + 1) * KP) - a0 * KP;
    } else {
        a = a0 + 1;
        lo = 0;
        hi = s1 - (a0 + 1) * KP;
    }
    w.kcnt = 0;
    if (hi <= lo) return w;
    // chunks that reach into tile a: from the one that holds its first pair to the one that holds its last pair
    const int64_t c_lo = ((a * KP + 1) * tail_chunks + total - 1) / total - 1;
    const int64_t c_hi = (((a + 1) * KP) * tail_chunks + total - 1) / total - 1;
    w.tile = split_from + (int)a;
    w.slot = (int)a;
    w.nsplit = (int)(c_hi - c_lo + 1);
    w.split = (int)(c - c_lo);
    w.kbeg = (int)(2 * lo);
    w.kcnt = (int)(2 * (hi - lo));
    return w;
}

// Launch geometry: blocks below split_from own whole tiles; block split_from + piece * tail_chunks + c owns piece
// `piece` of range c of the shared tail (kcnt = 0: that range has no such piece).
__device__ __host__ __forceinline__ WorkItem locate_block(int split_from, int tail_tiles, int tail_chunks, int bid, int KT_all)
{
    if (tail_chunks == 0 || bid < split_from) return WorkItem{bid, 0, 0, 1, 0, KT_all};
    const int v = bid - split_from;
    return locate_workgroup(split_from, tail_tiles, tail_chunks, split_from + v % tail_chunks, v / tail_chunks, KT_all);
}

// ---------------------------------------------------------------------------------
// Split-K exchange.  Every workgroup of a tile leaves its fp32 partial in the workspace and takes a
// ticket; all but the last one to arrive return false (and must exit); the last one gets the sum of all partials,
// added in split order so that it does not depend on who arrived last, and returns true.
//
// Coherence without cache-wide operations.  The workgroups of a tile may run on different XCDs, whose L2 caches are not
// coherent with each other.  A device-scope release / acquire fence pair would write back and invalidate the WHOLE L2 of
// the XCD (every dirty output line of every other tile on it, every operand panel its neighbours are re-using): that
// cost the exchange about 35 us and slowed the tiles that run beside it.  Instead every access to the partials is a
// device-scope (agent) relaxed atomic, which the hardware performs at the device's point of coherence (sc1: stores
// write through, loads do not hit in a non-coherent cache), so only these lines travel:
//   writer: sc1 stores of the partial (16 bytes per lane, inline asm: the compiler offers the scope bit only through
//           atomics of at most 8 bytes); wait until they are acknowledged (vmcnt 0); workgroup barrier; one thread
//           takes the ticket with a device-scope atomic add, issued after the barrier, hence after every store of the
//           workgroup has been performed;
//   reader: the ticket it drew (or the counter it read on arrival) says that all other workgroups' tickets, and therefore
//           their stores, were performed; its sc1 loads, issued after that value returned, then read those values.
// ---------------------------------------------------------------------------------
// 16-byte device-scope (sc1) store / load.  The loads are issued from inline asm, invisible to the compiler's waitcnt
// insertion: the caller waits with coherent_wait8 before it touches the values.
__device__ __forceinline__ void coherent_store16(f32x4 *dst, f32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void coherent_load16(f32x4 &v, const f32x4 *src)
{
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(src) : "memory");
}
// wait for all outstanding loads; the loaded values are operands so that no use of them can be scheduled ahead of the wait
__device__ __forceinline__ void coherent_wait(f32x4 (&b)[8])
{
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7])
                 :
                 : "memory");
}
__device__ __forceinline__ void coherent_wait(f32x4 (&b)[4])
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]) : : "memory");
}

template <class C, class ACC>
__device__ __forceinline__ bool splitk_exchange(ACC &acc, const GemmParams &p, int slot, int split, int nsplit, float *red, int tid)   // slot: the tile's index within the tail
{
    // Partial tile <-> workspace in register order: float4 q of thread t at [q][t], fully coalesced.  The layout is
    // private to this exchange.
    constexpr int NQ = ACC::NB * ACC::NU;
    static_assert(NQ * 4 * C::NT == C::BM * C::BN && NQ % 8 == 0, "one float per output element, whole batches of loads");
    f32x4 *part = reinterpret_cast<f32x4 *>(p.ws_part) + (size_t)slot * p.ws_stride * NQ * C::NT;
    int *flag = reinterpret_cast<int *>(red);
    // Has everybody else already left their part?  Then this workgroup finishes the tile and need not store its own
    // (the usual case for the workgroup that takes the longest or the latest part of a tile: half of the exchange's
    // traffic).  The counter only ever counts parts whose stores have been performed.
    if (tid == 0) *flag = __hip_atomic_load(p.ws_cnt + slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(nsplit - 1);
    __syncthreads();
    int is_last = *flag;
    __syncthreads();
    if (!is_last) {
        f32x4 *mine = part + (size_t)split * NQ * C::NT + tid;
#pragma unroll
        for (int i = 0; i < ACC::NB; ++i)
#pragma unroll
            for (int u = 0; u < ACC::NU; ++u) coherent_store16(mine + (i * ACC::NU + u) * C::NT, acc.get(i, u));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const unsigned ticket = __hip_atomic_fetch_add(p.ws_cnt + slot, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = ticket == (unsigned)(nsplit - 1);
        }
        __syncthreads();
        is_last = *flag;
        __syncthreads();             // the flag lies in LDS that the epilogue, or the fill of a following piece, reuses
        if (!is_last) return false;  // uniform: the whole workgroup leaves this tile; nobody waits for anybody
    }
    // Sum of all parts in part order, P0 + P1 + ..., so that it does not depend on who came last; this workgroup's own
    // part comes from its registers (the same values it stored, or would have).  QB float4 per thread at a time: the
    // batch's running sum is built beside the accumulators and replaces them (eight in flight with the 16-row
    // accumulator layout; the 32-row layout's 16-register blocks leave room for four).
    constexpr int QB = ACC::LR == 16 ? 8 : 4;
#pragma unroll
    for (int q0 = 0; q0 < NQ; q0 += QB) {
        f32x4 t[QB];
        for (int sp = 0; sp < nsplit; ++sp) {
            f32x4 b[QB];
            if (sp == split) {
#pragma unroll
                for (int k = 0; k < QB; ++k) b[k] = acc.get((q0 + k) / ACC::NU, (q0 + k) % ACC::NU);
            } else {
                const f32x4 *src = part + (size_t)sp * NQ * C::NT + tid;
#pragma unroll
                for (int k = 0; k < QB; ++k) coherent_load16(b[k], src + (q0 + k) * C::NT);
                coherent_wait(b);
            }
#pragma unroll
            for (int k = 0; k < QB; ++k) t[k] = sp == 0 ? b[k] : t[k] + b[k];
        }
#pragma unroll
        for (int k = 0; k < QB; ++k) acc.set((q0 + k) / ACC::NU, (q0 + k) % ACC::NU, t[k]);
    }
    return true;
}

// One 16-row operand fragment of v_mfma_f32_16x16x32_bf16 from a BK = 32 tile of the ring:
// lane l holds row (l % 16), k = 8*(l/16) .. 8*(l/16)+7.
template <int ROWS, bool KCONT>
__device__ __forceinline__ bf16x8 dl_frag16(const unsigned char *tile, int row_base, int lane)
{
    if (KCONT) {   // 64-byte rows, 4 chunks
        const int r = row_base + (lane & 15);
        const int c = (lane >> 4) ^ kc16_swz(r);
        return *reinterpret_cast<const bf16x8 *>(tile + r * 64 + c * 16);
    } else {
        // transposing read: within each 16-lane group, lane i supplies the address of k-row (i/4), columns 4*(i%4)..+3
        // of the 16-row granule and receives column i of those four k-rows
        const int i = lane & 15, kq = lane >> 4;
        const int gr = row_base >> 4;
        const int k_lo = 8 * kq + (i >> 2);
        const uint32_t sub = (uint32_t)((i & 3) << 3);
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + lds_mn<ROWS>(k_lo, gr) + sub));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + lds_mn<ROWS>(k_lo + 4, gr) + sub));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    }
}

// bf16 kernel.  One K-step of 32 is ONE v_mfma_f32_16x16x32_bf16 per 16x16 block (this shape draws less power per
// FLOP than 32x32x16 and sustains a higher clock on non-trivial operands); the wave's 128 x 64 tile is 8 x 4 blocks.
// A K-step of a wave is four phases, a workgroup barrier between them, alternately "memory" and "compute":
//   M1  issue the loads of tile kt+S-1 into the slot freed by tile kt-1 (a K-contiguous A operand: half of the wave's
//       loads of the PAIR of K-steps kt+S, kt+S+1 for even kt / the other half for odd kt, into the slot freed by the
//       pair that ended with kt-1: 128-byte rows, whole cache lines per request; a K-contiguous B beside it is fetched
//       in pairs too, the whole pair kt+3, kt+4 in phase M2 of odd steps); read the row fragments of the upper half
//       of tile kt; wait until this wave's loads of tile kt+1 have landed
//   C1  the MFMAs of the lower half of the rows (fragments read in M2 of the step before)
//   M2  read the lower-half row fragments and the column fragments of tile kt+1
//   C2  the MFMAs of the upper half
// The two waves of a SIMD (waves w and w + 4) run ONE PHASE APART -- the second group passes one barrier more ahead of the
// loop, the first one more behind it -- so while one computes the other is in a memory phase ("ping-pong").  A compute
// phase runs at raised priority: the matrix pipe then takes its MFMAs back to back and the partner's LDS, load and scalar
// instructions fill the other issue slots; it also forms the LDS addresses of the wave's next memory phase (one add each:
// loop-invariant lane parts plus the slot's scalar offset), since a vector instruction issued from a memory phase has to
// wait for a slot that the computing partner leaves free (measured: ~25 cycles each, which made the phases uneven).
// With all eight waves in step instead (one barrier per K-step, every wave reading and computing at the same time) the
// waves of a SIMD were stalled on LDS at the same moments and one of them reached the barrier ~400 cycles ahead of the
// other; this schedule measures +3 to +4 % on all four kernels of the benchmark step.
// The barriers order (i) every wave's reads of tile kt before that slot is refilled and (ii) all loads of tile kt+1 before
// anybody's phase M2 of step kt; a wave waits for what it has read from LDS at the end of each compute phase (issued a
// whole phase before: no stall), so reads never race a refill.  The loads are issued from inline asm, invisible to the
// compiler's waitcnt insertion; vmcnt is waited on explicitly (loads retire in order).  K-steps are walked in pairs so
// that the two column-fragment buffers swap roles without copies: the host guarantees an even, positive count per
// workgroup.
// RAGGED: M, N or K is not a whole number of tiles.  Tiles on the edge of M or N clamp their operand fetches and run the
// bounds-checked epilogue; K is rounded up to whole pairs of K-steps and the tile fill stores zeros at the positions
// past K.
// LDS plan of the bf16 kernel.  PAIRED (A K-contiguous): three pair slots of A (two K-steps each) followed by four
// single-step slots of B -- or, when B is K-contiguous as well (PAIRB), by two pair slots of B -- 160 KB; otherwise four
// slots of [A | B].  The epilogue stages through the first EPI_RING bytes either way; `red` (row-reduction exchange;
// second half: sum-exp of the log-sum-exp partials) follows them and, when PAIRED, lies inside the B slots, which are
// free once the mainloop is over.
template <class C, bool AK, bool BKC>
struct DlLds {
    static constexpr bool PAIRED = AK, PAIRB = AK && BKC;
    static constexpr int S = C::STAGES;
    static constexpr int EPI_RING = S * C::STAGE_BYTES, RED_BYTES = 2 * C::WGN * C::BM * 4;
    static constexpr int A_REGION = PAIRED ? 3 * 2 * C::A_BYTES : 0;
    static constexpr int LDS_BYTES = PAIRED ? A_REGION + S * C::B_BYTES : EPI_RING + RED_BYTES;
    static_assert(S == 4 && LDS_BYTES >= EPI_RING + RED_BYTES && LDS_BYTES <= 160 * 1024, "LDS plan");
};

// One work item: the K-steps [wi.kbeg, wi.kbeg + wi.kcnt) of tile wi.tile, then -- unless the tile is shared and another
// workgroup finishes it -- the epilogue program.
template <class C, bool AK, bool BKC, int EPI, bool RAGGED>
__device__ __forceinline__ void gemm_item_dl(const GemmParams &p, const WorkItem &wi, const int KT_all, unsigned char *smem)
{
    constexpr int BM = C::BM, BN = C::BN, BK = 32, S = C::STAGES;
    using ACC = Acc16<C>;
    constexpr int NI = ACC::NB, NJ = ACC::NU, HM = NI / 2;
    constexpr int LA = C::LA, LB = C::LB;
    static_assert(NI % 2 == 0, "two row halves");
    using L = DlLds<C, AK, BKC>;
    constexpr bool PAIRED = L::PAIRED, PAIRB = L::PAIRB;
    constexpr int EPI_RING = L::EPI_RING, A_REGION = L::A_REGION;
    float *red = reinterpret_cast<float *>(smem + EPI_RING);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % C::WGM, wn = wave / C::WGM;
    // this work item's part of the contraction: K-steps [kbeg, kbeg + KT)
    const int nsplit = wi.nsplit, kbeg = wi.kbeg, KT = wi.kcnt;
    int tm, tn;
    tile_coords(wi.tile, p.tiles_m * p.tiles_n, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    ACC acc;
    acc_zero(acc);

    // loop-invariant per-lane byte offsets of this wave's chunks; wave w issues wave-loads w*L .. w*L+L-1
    const int valid_m = RAGGED ? (p.M - m0 < BM ? p.M - m0 : BM) : BM;
    const int valid_n = RAGGED ? (p.N - n0 < BN ? p.N - n0 : BN) : BN;
    // A: LA wave-loads per wave and K-step, or (PAIRED) LAP per wave and pair of K-steps
    constexpr int LAP = 2 * LA;
    constexpr int LBP = 2 * LB;
    uint32_t offa[PAIRED ? LAP : LA], offb[PAIRB ? LBP : LB];
    if (PAIRED) {
#pragma unroll
        for (int i = 0; i < LAP; ++i) offa[i] = dl_goffset_pair<C, BM>(wave * LAP + i, lane, p.lda, valid_m);
    } else {
#pragma unroll
        for (int i = 0; i < LA; ++i) offa[i] = dl_goffset<C, BM, AK>(wave * LA + i, lane, p.lda, valid_m);
    }
    if (PAIRB) {
#pragma unroll
        for (int i = 0; i < LBP; ++i) offb[i] = dl_goffset_pair<C, BN>(wave * LBP + i, lane, p.ldb, valid_n);
    } else {
#pragma unroll
        for (int i = 0; i < LB; ++i) offb[i] = dl_goffset<C, BN, BKC>(wave * LB + i, lane, p.ldb, valid_n);
    }
    // scalar bases of the tile's first element; advance by one K-step per tile
    const int64_t stepa = AK ? (int64_t)BK * 2 : (int64_t)BK * p.lda * 2;
    const int64_t stepb = BKC ? (int64_t)BK * 2 : (int64_t)BK * p.ldb * 2;
    const unsigned char *ga = reinterpret_cast<const unsigned char *>(AK ? p.A + (int64_t)m0 * p.lda : p.A + m0) + kbeg * stepa;
    const unsigned char *gb = reinterpret_cast<const unsigned char *>(BKC ? p.B + (int64_t)n0 * p.ldb : p.B + n0) + kbeg * stepb;
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;

    // Both operands K-contiguous (every row's fetch of a K-step has the same low address bits, and all XCDs would walk K
    // in step): each XCD starts its K loop at a different eighth of K and wraps around -- all workgroups of an XCD
    // together, so that panel sharing in its L2 is kept.  Measured +3 to +4 % on the SwiGLU backward and +2 % on the RMSNorm
    // backward (their epilogue bursts no longer coincide chip-wide), nothing on a plain store; the other layouts lose 1-2 %
    // with it and walk K from zero.  The order of the fp32 additions of a tile depends on its XCD, not on timing.
    const int rot = (AK && BKC && !RAGGED && nsplit == 1 && KT == KT_all) ? ((((int)blockIdx.x & 7) * (KT / 8)) & ~1) : 0;
    auto rotated = [&](int t) {   // position along K of the workgroup's t-th K-step (rot and KT are even: pairs stay pairs)
        int tg = t + rot;
        if (tg >= KT) tg -= KT;
        return tg;
    };
    // LDS byte offsets of the slot that holds K-step t of A (PAIRED: the pair that contains t) and of B
    auto a_slot = [&](int t) { return PAIRED ? ((t >> 1) % 3) * (2 * C::A_BYTES) : (t % S) * C::STAGE_BYTES; };
    auto b_slot = [&](int t) {
        return PAIRB ? A_REGION + ((t >> 1) & 1) * (2 * C::B_BYTES)
                     : (PAIRED ? A_REGION + (t % S) * C::B_BYTES : (t % S) * C::STAGE_BYTES + C::A_BYTES);
    };
    // loads of A for K-step t (PAIRED: for K-steps t and t + 1, t even).  A K-step (pair) that reaches past K: a lane whose
    // chunk lies past K stores zeros at its LDS position instead of fetching.
    // PAIRED: `part` 0 / 1 issues the first / second half of the wave's loads of the pair, so that every K-step issues the
    // same number of loads; -1 issues all of them.
    // `inside`: the caller knows that the K-steps fetched lie within K (no test, no zero fill)
    auto issue_a = [&](int t, int part, bool inside = false) {
        constexpr int L = PAIRED ? LAP : LA, SPAN = PAIRED ? 2 : 1;
        const int slot = a_slot(t);
        const unsigned char *sa = ga + (int64_t)rotated(t) * stepa;
        const int i0 = part == 1 ? L / 2 : 0, i1 = part == 0 ? L / 2 : L;
        if (RAGGED && !inside && (kbeg + t + SPAN) * BK > p.K) {
            const int k_left = p.K - (kbeg + t) * BK;              // contraction elements from t on that exist (may be <= 0)
#pragma unroll
            for (int i = 0; i < L; ++i) {
                if (i < i0 || i >= i1) continue;
                const int wl = wave * L + i;
                const int ck = PAIRED ? dl_chunk_k_pair(wl, lane) : dl_chunk_k<BM, AK>(wl, lane);
                if (ck < k_left) dl_load16(offa[i], sa, lds0 + (uint32_t)(slot + wl * 1024));
                else *reinterpret_cast<u32x4 *>(smem + slot + wl * 1024 + lane * 16) = u32x4{0u, 0u, 0u, 0u};
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < L; ++i)
            if (i >= i0 && i < i1) dl_load16(offa[i], sa, lds0 + (uint32_t)(slot + (wave * L + i) * 1024));
    };
    // B of K-step t (PAIRB: of the pair t, t + 1, t even)
    auto issue_b = [&](int t, bool inside = false) {
        constexpr int L = PAIRB ? LBP : LB, SPAN = PAIRB ? 2 : 1;
        const int slot = b_slot(t);
        const unsigned char *sb = gb + (int64_t)rotated(t) * stepb;
        if (RAGGED && !inside && (kbeg + t + SPAN) * BK > p.K) {
            const int k_left = p.K - (kbeg + t) * BK;
#pragma unroll
            for (int i = 0; i < L; ++i) {
                const int wl = wave * L + i;
                const int ck = PAIRB ? dl_chunk_k_pair(wl, lane) : dl_chunk_k<BN, BKC>(wl, lane);
                if (ck < k_left) dl_load16(offb[i], sb, lds0 + (uint32_t)(slot + wl * 1024));
                else *reinterpret_cast<u32x4 *>(smem + slot + wl * 1024 + lane * 16) = u32x4{0u, 0u, 0u, 0u};
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < L; ++i) dl_load16(offb[i], sb, lds0 + (uint32_t)(slot + (wave * L + i) * 1024));
    };
    bf16x8 fal[HM], fah[HM], fb0[NJ], fb1[NJ];
    auto read_a = [&](bf16x8(&fa)[HM], int t, int half) {
        const unsigned char *sa = smem + a_slot(t);
#pragma unroll
        for (int i = 0; i < HM; ++i) {
            const int row = wm * C::WTM + (half * HM + i) * 16;
            fa[i] = PAIRED ? dl_frag16_pair(sa, row, lane, t & 1) : dl_frag16<BM, AK>(sa, row, lane);
        }
    };
    // The same fragment reads with the address arithmetic split off: the per-lane LDS byte offsets of a group of fragments
    // (one offset when the operand is K-contiguous -- the blocks of a group then lie a constant apart -- else one per
    // block) are worked out in a compute phase, where the wave's vector instructions slot in between its own MFMAs, and
    // the memory phase behind it issues nothing but the reads.  (In a memory phase every vector instruction waits for a
    // slot that the computing wave of the same SIMD, at raised priority, leaves free: measured at ~25 cycles each.)
    constexpr int NAA = AK ? 1 : HM, NAB = BKC ? 1 : NJ;
    auto frag_off = [&](auto kcont, auto paired, auto rows, int slot_off, int row0, int t) -> uint32_t {
        // offset of the 16-row fragment that starts at row row0 of the operand tile of K-step t
        if constexpr (decltype(paired)::value) {
            const int r = row0 + (lane & 15), c = (t & 1) * 4 + (lane >> 4);
            return (uint32_t)(slot_off + r * 128 + ((c ^ (r & 7)) << 4));
        } else if constexpr (decltype(kcont)::value) {
            const int r = row0 + (lane & 15);
            return (uint32_t)(slot_off + r * 64 + (((lane >> 4) ^ kc16_swz(r)) << 4));
        } else {
            const int i = lane & 15, kq = lane >> 4;
            return (uint32_t)slot_off + lds_mn<decltype(rows)::value>(8 * kq + (i >> 2), row0 >> 4) + (uint32_t)((i & 3) << 3);
        }
    };
    auto pin = [](uint32_t &x) { asm volatile("" : "+v"(x)); };
    // Loop-invariant lane parts, computed once: per K-step parity for a K-contiguous operand fetched in pairs (the
    // step's position inside the 128-byte rows), per 16-row block for an MN-contiguous one (the XOR swizzle permutes the
    // blocks lane by lane).  In the loop an address is one add of the slot's (scalar) offset.
    constexpr int NLA = AK ? 2 : 2 * HM, NLB = BKC ? (PAIRB ? 2 : 1) : NJ;
    uint32_t la[NLA], lb[NLB];
#pragma unroll
    for (int q = 0; q < NLA; ++q) {
        la[q] = frag_off(std::integral_constant<bool, AK>{}, std::integral_constant<bool, PAIRED>{}, std::integral_constant<int, BM>{},
                         0, AK ? wm * C::WTM : wm * C::WTM + q * 16, AK ? q : 0);
        pin(la[q]);
    }
#pragma unroll
    for (int q = 0; q < NLB; ++q) {
        lb[q] = frag_off(std::integral_constant<bool, BKC>{}, std::integral_constant<bool, PAIRB>{}, std::integral_constant<int, BN>{},
                         0, BKC ? wn * C::WTN : wn * C::WTN + q * 16, PAIRB ? q : 0);
        pin(lb[q]);
    }
    // `par`: parity of K-step t (known where the call is written)
    // (the slot offset is pinned in a scalar register so that the sum is formed here, as one add, and not re-associated
    // into pieces that land elsewhere)
    auto prep_a = [&](uint32_t(&x)[NAA], int t, int par, int half) {
        uint32_t so = (uint32_t)(a_slot(t) + (AK ? half * HM * 16 * 128 : 0));
        asm volatile("" : "+s"(so));
#pragma unroll
        for (int i = 0; i < NAA; ++i) {
            x[i] = (AK ? la[par] : la[AK ? 0 : half * HM + i]) + so;
            pin(x[i]);
        }
    };
    auto prep_b = [&](uint32_t(&x)[NAB], int t, int par) {
        uint32_t so = (uint32_t)b_slot(t);
        asm volatile("" : "+s"(so));
#pragma unroll
        for (int j = 0; j < NAB; ++j) {
            x[j] = (BKC ? lb[PAIRB ? par : 0] : lb[BKC ? 0 : j]) + so;
            pin(x[j]);
        }
    };
    auto load_frag = [&](auto kcont, auto rows, uint32_t off) -> bf16x8 {
        if constexpr (decltype(kcont)::value) {
            return *reinterpret_cast<const bf16x8 *>(smem + off);
        } else {
            typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + off));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + off + 4 * decltype(rows)::value * 2));
            return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    };
    auto load_a = [&](bf16x8(&fa)[HM], const uint32_t(&x)[NAA]) {
#pragma unroll
        for (int i = 0; i < HM; ++i)
            fa[i] = load_frag(std::integral_constant<bool, AK>{}, std::integral_constant<int, BM>{},
                              AK ? x[0] + (uint32_t)(i * 16 * (PAIRED ? 128 : 64)) : x[AK ? 0 : i]);
    };
    auto load_b = [&](bf16x8(&fb)[NJ], const uint32_t(&x)[NAB]) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            fb[j] = load_frag(std::integral_constant<bool, BKC>{}, std::integral_constant<int, BN>{},
                              BKC ? x[0] + (uint32_t)(j * 16 * (PAIRB ? 128 : 64)) : x[BKC ? 0 : j]);
    };
    auto read_b = [&](bf16x8(&fb)[NJ], int t) {
        const unsigned char *sb = smem + b_slot(t);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int col = wn * C::WTN + j * 16;
            fb[j] = PAIRB ? dl_frag16_pair(sb, col, lane, t & 1) : dl_frag16<BN, BKC>(sb, col, lane);
        }
    };
    auto mma = [&](const bf16x8(&fa)[HM], const bf16x8(&fb)[NJ], int half) {
#pragma unroll
        for (int i = 0; i < HM; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                acc.a[half * HM + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc.a[half * HM + i][j], 0, 0, 0);
    };
    // Phase boundary: a workgroup barrier that no instruction may be moved across.  The barrier instruction alone: what a
    // wave has read from LDS it has waited for at the end of the compute phase before (below), and what it has loaded into
    // LDS it has waited for (vmcnt) in its memory phase.
    auto phase_barrier = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // Each compute phase runs with the wave's priority raised (its SIMD partner is in a memory phase meanwhile) and works
    // out the addresses of the memory phase that follows; at its end everything this wave has read from LDS so far has
    // arrived (issued a whole phase ago: no stall), so that a slot is never refilled while a read of it is still queued.
    uint32_t xah[NAA], xal[NAA], xb[NAB];
    // Refill issued in step kt: B of K-step kt+S-1 into the slot freed by kt-1; A of K-step kt+S-1 likewise, or (PAIRED) half
    // of the loads of the pair kt+S, kt+S+1 (kt even; the other half in step kt+1) into the slot freed by the pair kt-2, kt-1.
    // Either way every step issues LA+LB loads per wave, A first, and (S-2)*(LA+LB) loads of later K-steps are in flight when
    // everything that K-step kt+1 needs has landed -- provided all of them were issued in full (`exact`); otherwise
    // everything is waited for.
    // `steady`: the caller knows that every refill of this step exists (no test in the body); `even`: kt is even.
    auto step = [&](int kt, const bf16x8(&fbc)[NJ], bf16x8(&fbn)[NJ], bool last, bool steady, bool even) {
        const bool refill = steady || kt + S - 1 < KT;
        bool exact;
        if (PAIRB) {
            // B's pair kt+3, kt+4 is issued in odd steps only, in memory phase 2: its slot held the pair that ended with
            // K-step kt, read for the last time in memory phase 2 of step kt-1.  Two loads per step before the waits;
            // even steps need no wait at all (both operands of kt+1 are in the pairs already in use)
            const int tp = (kt & ~1) + S;
            if (steady || tp + 1 < KT) issue_a(tp, even ? 0 : 1, steady);  // A
            exact = steady && (!RAGGED || (kbeg + (kt | 1) + S + 1) * BK <= p.K);
        } else if (PAIRED) {
            const int tp = (kt & ~1) + S;                                 // first K-step of the pair being fetched
            if (steady || tp + 1 < KT) issue_a(tp, even ? 0 : 1, steady);  // A
            if (refill) issue_b(kt + S - 1, steady);
            exact = steady && (!RAGGED || (kbeg + (kt | 1) + S + 1) * BK <= p.K);
        } else {
            if (refill) {
                issue_a(kt + S - 1, -1, steady);                          // A
                issue_b(kt + S - 1, steady);
            }
            exact = refill && (!RAGGED || (kbeg + kt + S) * BK <= p.K);
        }
        load_a(fah, xah);                                                // memory phase 1 (behind the loads issued above)
        if (!last) {
            // K-step kt+1 must have landed before anybody's memory phase 2, the loads of kt+2 and kt+3 may be in flight
            if (PAIRB) {
                if (!even) {
                    if (exact) {
                        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LA) : "memory");   // the two halves of A's newest pair
                    } else {
                        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    }
                }
            } else if (exact) {
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * (LA + LB)) : "memory");
            } else {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        }
        phase_barrier();
        __builtin_amdgcn_s_setprio(1);                                   // compute phase 1
        mma(fal, fbc, 0);
        if (!last) {
            prep_b(xb, kt + 1, even ? 1 : 0);
            prep_a(xal, kt + 1, even ? 1 : 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        phase_barrier();
        if (!last) {                                                     // memory phase 2
            if (PAIRB && !even && (steady || kt + S < KT)) issue_b(kt + S - 1, steady);
            load_b(fbn, xb);
            load_a(fal, xal);
        }
        phase_barrier();
        __builtin_amdgcn_s_setprio(1);                                   // compute phase 2
        mma(fah, fbc, 1);
        if (!last) prep_a(xah, kt + 1, even ? 1 : 0, 1);
        __builtin_amdgcn_s_setprio(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        phase_barrier();
    };

    if (KT > 0) {
        // prologue: fill the ring; only K-step 0 has to have landed (loads retire in order)
        bool exact;
        if (PAIRB) {
            issue_a(0, -1);
            issue_b(0);
            if (2 < KT) issue_a(2, -1);
            if (2 < KT) issue_b(2);
            exact = KT >= S && (!RAGGED || (kbeg + S) * BK <= p.K);      // A 2-3 and B 2-3 issued in full: (S-2)*(LA+LB) loads
        } else if (PAIRED) {
            issue_a(0, -1);
            issue_b(0);
            if (1 < KT) issue_b(1);
            if (2 < KT) issue_a(2, -1);
            if (2 < KT) issue_b(2);
            exact = KT >= S && (!RAGGED || (kbeg + S) * BK <= p.K);      // B 1, A 2-3, B 2 all issued in full
        } else {
#pragma unroll
            for (int t = 0; t < S - 1; ++t)
                if (t < KT) {
                    issue_a(t, -1);
                    issue_b(t);
                }
            exact = KT >= S - 1 && (!RAGGED || (kbeg + S - 1) * BK <= p.K);
        }
        if (exact) {
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * (LA + LB)) : "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();
        read_a(fal, 0, 0);
        read_b(fb0, 0);
        prep_a(xah, 0, 0, 1);
        // The second wave of every SIMD runs one phase behind the first: while one computes, the other is in a memory phase.
        if (wave >= C::WGM * C::WGN / 2) phase_barrier();
        int kt = 0;
        // every refill of both steps exists -- and, in a ragged launch, lies within K (only the last pair of K-steps can
        // reach past it): branch-free body
        for (; kt + S + (PAIRED ? 1 : 0) + (RAGGED ? 2 : 0) < KT; kt += 2) {
            step(kt, fb0, fb1, false, true, true);
            step(kt + 1, fb1, fb0, false, true, false);
        }
        for (; kt < KT - 2; kt += 2) {            // ring runs dry
            step(kt, fb0, fb1, false, false, true);
            step(kt + 1, fb1, fb0, false, false, false);
        }
        step(KT - 2, fb0, fb1, false, false, true);
        step(KT - 1, fb1, fb0, true, false, false);
        if (wave < C::WGM * C::WGN / 2) phase_barrier();   // every wave passes the same number of barriers
    }
    __syncthreads();  // every wave is done with the operand ring before the epilogue reuses it

    if (nsplit > 1 && !splitk_exchange<C>(acc, p, wi.slot, wi.split, nsplit, red, tid)) return;

    // a tile that lies wholly inside the matrix takes the epilogue without bounds checks
    if (RAGGED && (m0 + BM > p.M || n0 + BN > p.N))
        run_epilogue<C, ACC, EPI, true, S * C::STAGE_BYTES>(acc, p, m0, n0, tn, smem, red, tid);
    else
        run_epilogue<C, ACC, EPI, false, S * C::STAGE_BYTES>(acc, p, m0, n0, tn, smem, red, tid);
}

// The kernel: one work item per workgroup.  TAIL = false is the kernel of every launch without shared tiles (nothing of
// the exchange is in it).  With shared tiles, workgroup split_from + piece * tail_chunks + c takes piece 0 or 1 of
// range c of the tail; a range that lies in one tile has no second piece and that workgroup leaves at once.  (The two
// pieces of a range are separate workgroups rather than a loop in one: the loop cost the kernels up to 350 spilled
// registers, and the dispatcher hands the pieces to compute units as they free up, which balances them as well.)
// A ragged K is rounded up to whole pairs of K-steps, the positions past K are zero-filled by the tile fill.
template <class C, bool AK, bool BKC, int EPI, bool RAGGED, bool TAIL>
__global__ __launch_bounds__(C::NT) __attribute__((amdgpu_waves_per_eu(C::WPE, C::WPE))) void gemm_kernel_dl(const GemmParams p)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[DlLds<C, AK, BKC>::LDS_BYTES];
    const int KT_all = RAGGED ? ((p.K + 63) / 64) * 2 : p.K / 32;
    WorkItem wi = {(int)blockIdx.x, 0, 0, 1, 0, KT_all};
    if (TAIL) {
        wi = locate_block(p.split_from, p.tail_tiles, p.tail_chunks, (int)blockIdx.x, KT_all);
        if ((int)blockIdx.x >= p.split_from && wi.kcnt == 0) return;
    }
    gemm_item_dl<C, AK, BKC, EPI, RAGGED>(p, wi, KT_all, smem);
}

// ---------------------------------------------------------------------------------
// 8-bit operands (OCP E4M3).  First the layout with both operands stored with the contraction index contiguous: A [M x K], B [N x K] bytes.
// One K-step is 64 elements = 64 bytes per row, so operand tiles, LDS slots and the direct-to-LDS fill have the byte
// geometry of the bf16 A*B^T kernel's 32-element step: both operands in pair slots (128-byte rows).
// v_mfma_f32_32x32x64_f8f6f4 takes 32 bytes
// per lane and operand: lane (row = lane % 32, half = lane / 32) holds bytes 32*half .. 32*half+31 of its row's 64;
// both operands are loaded with the same rule, so every product pairs bytes of equal k.  The accumulator layout is
// that of v_mfma_f32_32x32x16_bf16 (Acc32), and the epilogues are shared.
// Per K-step (one MFMA per 32x32 block, eight per wave) the schedule is the bf16 kernel's: four phases with a workgroup
// barrier between them, the two waves of a SIMD one phase apart, compute phases (four 64-cycle MFMAs) at raised priority:
//   M1  issue half of A's loads of the pair kt+S, kt+S+1 (kt even) / the other half (kt odd); read the row fragments of
//       the upper half of tile kt; odd steps wait for all loads but A's newest pair
//   C1  MFMAs of the lower half; LDS addresses of M2
//   M2  odd steps: issue B's pair kt+3, kt+4; read the lower-half row fragments and the column fragments of tile kt+1
//   C2  MFMAs of the upper half; LDS addresses of the next M1
// ---------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) int i32x8;

// Both operands are fetched for two K-steps at a time, as in the bf16 A*B^T kernel: [256][128 B] tiles, chunk c (of 8) of
// row r at position c ^ ((r >> 1) & 7), which is conflict-free for the 32-row fragment read (timed; c ^ (r & 7) costs a
// 2-way conflict here).  `valid`: rows of the operand tile that exist; positions past it fetch the last existing row again.
__device__ __forceinline__ uint32_t dl_goffset_pair_f8(int j, int lane, int64_t ld, int valid)
{
    const int r = j * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    const int rg = r < valid ? r : valid - 1;
    return (uint32_t)((int64_t)rg * ld + c * 16);
}
// first contraction index, within the 128-wide pair, of the 16-byte chunk that lane `lane` of wave-load `j` fetches
__device__ __forceinline__ int dl_chunk_k_pair_f8(int j, int lane)
{
    const int r = j * 8 + (lane >> 3);
    return ((lane & 7) ^ ((r >> 1) & 7)) * 16;
}
// fragment of K-step hs (0 / 1) of the pair: bytes 64 hs + 32 (lane / 32) .. + 31 of row row_base + lane % 32
__device__ __forceinline__ i32x8 dl_frag_pair_f8(const unsigned char *tile, int row_base, int lane, int hs)
{
    const int r = row_base + (lane & 31), c = hs * 4 + 2 * (lane >> 5), sw = (r >> 1) & 7;
    const u32x4 lo = *reinterpret_cast<const u32x4 *>(tile + r * 128 + ((c ^ sw) << 4));
    const u32x4 hi = *reinterpret_cast<const u32x4 *>(tile + r * 128 + (((c + 1) ^ sw) << 4));
    return i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
}

// RAGGED as in the bf16 kernel: clamped fetches and the bounds-checked epilogue on the edges of M and N; K (a multiple of
// 16) is rounded up to whole pairs of K-steps, with zeros stored at the positions past it.
// An 8-bit operand whose OUTPUT index is contiguous in memory (A stored [K x M], B stored [K x N] bytes), a pair of
// K-steps: [128 k][256 B] tiles (32 KB, the size of the K-contiguous pair tiles), filled k-row by k-row (a wave-load is
// four k-rows of 256 bytes) and read with the transposing ds_read_b64_tr_b8: within 16 lanes, lane i supplies the
// address of 8 bytes -- k-row i / 2, byte half i % 2 of a 16-byte chunk -- and receives byte i of each of the eight
// k-rows, i.e. eight consecutive k of ONE output row / column (the hardware's documented transpose; checked by a
// probe).  Four such reads give a lane the 32 consecutive k bytes that v_mfma_f32_32x32x64_f8f6f4 wants, in the byte
// order of the K-contiguous fragment.  The 16-byte chunk c of k-row k sits at chunk position c ^ (2 * (k & 7)): the
// eight k-rows of a read then fall into eight different bank groups and the two 16-lane groups that share a cycle
// (adjacent chunks) into the even and the odd ones.
__device__ __forceinline__ uint32_t dl_goffset_mn_f8(int j, int lane, int64_t ld, int valid)   // valid: a multiple of 16
{
    const int k = j * 4 + (lane >> 4);
    const int c = (lane & 15) ^ (2 * (k & 7));
    const int col = c * 16;
    const int cg = col < valid ? col : valid - 16;
    return (uint32_t)((int64_t)k * ld + cg);
}
// k-row, within the 128-wide pair, that lane `lane` of wave-load `j` fetches
__device__ __forceinline__ int dl_chunk_k_mn_f8(int j, int lane) { return j * 4 + (lane >> 4); }
// fragment of K-step hs (0 / 1) of the pair: lane -> output row / column col_base + lane % 32, k bytes 32 * (lane / 32) .. + 31
__device__ __forceinline__ i32x8 dl_frag_mn_f8(const unsigned char *tile, int col_base, int lane, int hs)
{
    typedef int v2i __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(3))) v2i lds_v2i;
    const int i = lane & 15, g = lane >> 4;
    const int chunk = (col_base >> 4) + (g & 1);
    const int k0 = 64 * hs + 32 * (g >> 1) + (i >> 1);                       // k-row of the first of the four reads
    const unsigned char *a = tile + k0 * 256 + ((chunk ^ (2 * (k0 & 7))) << 4) + ((i & 1) << 3);
    const v2i r0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(a));
    const v2i r1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(a + 8 * 256));
    const v2i r2 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(a + 16 * 256));
    const v2i r3 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(a + 24 * 256));
    return i32x8{r0[0], r0[1], r1[0], r1[1], r2[0], r2[1], r3[0], r3[1]};
}

template <class C>
struct F8Lds {
    // LDS plan of the bf16 A*B^T kernel: three pair slots of A, two pair slots of B, 160 KB; the epilogue stages through
    // the first EPI_RING bytes and `red` follows them (inside B slots that are free by then).
    static constexpr int S = C::STAGES;
    static constexpr int EPI_RING = S * C::STAGE_BYTES, RED_BYTES = 2 * C::WGN * C::BM * 4;
    static constexpr int A_REGION = 3 * 2 * C::A_BYTES, LDS_BYTES = A_REGION + S * C::B_BYTES;
    static_assert(S == 4 && LDS_BYTES >= EPI_RING + RED_BYTES && LDS_BYTES <= 160 * 1024, "LDS plan");
};

// AK / BKC: the operand is stored with the contraction index contiguous (A [M x K], B [N x K]); otherwise with the
// output index contiguous (A [K x M], B [K x N]).
template <class C, bool AK, bool BKC, int EPI, bool RAGGED>
__device__ __forceinline__ void gemm_item_dl_f8(const GemmParams &p, const WorkItem &wi, const int KT_all, unsigned char *smem)
{
    constexpr int BM = C::BM, BN = C::BN, BKB = 64, FM = C::FM, FN = C::FN, S = C::STAGES, HM = FM / 2;
    constexpr int LA = C::LA, LB = C::LB, LAP = 2 * LA, LBP = 2 * LB;
    static_assert(FM % 2 == 0, "two row halves");
    constexpr int EPI_RING = F8Lds<C>::EPI_RING, A_REGION = F8Lds<C>::A_REGION;
    float *red = reinterpret_cast<float *>(smem + EPI_RING);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % C::WGM, wn = wave / C::WGM;
    // this work item's K-steps [kbeg, kbeg + KT): an even count
    const int nsplit = wi.nsplit, kbeg = wi.kbeg, KT = wi.kcnt;
    int tm, tn;
    tile_coords(wi.tile, p.tiles_m * p.tiles_n, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    using ACC = Acc32<C>;
    ACC acc;
    acc_zero(acc);

    const int valid_m = RAGGED ? (p.M - m0 < BM ? p.M - m0 : BM) : BM;
    const int valid_n = RAGGED ? (p.N - n0 < BN ? p.N - n0 : BN) : BN;
    uint32_t offa[LAP], offb[LBP];
#pragma unroll
    for (int i = 0; i < LAP; ++i)
        offa[i] = AK ? dl_goffset_pair_f8(wave * LAP + i, lane, p.lda, valid_m) : dl_goffset_mn_f8(wave * LAP + i, lane, p.lda, valid_m);
#pragma unroll
    for (int i = 0; i < LBP; ++i)
        offb[i] = BKC ? dl_goffset_pair_f8(wave * LBP + i, lane, p.ldb, valid_n) : dl_goffset_mn_f8(wave * LBP + i, lane, p.ldb, valid_n);
    // byte advance per K-step and the tile's first byte
    const int64_t stepa = AK ? (int64_t)BKB : (int64_t)BKB * p.lda, stepb = BKC ? (int64_t)BKB : (int64_t)BKB * p.ldb;
    const unsigned char *ga = reinterpret_cast<const unsigned char *>(p.A) + (AK ? (int64_t)m0 * p.lda : (int64_t)m0) + kbeg * stepa;
    const unsigned char *gb = reinterpret_cast<const unsigned char *>(p.B) + (BKC ? (int64_t)n0 * p.ldb : (int64_t)n0) + kbeg * stepb;
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;

    auto a_slot = [&](int t) { return ((t >> 1) % 3) * (2 * C::A_BYTES); };      // the pair that contains K-step t
    auto b_slot = [&](int t) { return A_REGION + ((t >> 1) & 1) * (2 * C::B_BYTES); };   // the pair that contains K-step t
    // loads of A for the pair of K-steps t, t + 1 (t even): `part` 0 / 1 = first / second half of the wave's loads, -1 = all
    // `inside`: the caller knows that the pair lies within K (no test, no zero fill)
    auto issue_a = [&](int t, int part, bool inside = false) {
        const int slot = a_slot(t);
        const unsigned char *sa = ga + (int64_t)t * stepa;
        const int i0 = part == 1 ? LAP / 2 : 0, i1 = part == 0 ? LAP / 2 : LAP;
        if (RAGGED && !inside && (kbeg + t + 2) * BKB > p.K) {
            // the pair reaches past K: a lane whose chunk lies past K stores zeros at its LDS position instead of fetching
            const int k_left = p.K - (kbeg + t) * BKB;
#pragma unroll
            for (int i = 0; i < LAP; ++i) {
                if (i < i0 || i >= i1) continue;
                const int wl = wave * LAP + i;
                if ((AK ? dl_chunk_k_pair_f8(wl, lane) : dl_chunk_k_mn_f8(wl, lane)) < k_left) dl_load16(offa[i], sa, lds0 + (uint32_t)(slot + wl * 1024));
                else *reinterpret_cast<u32x4 *>(smem + slot + wl * 1024 + lane * 16) = u32x4{0u, 0u, 0u, 0u};
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LAP; ++i)
            if (i >= i0 && i < i1) dl_load16(offa[i], sa, lds0 + (uint32_t)(slot + (wave * LAP + i) * 1024));
    };
    // loads of B for the pair of K-steps t, t + 1 (t even)
    auto issue_b = [&](int t, bool inside = false) {
        const int slot = b_slot(t);
        const unsigned char *sb = gb + (int64_t)t * stepb;
        if (RAGGED && !inside && (kbeg + t + 2) * BKB > p.K) {
            const int k_left = p.K - (kbeg + t) * BKB;
#pragma unroll
            for (int i = 0; i < LBP; ++i) {
                const int wl = wave * LBP + i;
                if ((BKC ? dl_chunk_k_pair_f8(wl, lane) : dl_chunk_k_mn_f8(wl, lane)) < k_left) dl_load16(offb[i], sb, lds0 + (uint32_t)(slot + wl * 1024));
                else *reinterpret_cast<u32x4 *>(smem + slot + wl * 1024 + lane * 16) = u32x4{0u, 0u, 0u, 0u};
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LBP; ++i) dl_load16(offb[i], sb, lds0 + (uint32_t)(slot + (wave * LBP + i) * 1024));
    };
    i32x8 fal[HM], fah[HM], fb0[FN], fb1[FN];
    auto read_a = [&](i32x8(&fa)[HM], int t, int half) {
        const unsigned char *sa = smem + a_slot(t);
#pragma unroll
        for (int i = 0; i < HM; ++i) {
            const int row = wm * C::WTM + (half * HM + i) * 32;
            fa[i] = AK ? dl_frag_pair_f8(sa, row, lane, t & 1) : dl_frag_mn_f8(sa, row, lane, t & 1);
        }
    };
    auto read_b = [&](i32x8(&fb)[FN], int t) {
        const unsigned char *sb = smem + b_slot(t);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = wn * C::WTN + j * 32;
            fb[j] = BKC ? dl_frag_pair_f8(sb, col, lane, t & 1) : dl_frag_mn_f8(sb, col, lane, t & 1);
        }
    };
    auto mma = [&](const i32x8(&fa)[HM], const i32x8(&fb)[FN], int half) {
#pragma unroll
        for (int i = 0; i < HM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc.a[half * HM + i][j] =
                    __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j], fa[i], acc.a[half * HM + i][j], 0, 0, 0, 0, 0, 0);
    };
    // Fragment reads with the address arithmetic split off, as in the bf16 kernel: loop-invariant lane parts (K-contiguous:
    // the two 16-byte halves of a lane's 32 bytes, whose order the XOR swizzle decides lane by lane; output-contiguous: one
    // per 32-row block, which the swizzle permutes lane by lane), the slot's scalar offset added in a compute phase.
    // K-step parity h adds 64 bytes (K-contiguous: rows of 128) or 64 k-rows of 256 bytes.
    constexpr int NXA = AK ? 2 : HM, NXB = BKC ? 2 : FN, NLA8 = AK ? 2 : 2 * HM;
    auto pin = [](uint32_t &x) { asm volatile("" : "+v"(x)); };
    auto lane_pair = [&](int row0, int which) -> uint32_t {            // which: 0 = low 16 bytes, 1 = high
        const int r = row0 + (lane & 31), c = 2 * (lane >> 5) + which, sw = (r >> 1) & 7;
        return (uint32_t)(r * 128 + ((c ^ sw) << 4));
    };
    auto lane_mn = [&](int col0) -> uint32_t {
        const int i = lane & 15, g = lane >> 4;
        const int chunk = (col0 >> 4) + (g & 1), k0 = 32 * (g >> 1) + (i >> 1);
        return (uint32_t)(k0 * 256 + ((chunk ^ (2 * (k0 & 7))) << 4) + ((i & 1) << 3));
    };
    uint32_t la8[NLA8], lb8[NXB];
#pragma unroll
    for (int q = 0; q < NLA8; ++q) {
        la8[q] = AK ? lane_pair(wm * C::WTM, q) : lane_mn(wm * C::WTM + q * 32);
        pin(la8[q]);
    }
#pragma unroll
    for (int q = 0; q < NXB; ++q) {
        lb8[q] = BKC ? lane_pair(wn * C::WTN, q) : lane_mn(wn * C::WTN + q * 32);
        pin(lb8[q]);
    }
    // K-contiguous swizzle check: with c even, (c + 4h) ^ sw = (c ^ sw) ^ 4h when bit 2 of c is clear (c < 4), so parity h
    // flips bit 6 of the byte position -- lane-dependent sign, hence it goes into the lane part below via XOR
    auto prep_a8 = [&](uint32_t(&x)[NXA], int t, int par, int half) {
        uint32_t so = (uint32_t)(a_slot(t) + (AK ? half * HM * 32 * 128 : par * 64 * 256));
        asm volatile("" : "+s"(so));
#pragma unroll
        for (int i = 0; i < NXA; ++i) {
            x[i] = (AK ? (la8[i] ^ (uint32_t)(par * 64)) : la8[AK ? 0 : half * HM + i]) + so;
            pin(x[i]);
        }
    };
    auto prep_b8 = [&](uint32_t(&x)[NXB], int t, int par) {
        uint32_t so = (uint32_t)(b_slot(t) + (BKC ? 0 : par * 64 * 256));
        asm volatile("" : "+s"(so));
#pragma unroll
        for (int j = 0; j < NXB; ++j) {
            x[j] = (BKC ? (lb8[j] ^ (uint32_t)(par * 64)) : lb8[j]) + so;
            pin(x[j]);
        }
    };
    auto load_pair8 = [&](uint32_t lo, uint32_t hi) -> i32x8 {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(smem + lo), b = *reinterpret_cast<const u32x4 *>(smem + hi);
        return i32x8{(int)a[0], (int)a[1], (int)a[2], (int)a[3], (int)b[0], (int)b[1], (int)b[2], (int)b[3]};
    };
    auto load_mn8 = [&](uint32_t off) -> i32x8 {
        typedef int v2i __attribute__((ext_vector_type(2)));
        typedef __attribute__((address_space(3))) v2i lds_v2i;
        const unsigned char *a = smem + off;
        const v2i r0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(a));
        const v2i r1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(a + 8 * 256));
        const v2i r2 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(a + 16 * 256));
        const v2i r3 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(a + 24 * 256));
        return i32x8{r0[0], r0[1], r1[0], r1[1], r2[0], r2[1], r3[0], r3[1]};
    };
    auto load_a8 = [&](i32x8(&fa)[HM], const uint32_t(&x)[NXA]) {
#pragma unroll
        for (int i = 0; i < HM; ++i)
            fa[i] = AK ? load_pair8(x[0] + (uint32_t)(i * 32 * 128), x[AK ? 1 : 0] + (uint32_t)(i * 32 * 128)) : load_mn8(x[AK ? 0 : i]);
    };
    auto load_b8 = [&](i32x8(&fb)[FN], const uint32_t(&x)[NXB]) {
#pragma unroll
        for (int j = 0; j < FN; ++j)
            fb[j] = BKC ? load_pair8(x[0] + (uint32_t)(j * 32 * 128), x[BKC ? 1 : 0] + (uint32_t)(j * 32 * 128)) : load_mn8(x[BKC ? 0 : j]);
    };
    auto phase_barrier = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    uint32_t xah[NXA], xal[NXA], xb[NXB];
    // The K-step as four phases with the two waves of a SIMD one phase apart, as in the bf16 kernel; refills and waits as in
    // the bf16 A*B^T kernel: half of A's pair kt+S, kt+S+1 at the head of every step, B's whole pair kt+3, kt+4 in memory
    // phase 2 of every odd step; only odd steps wait, for all but A's newest pair.
    auto step = [&](int kt, const i32x8(&fbc)[FN], i32x8(&fbn)[FN], bool last, bool steady, bool even) {
        const int tp = (kt & ~1) + S;                                    // first K-step of the pair being fetched
        if (steady || tp + 1 < KT) issue_a(tp, even ? 0 : 1, steady);    // memory phase 1
        const bool exact = steady && (!RAGGED || (kbeg + (kt | 1) + S + 1) * BKB <= p.K);
        load_a8(fah, xah);
        if (!last && !even) {
            if (exact) {
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LA) : "memory");
            } else {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        }
        phase_barrier();
        __builtin_amdgcn_s_setprio(1);                                   // compute phase 1
        mma(fal, fbc, 0);
        if (!last) {
            prep_b8(xb, kt + 1, even ? 1 : 0);
            prep_a8(xal, kt + 1, even ? 1 : 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        phase_barrier();
        if (!last) {                                                     // memory phase 2
            if (!even && (steady || kt + S < KT)) issue_b(kt + S - 1, steady);
            load_b8(fbn, xb);
            load_a8(fal, xal);
        }
        phase_barrier();
        __builtin_amdgcn_s_setprio(1);                                   // compute phase 2
        mma(fah, fbc, 1);
        if (!last) prep_a8(xah, kt + 1, even ? 1 : 0, 1);
        __builtin_amdgcn_s_setprio(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        phase_barrier();
    };

    if (KT > 0) {
        issue_a(0, -1);
        issue_b(0);
        if (2 < KT) issue_a(2, -1);
        if (2 < KT) issue_b(2);
        if (KT >= S && (!RAGGED || (kbeg + S) * BKB <= p.K)) {
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * (LA + LB)) : "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();
        read_a(fal, 0, 0);
        read_b(fb0, 0);
        prep_a8(xah, 0, 0, 1);
        if (wave >= C::WGM * C::WGN / 2) phase_barrier();   // the second wave of every SIMD runs one phase behind
        // two K-steps per trip, so that the two column-fragment buffers swap roles without copies
        int kt = 0;
        for (; kt + S + 1 + (RAGGED ? 2 : 0) < KT; kt += 2) {   // every refill of both steps exists and lies within K
            step(kt, fb0, fb1, false, true, true);
            step(kt + 1, fb1, fb0, false, true, false);
        }
        for (; kt < KT - 2; kt += 2) {            // ring runs dry
            step(kt, fb0, fb1, false, false, true);
            step(kt + 1, fb1, fb0, false, false, false);
        }
        step(KT - 2, fb0, fb1, false, false, true);
        step(KT - 1, fb1, fb0, true, false, false);
        if (wave < C::WGM * C::WGN / 2) phase_barrier();    // every wave passes the same number of barriers
    }
    __syncthreads();  // every wave is done with the operand ring before the epilogue reuses it

    if (nsplit > 1 && !splitk_exchange<C>(acc, p, wi.slot, wi.split, nsplit, red, tid)) return;

    run_epilogue<C, ACC, EPI, RAGGED, S * C::STAGE_BYTES>(acc, p, m0, n0, tn, smem, red, tid);
}

// one work item per workgroup, as in the bf16 kernel
template <class C, bool AK, bool BKC, int EPI, bool RAGGED, bool TAIL>
__global__ __launch_bounds__(C::NT) __attribute__((amdgpu_waves_per_eu(C::WPE, C::WPE))) void gemm_kernel_dl_f8(const GemmParams p)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[F8Lds<C>::LDS_BYTES];
    const int KT_all = RAGGED ? ((p.K + 127) / 128) * 2 : p.K / 64;
    WorkItem wi = {(int)blockIdx.x, 0, 0, 1, 0, KT_all};
    if (TAIL) {
        wi = locate_block(p.split_from, p.tail_tiles, p.tail_chunks, (int)blockIdx.x, KT_all);
        if ((int)blockIdx.x >= p.split_from && wi.kcnt == 0) return;
    }
    gemm_item_dl_f8<C, AK, BKC, EPI, RAGGED>(p, wi, KT_all, smem);
}

// Host-side launcher, one per (operand layouts, epilogue mode, kernel kind).
enum KernelKind : int { KIND_WHOLE = 0, KIND_RAGGED = 1 };
template <bool AK, bool BKC, int EPI, int KIND>
hipError_t launch_gemm(const GemmParams &p, hipStream_t stream);

}  // namespace coda
