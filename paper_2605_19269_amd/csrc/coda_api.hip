// coda_api.hip -- the C ABI (include/coda.h): argument validation, canonicalisation of
// the epilogue program into one of the pre-instantiated kernel variants, launch.
// Nothing here allocates, synchronises or keeps state beyond the last HIP error.
#include "../../include/coda.h"

#include "aux_kernels.hpp"
#include "gemm_launch.hpp"
#include "splitk_plan.hpp"

#include <mutex>

namespace {

static_assert(coda::PLAN_TILE_M == coda::TILE_M && coda::PLAN_TILE_N == coda::TILE_N, "the split-K plan counts the kernels' tiles");

thread_local int g_last_hip_error = 0;

coda_status launch_status(hipError_t e)
{
    if (e == hipSuccess) return CODA_OK;
    g_last_hip_error = (int)e;
    return CODA_ERR_LAUNCH;
}

// The kernels form per-lane byte offsets of up to 256 rows in 32 bits: row pitches are bounded accordingly.
constexpr int64_t MAX_LD = int64_t(1) << 22;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

// Shape / alignment checks of a bf16 operand whose op() shape must be [r x c].
coda_status check_operand(const coda_mat *X, int64_t r, int64_t c)
{
    if (!X) return CODA_ERR_NULL;
    if (X->dtype != CODA_BF16 && X->dtype != CODA_F8E4M3) return CODA_ERR_DTYPE;
    const int64_t sr = X->trans ? c : r, sc = X->trans ? r : c;
    if (X->rows != sr || X->cols != sc || X->ld < sc || X->ld > MAX_LD) return CODA_ERR_SHAPE;
    if (sr > 0 && sc > 0 && !X->ptr) return CODA_ERR_NULL;
    if (!aligned16(X->ptr) || (X->ld & (X->dtype == CODA_F8E4M3 ? 15 : 7))) return CODA_ERR_ALIGN;   // 16-byte rows
    return CODA_OK;
}

coda_status check_tile(const void *p, int64_t ld, int64_t width)
{
    if (!p) return CODA_ERR_NULL;
    if (ld < width || ld > MAX_LD) return CODA_ERR_SHAPE;
    if (!aligned16(p) || (ld & 7)) return CODA_ERR_ALIGN;
    return CODA_OK;
}

coda_status check_vec(const void *p)
{
    if (!p) return CODA_ERR_NULL;
    return aligned4(p) ? CODA_OK : CODA_ERR_ALIGN;
}

struct Parsed {
    int mode = -1;
    coda::GemmParams p{};
};

// Canonical order: ROW_SCALE < ADD_TILE < ROW_SUMSQ < COL_SCALE_SIDE < final; ROPE only between ROW_SCALE and STORE.
coda_status parse_program(const coda_epi_op *prog, int32_t n_ops, int64_t N, Parsed &out)
{
    if (n_ops < 0 || (n_ops > 0 && !prog)) return CODA_ERR_NULL;
    coda::GemmParams &p = out.p;
    int stage = 0;           // next admissible position in the canonical order
    int pair = 0;            // 0 none, 1 swiglu fwd, 2 swiglu bwd
    bool final_seen = false;
    bool linear_only = false;  // an op that only the linear program supports was used
    bool rmsbwd = false;       // RMSNORM_BWD seen: only ADD_TILE and a bf16 STORE may follow
    for (int i = 0; i < n_ops; ++i) {
        const coda_epi_op &op = prog[i];
        if (final_seen) return CODA_ERR_PROGRAM;
        coda_status st;
        switch (op.kind) {
        case CODA_EPI_ROW_SCALE:
            if (stage > 0 || pair) return CODA_ERR_PROGRAM;
            if ((st = check_vec(op.in)) != CODA_OK) return st;
            p.row_scale = static_cast<const float *>(op.in);
            stage = 1;
            break;
        case CODA_EPI_ROPE:
            if (stage > 1 || pair || rmsbwd) return CODA_ERR_PROGRAM;
            if ((st = check_vec(op.in)) != CODA_OK || (st = check_vec(op.in2)) != CODA_OK || (st = check_vec(op.in3)) != CODA_OK)
                return st;
            if ((reinterpret_cast<uintptr_t>(op.in) & 7u) || (reinterpret_cast<uintptr_t>(op.in2) & 7u)) return CODA_ERR_ALIGN;
            if (op.i0 <= 0 || (op.i0 & 7) || op.i0 > INT32_MAX || op.i1 < 0 || (op.i1 & 7) || op.i1 > N || op.ld_in <= 0 ||
                op.ld_in > INT32_MAX / (op.i0 / 2))    // T rows of head_dim / 2 entries, indexed in 31 bits
                return CODA_ERR_SHAPE;
            p.rope_cos = static_cast<const float *>(op.in);
            p.rope_sin = static_cast<const float *>(op.in2);
            p.rope_pos = static_cast<const int *>(op.in3);
            p.rope_half = (int)(op.i0 / 2);
            p.rope_cols = (int)op.i1;
            p.rope_T = (int)op.ld_in;
            stage = 4;          // only STORE may follow
            linear_only = true;
            break;
        case CODA_EPI_LSE_PARTIAL:
            if (stage > 1 || pair || rmsbwd) return CODA_ERR_PROGRAM;
            if ((st = check_vec(op.in3)) != CODA_OK || (st = check_vec(op.out)) != CODA_OK ||
                (st = check_vec(op.out2)) != CODA_OK || (st = check_vec(op.out3)) != CODA_OK)
                return st;
            p.lse_y = static_cast<const int *>(op.in3);
            p.lse_max = static_cast<float *>(op.out);
            p.lse_sum = static_cast<float *>(op.out2);
            p.lse_tgt = static_cast<float *>(op.out3);
            stage = 4;          // only STORE may follow
            linear_only = true;
            break;
        case CODA_EPI_RMSNORM_BWD:
            if (stage > 0 || pair) return CODA_ERR_PROGRAM;
            if ((st = check_tile(op.in, op.ld_in, N)) != CODA_OK) return st;
            if ((st = check_vec(op.in2)) != CODA_OK || (st = check_vec(op.in3)) != CODA_OK || (st = check_vec(op.in4)) != CODA_OK)
                return st;
            if (!aligned16(op.in4)) return CODA_ERR_ALIGN;
            p.rn_c = static_cast<const uint16_t *>(op.in);
            p.ld_rn_c = op.ld_in;
            p.rn_r = static_cast<const float *>(op.in2);
            p.rn_z = static_cast<const float *>(op.in3);
            p.rn_gamma = static_cast<const float *>(op.in4);
            if (op.i0 < 0 || op.i0 > INT32_MAX) return CODA_ERR_SHAPE;
            p.rn_zscale = op.i0 > 0 ? 1.0f / (float)op.i0 : 1.0f;
            if (op.out) {
                if ((st = check_tile(op.out, op.ld_out, N)) != CODA_OK) return st;
                p.out2 = static_cast<uint16_t *>(op.out);
                p.ld_out2 = op.ld_out;
            }
            if (op.out2) {
                if ((st = check_vec(op.out2)) != CODA_OK) return st;
                if ((op.flags & ~1u) != 0) return CODA_ERR_PROGRAM;
                p.colred = static_cast<float *>(op.out2);
                p.colred_mode = (op.flags & CODA_REDUCE_ATOMIC) ? coda::ROWRED_ATOMIC : coda::ROWRED_PARTIALS;
            }
            rmsbwd = true;
            stage = 1;          // only ADD_TILE and STORE may follow
            break;
        case CODA_EPI_ADD_TILE:
            if (stage > 1 || pair) return CODA_ERR_PROGRAM;
            if ((st = check_tile(op.in, op.ld_in, N)) != CODA_OK) return st;
            p.add = static_cast<const uint16_t *>(op.in);
            p.ld_add = op.ld_in;
            stage = 2;
            linear_only = true;
            break;
        case CODA_EPI_ROW_SUMSQ:
            if (stage > 2 || pair || rmsbwd) return CODA_ERR_PROGRAM;
            if ((st = check_vec(op.out)) != CODA_OK) return st;
            if (op.flags != CODA_REDUCE_PARTIALS && op.flags != CODA_REDUCE_ATOMIC) return CODA_ERR_PROGRAM;
            p.rowred = static_cast<float *>(op.out);
            p.rowred_mode = op.flags == CODA_REDUCE_ATOMIC ? coda::ROWRED_ATOMIC : coda::ROWRED_PARTIALS;
            stage = 3;
            linear_only = true;
            break;
        case CODA_EPI_COL_SCALE_SIDE:
            if (stage > 3 || pair || p.rope_cos || rmsbwd) return CODA_ERR_PROGRAM;
            if ((st = check_vec(op.in)) != CODA_OK) return st;
            if (!aligned16(op.in)) return CODA_ERR_ALIGN;
            if ((st = check_tile(op.out, op.ld_out, N)) != CODA_OK) return st;
            p.col_scale = static_cast<const float *>(op.in);
            p.side = static_cast<uint16_t *>(op.out);
            p.ld_side = op.ld_out;
            stage = 4;
            linear_only = true;
            break;
        case CODA_EPI_SWIGLU_FWD:
            if (pair || linear_only || rmsbwd || (N & 1)) return CODA_ERR_PROGRAM;
            if (op.out) {
                if ((st = check_tile(op.out, op.ld_out, N)) != CODA_OK) return st;
                p.out2 = static_cast<uint16_t *>(op.out);
                p.ld_out2 = op.ld_out;
            }
            pair = 1;
            stage = 5;
            break;
        case CODA_EPI_SWIGLU_BWD:
            if (pair || linear_only || stage > 0) return CODA_ERR_PROGRAM;
            if ((st = check_tile(op.in, op.ld_in, 2 * N)) != CODA_OK) return st;
            p.Z = static_cast<const uint16_t *>(op.in);
            p.ldz = op.ld_in;
            if (op.out) {
                if ((st = check_tile(op.out, op.ld_out, N)) != CODA_OK) return st;
                p.out2 = static_cast<uint16_t *>(op.out);
                p.ld_out2 = op.ld_out;
            }
            if (op.out2) {
                if ((st = check_vec(op.out2)) != CODA_OK) return st;
                if ((op.flags & ~1u) != 0) return CODA_ERR_PROGRAM;
                p.rowred = static_cast<float *>(op.out2);
                p.rowred_mode = (op.flags & CODA_REDUCE_ATOMIC) ? coda::ROWRED_ATOMIC : coda::ROWRED_PARTIALS;
            }
            pair = 2;
            stage = 5;
            break;
        case CODA_EPI_STORE: {
            const bool f32 = (op.flags & CODA_STORE_F32) != 0;
            if ((op.flags & ~CODA_STORE_F32) != 0) return CODA_ERR_PROGRAM;
            if ((pair || rmsbwd) && f32) return CODA_ERR_PROGRAM;
            const int64_t width = pair == 1 ? N / 2 : pair == 2 ? 2 * N : N;
            if (!op.out) return CODA_ERR_NULL;
            if (op.ld_out < width || op.ld_out > MAX_LD) return CODA_ERR_SHAPE;
            if (!aligned16(op.out) || (op.ld_out & (f32 ? 3 : 7))) return CODA_ERR_ALIGN;
            p.out = op.out;
            p.ld_out = op.ld_out;
            p.out_f32 = f32 ? 1 : 0;
            out.mode = pair == 1 ? coda::EPI_SWIGLU_FWD : pair == 2 ? coda::EPI_SWIGLU_BWD
                     : rmsbwd  ? coda::EPI_RMSNORM_BWD : coda::EPI_LINEAR;
            final_seen = true;
            break;
        }
        case CODA_EPI_ACCUM_F32:
            if (stage > 0 || pair) return CODA_ERR_PROGRAM;
            if (!op.out) return CODA_ERR_NULL;
            if (op.ld_out < N || op.ld_out > MAX_LD) return CODA_ERR_SHAPE;
            if (!aligned16(op.out) || (op.ld_out & 3)) return CODA_ERR_ALIGN;
            p.out = op.out;
            p.ld_out = op.ld_out;
            out.mode = coda::EPI_ACCUM;
            final_seen = true;
            break;
        default:
            return CODA_ERR_PROGRAM;
        }
    }
    return final_seen ? CODA_OK : CODA_ERR_PROGRAM;
}

__global__ void zero_counters_kernel(unsigned *c, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) c[i] = 0u;
}

template <bool AK, bool BKC, int EPI>
hipError_t dispatch_kind(int kind, const coda::GemmParams &p, hipStream_t s)
{
    using namespace coda;
    switch (kind) {
    case KIND_WHOLE: return launch_gemm<AK, BKC, EPI, KIND_WHOLE>(p, s);
    default: return launch_gemm<AK, BKC, EPI, KIND_RAGGED>(p, s);
    }
}

template <bool AK, bool BKC>
hipError_t dispatch_mode(int mode, int kind, const coda::GemmParams &p, hipStream_t s)
{
    using namespace coda;
    switch (mode) {
    case EPI_LINEAR: return dispatch_kind<AK, BKC, EPI_LINEAR>(kind, p, s);
    case EPI_SWIGLU_FWD: return dispatch_kind<AK, BKC, EPI_SWIGLU_FWD>(kind, p, s);
    case EPI_SWIGLU_BWD: return dispatch_kind<AK, BKC, EPI_SWIGLU_BWD>(kind, p, s);
    case EPI_RMSNORM_BWD: return dispatch_kind<AK, BKC, EPI_RMSNORM_BWD>(kind, p, s);
    default: return dispatch_kind<AK, BKC, EPI_ACCUM>(kind, p, s);
    }
}

template <bool AK, bool BKC, int EPI>
hipError_t dispatch_kind_f8(int kind, const coda::GemmParams &p, hipStream_t s)
{
    using namespace coda;
    return kind == KIND_WHOLE ? launch_gemm_f8<AK, BKC, EPI, KIND_WHOLE>(p, s) : launch_gemm_f8<AK, BKC, EPI, KIND_RAGGED>(p, s);
}

template <bool AK, bool BKC>
hipError_t dispatch_mode_f8(int mode, int kind, const coda::GemmParams &p, hipStream_t s)
{
    using namespace coda;
    switch (mode) {
    case EPI_LINEAR: return dispatch_kind_f8<AK, BKC, EPI_LINEAR>(kind, p, s);
    case EPI_SWIGLU_FWD: return dispatch_kind_f8<AK, BKC, EPI_SWIGLU_FWD>(kind, p, s);
    case EPI_SWIGLU_BWD: return dispatch_kind_f8<AK, BKC, EPI_SWIGLU_BWD>(kind, p, s);
    case EPI_RMSNORM_BWD: return dispatch_kind_f8<AK, BKC, EPI_RMSNORM_BWD>(kind, p, s);
    default: return dispatch_kind_f8<AK, BKC, EPI_ACCUM>(kind, p, s);
    }
}

// coda_gemm proper (shared by the entry points that differ only in where the split-K workspace comes from).
coda_status gemm_impl(void *stream, int64_t M, int64_t N, int64_t K, const coda_mat *A, const coda_mat *B,
                      const coda_epi_op *prog, int32_t n_ops, void *workspace, size_t workspace_bytes)
{
    // the kernels index in 32 bits; K is rounded up to whole pairs of K-steps (64 bf16 or 128 8-bit elements) there
    if (M < 0 || N < 0 || K < 0 || M > INT32_MAX - 256 || N > INT32_MAX / 2 || K > INT32_MAX - 128) return CODA_ERR_SHAPE;
    coda_status st;
    if ((st = check_operand(A, M, K)) != CODA_OK) return st;
    if ((st = check_operand(B, K, N)) != CODA_OK) return st;
    const bool f8 = A->dtype == CODA_F8E4M3 || B->dtype == CODA_F8E4M3;
    if (f8 && A->dtype != B->dtype) return CODA_ERR_DTYPE;                               // both 8-bit
    // 8-bit operands move in 16-byte chunks: 16 elements along whichever index is contiguous in memory
    if (f8 && ((K & 15) || (A->trans && (M & 15)) || (!B->trans && (N & 15)))) return CODA_ERR_SHAPE;
    if ((K & 7) || (N & 7) || (A->trans && (M & 7))) return CODA_ERR_SHAPE;
    Parsed ps;
    if ((st = parse_program(prog, n_ops, N, ps)) != CODA_OK) return st;
    if (M == 0 || N == 0) return CODA_OK;

    coda::GemmParams &p = ps.p;
    p.A = static_cast<const uint16_t *>(A->ptr);
    p.B = static_cast<const uint16_t *>(B->ptr);
    p.lda = A->ld;
    p.ldb = B->ld;
    p.M = (int)M;
    p.N = (int)N;
    p.K = (int)K;
    if (((M + coda::TILE_M - 1) / coda::TILE_M) * ((N + coda::TILE_N - 1) / coda::TILE_N) * 2 > INT32_MAX) return CODA_ERR_SHAPE;
    const int64_t k_pair = f8 ? 2 * coda::TILE_K : coda::TILE_K;   // elements of a pair of K-steps
    const int kind = ((K % k_pair) || (M % coda::TILE_M) || (N % coda::TILE_N)) ? coda::KIND_RAGGED : coda::KIND_WHOLE;
    const bool ak = !A->trans;   // A stored [M x K]: contraction index contiguous
    const bool bkc = B->trans;   // B stored [N x K]: contraction index contiguous
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    // split-K only when the caller brought the workspace for it; without one the shape runs unsplit
    if (workspace) {
        const coda::SplitPlan pl = coda::plan_splitk(M, N, K, f8);
        const size_t need = coda::splitk_bytes(pl);
        if (!aligned16(workspace)) return CODA_ERR_ALIGN;
        if (workspace_bytes < need) return CODA_ERR_WORKSPACE;
        if (pl.chunks > 0) {
            p.split_from = pl.first;
            p.tail_tiles = pl.tail;
            p.tail_chunks = pl.chunks;
            p.tail_pieces = pl.pieces;
            p.ws_stride = pl.stride;
            p.ws_cnt = static_cast<unsigned *>(workspace);
            p.ws_part = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + coda::SPLITK_CNT_BYTES);
            hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(256), 0, s, p.ws_cnt, pl.tail);
            if ((e = hipGetLastError()) != hipSuccess) return launch_status(e);
        }
    }
    if (f8) {
        if (ak && !bkc)
            e = dispatch_mode_f8<true, false>(ps.mode, kind, p, s);
        else if (ak && bkc)
            e = dispatch_mode_f8<true, true>(ps.mode, kind, p, s);
        else if (!ak && !bkc)
            e = dispatch_mode_f8<false, false>(ps.mode, kind, p, s);
        else
            e = dispatch_mode_f8<false, true>(ps.mode, kind, p, s);
    } else if (ak && !bkc)
        e = dispatch_mode<true, false>(ps.mode, kind, p, s);
    else if (ak && bkc)
        e = dispatch_mode<true, true>(ps.mode, kind, p, s);
    else if (!ak && !bkc)
        e = dispatch_mode<false, false>(ps.mode, kind, p, s);
    else
        e = dispatch_mode<false, true>(ps.mode, kind, p, s);
    return launch_status(e);
}

// ---- static scratch of coda_gemm_static_ws: one array per GPU, in the code object's own data, held until the process ends
constexpr size_t STATIC_WS_BYTES = coda::SPLITK_CNT_BYTES + (size_t)32 * 1024 * 1024;
static __device__ __align__(256) unsigned char scratch[STATIC_WS_BYTES];
constexpr int STATIC_WS_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[STATIC_WS_MAX_DEVICES] = {};   // device address of `scratch` on each GPU, looked up once per GPU

// Device address of the current GPU's copy of `scratch` (the array's name is only a host-side handle).
hipError_t static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= STATIC_WS_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" {

coda_status coda_gemm(void *stream, int64_t M, int64_t N, int64_t K, const coda_mat *A, const coda_mat *B,
                      const coda_epi_op *prog, int32_t n_ops, void *workspace, size_t workspace_bytes)
{
    return gemm_impl(stream, M, N, K, A, B, prog, n_ops, workspace, workspace_bytes);
}

coda_status coda_gemm_static_ws(void *stream, int64_t M, int64_t N, int64_t K, const coda_mat *A, const coda_mat *B,
                                const coda_epi_op *prog, int32_t n_ops)
{
    // the size check comes first and needs no GPU: a plan beyond the static array is an error, not a silent unsplit run
    if (M < 0 || N < 0 || K < 0 || M > INT32_MAX - 256 || N > INT32_MAX / 2 || K > INT32_MAX - 128) return CODA_ERR_SHAPE;
    if (!A || !B) return CODA_ERR_NULL;
    const bool f8 = A->dtype == CODA_F8E4M3 || B->dtype == CODA_F8E4M3;
    if (coda::splitk_bytes(coda::plan_splitk(M, N, K, f8)) > STATIC_WS_BYTES) return CODA_ERR_WORKSPACE;
    void *ws = nullptr;
    const hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return launch_status(e);
    return gemm_impl(stream, M, N, K, A, B, prog, n_ops, ws, STATIC_WS_BYTES);
}

size_t coda_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, const coda_epi_op *, int32_t)
{
    if (M < 0 || N < 0 || K < 0 || M > INT32_MAX - 256 || N > INT32_MAX / 2 || K > INT32_MAX - 128) return 0;
    // the plan depends on the operand width (an 8-bit K-step covers twice the elements): report what covers both
    const size_t b16 = coda::splitk_bytes(coda::plan_splitk(M, N, K, false)), b8 = coda::splitk_bytes(coda::plan_splitk(M, N, K, true));
    return b16 > b8 ? b16 : b8;
}

int64_t coda_row_partial_blocks(int64_t N, const coda_epi_op *, int32_t)
{
    return N <= 0 ? 0 : (N + coda::TILE_N - 1) / coda::TILE_N;
}

coda_status coda_lse_finalize(void *stream, const float *pmax, const float *psum, int64_t M, int64_t nblk, const float *ztgt,
                              float *lse_out, float *loss_out)
{
    if (M < 0 || nblk <= 0) return CODA_ERR_SHAPE;
    if (!pmax || !psum || (!lse_out && !loss_out) || (loss_out && !ztgt)) return CODA_ERR_NULL;
    if (M == 0) return CODA_OK;
    if (!aligned4(pmax) || !aligned4(psum) || !aligned4(ztgt) || !aligned4(lse_out) || !aligned4(loss_out)) return CODA_ERR_ALIGN;
    return launch_status(coda::launch_lse_finalize(static_cast<hipStream_t>(stream), pmax, psum, M, nblk, ztgt, lse_out, loss_out));
}

int64_t coda_col_partial_blocks(int64_t M)
{
    return M <= 0 ? 0 : (M + coda::TILE_M - 1) / coda::TILE_M;
}

coda_status coda_col_finalize(void *stream, const float *partials, int64_t N, int64_t nblk, float *out)
{
    if (N < 0 || nblk < 0) return CODA_ERR_SHAPE;
    if (!out) return CODA_ERR_NULL;
    if (N == 0) return CODA_OK;
    if (nblk > 0 && !partials) return CODA_ERR_NULL;
    if (!aligned4(partials) || !aligned4(out)) return CODA_ERR_ALIGN;
    return launch_status(coda::launch_col_finalize(static_cast<hipStream_t>(stream), partials, N, nblk, out));
}

coda_status coda_row_finalize(void *stream, const float *partials, int64_t M, int64_t nblk, float *sum_out,
                              float *rstd_out, int64_t d, float eps)
{
    if (M < 0 || nblk < 0 || d <= 0) return CODA_ERR_SHAPE;
    if (!sum_out && !rstd_out) return CODA_ERR_NULL;
    if (M == 0) return CODA_OK;
    if (nblk > 0 && !partials) return CODA_ERR_NULL;
    if (!aligned4(partials) || !aligned4(sum_out) || !aligned4(rstd_out)) return CODA_ERR_ALIGN;
    return launch_status(coda::launch_row_finalize(static_cast<hipStream_t>(stream), partials, M, nblk, sum_out,
                                                   rstd_out, 1.0f / (float)d, eps));
}

coda_status coda_row_sumsq(void *stream, const coda_mat *X, float *sum_out)
{
    if (!X || !sum_out) return CODA_ERR_NULL;
    if (X->dtype != CODA_BF16) return CODA_ERR_DTYPE;
    if (X->trans || X->rows < 0 || X->cols < 0 || X->ld < X->cols || (X->cols & 7)) return CODA_ERR_SHAPE;
    if (X->rows == 0) return CODA_OK;
    if (!X->ptr) return CODA_ERR_NULL;
    if (!aligned16(X->ptr) || (X->ld & 7) || !aligned4(sum_out)) return CODA_ERR_ALIGN;
    return launch_status(coda::launch_row_sumsq(static_cast<hipStream_t>(stream), static_cast<const uint16_t *>(X->ptr),
                                                X->rows, X->cols, X->ld, sum_out));
}

coda_status coda_fold_gamma(void *stream, const coda_mat *W, const float *gamma, void *W_out, int64_t ld_out)
{
    if (!W || !gamma || !W_out) return CODA_ERR_NULL;
    if (W->dtype != CODA_BF16) return CODA_ERR_DTYPE;
    if (W->trans || W->rows < 0 || W->cols < 0 || W->ld < W->cols || ld_out < W->cols || (W->cols & 7))
        return CODA_ERR_SHAPE;
    if (W->rows == 0 || W->cols == 0) return CODA_OK;
    if (!W->ptr) return CODA_ERR_NULL;
    if (!aligned16(W->ptr) || !aligned16(W_out) || (W->ld & 7) || (ld_out & 7) || !aligned4(gamma)) return CODA_ERR_ALIGN;
    return launch_status(coda::launch_fold_gamma(static_cast<hipStream_t>(stream), static_cast<const uint16_t *>(W->ptr),
                                                 W->rows, W->cols, W->ld, gamma, static_cast<uint16_t *>(W_out), ld_out));
}

coda_status coda_interleave_pairs(void *stream, const coda_mat *Wa, const coda_mat *Wb, void *W_out, int64_t ld_out)
{
    if (!Wa || !Wb || !W_out) return CODA_ERR_NULL;
    if (Wa->dtype != CODA_BF16 || Wb->dtype != CODA_BF16) return CODA_ERR_DTYPE;
    if (Wa->trans || Wb->trans || Wa->rows != Wb->rows || Wa->cols != Wb->cols || Wa->rows < 0 || Wa->cols < 0 ||
        Wa->ld < Wa->cols || Wb->ld < Wb->cols || ld_out < 2 * Wa->cols || (Wa->cols & 7))
        return CODA_ERR_SHAPE;
    if (Wa->rows == 0 || Wa->cols == 0) return CODA_OK;
    if (!Wa->ptr || !Wb->ptr) return CODA_ERR_NULL;
    if (!aligned16(Wa->ptr) || !aligned16(Wb->ptr) || !aligned16(W_out) || (Wa->ld & 7) || (Wb->ld & 7) || (ld_out & 7))
        return CODA_ERR_ALIGN;
    return launch_status(coda::launch_interleave_pairs(
        static_cast<hipStream_t>(stream), static_cast<const uint16_t *>(Wa->ptr), Wa->ld,
        static_cast<const uint16_t *>(Wb->ptr), Wb->ld, Wa->rows, Wa->cols, static_cast<uint16_t *>(W_out), ld_out));
}

const char *coda_status_string(coda_status s)
{
    switch (s) {
    case CODA_OK: return "ok";
    case CODA_ERR_NULL: return "required pointer is null";
    case CODA_ERR_SHAPE: return "unsupported or inconsistent shape";
    case CODA_ERR_ALIGN: return "pointer or leading dimension misaligned";
    case CODA_ERR_DTYPE: return "unsupported dtype";
    case CODA_ERR_PROGRAM: return "unsupported epilogue program";
    case CODA_ERR_WORKSPACE: return "workspace too small";
    case CODA_ERR_LAUNCH: return "HIP launch error";
    }
    return "unknown status";
}

int coda_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
