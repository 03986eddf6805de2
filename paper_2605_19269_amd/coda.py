"""ctypes binding of libcoda.so -- argument marshalling only.

Every function here has the name of the C entry point it forwards to (include/coda.h)
and does nothing but turn torch tensors into raw device pointers, sizes and pitches.
All arithmetic happens in the HIP kernels.  If the library has not been built the
import of this module fails loudly; there is no fallback path of any kind.
The measurement-only entry points (include/coda_unfused.h, include/coda_calib.h) live in
a second library, libcoda_bench.so, loaded here as well.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcoda.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libcoda.so is not built (%s). Build it with `python -m paper_2605_19269_amd.build`; "
        "there is no fallback implementation." % LIB_PATH)

LIB_BENCH_PATH = os.path.join(_HERE, "libcoda_bench.so")
if not os.path.exists(LIB_BENCH_PATH):
    raise ImportError("libcoda_bench.so is not built (%s). Build it with `python -m paper_2605_19269_amd.build`." % LIB_BENCH_PATH)

_lib = ctypes.CDLL(LIB_PATH)
_blib = ctypes.CDLL(LIB_BENCH_PATH)

# status codes / enums (mirrors of include/coda.h)
CODA_OK, CODA_ERR_NULL, CODA_ERR_SHAPE, CODA_ERR_ALIGN, CODA_ERR_DTYPE, CODA_ERR_PROGRAM, \
    CODA_ERR_WORKSPACE, CODA_ERR_LAUNCH = range(8)
CODA_BF16, CODA_F32, CODA_F8E4M3 = 0, 1, 2
(CODA_EPI_ROW_SCALE, CODA_EPI_COL_SCALE_SIDE, CODA_EPI_ADD_TILE, CODA_EPI_SWIGLU_FWD, CODA_EPI_SWIGLU_BWD,
 CODA_EPI_ROW_SUMSQ, CODA_EPI_STORE, CODA_EPI_ACCUM_F32, CODA_EPI_ROPE, CODA_EPI_RMSNORM_BWD, CODA_EPI_LSE_PARTIAL) = range(11)
CODA_REDUCE_PARTIALS, CODA_REDUCE_ATOMIC, CODA_STORE_F32 = 0, 1, 2

EXPORTS = ["coda_gemm", "coda_gemm_static_ws", "coda_gemm_workspace_bytes", "coda_row_partial_blocks", "coda_row_finalize",
           "coda_col_partial_blocks", "coda_col_finalize", "coda_lse_finalize",
           "coda_row_sumsq", "coda_fold_gamma", "coda_interleave_pairs", "coda_status_string",
           "coda_last_hip_error"]
EXPORTS_UNFUSED = ["coda_unfused_rmsnorm_apply", "coda_unfused_swiglu_fwd", "coda_unfused_swiglu_bwd",
                   "coda_unfused_add_sumsq", "coda_unfused_accumulate"]
EXPORTS_CALIB = ["coda_calib_mfma_loop", "coda_calib_mfma_loop16"]


class coda_mat(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("trans", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class coda_epi_op(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("flags", ctypes.c_uint32), ("in_", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("out2", ctypes.c_void_p), ("ld_in", ctypes.c_int64),
                ("ld_out", ctypes.c_int64), ("in2", ctypes.c_void_p), ("in3", ctypes.c_void_p),
                ("in4", ctypes.c_void_p), ("out3", ctypes.c_void_p), ("i0", ctypes.c_int64), ("i1", ctypes.c_int64)]


_vp, _i64, _i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
_lib.coda_gemm.restype = ctypes.c_int
_lib.coda_gemm.argtypes = [_vp, _i64, _i64, _i64, ctypes.POINTER(coda_mat), ctypes.POINTER(coda_mat),
                           ctypes.POINTER(coda_epi_op), _i32, _vp, ctypes.c_size_t]
_lib.coda_gemm_static_ws.restype = ctypes.c_int
_lib.coda_gemm_static_ws.argtypes = [_vp, _i64, _i64, _i64, ctypes.POINTER(coda_mat), ctypes.POINTER(coda_mat),
                                     ctypes.POINTER(coda_epi_op), _i32]
_lib.coda_gemm_workspace_bytes.restype = ctypes.c_size_t
_lib.coda_gemm_workspace_bytes.argtypes = [_i64, _i64, _i64, ctypes.POINTER(coda_epi_op), _i32]
_lib.coda_row_partial_blocks.restype = _i64
_lib.coda_row_partial_blocks.argtypes = [_i64, ctypes.POINTER(coda_epi_op), _i32]
_lib.coda_row_finalize.restype = ctypes.c_int
_lib.coda_row_finalize.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp, _i64, ctypes.c_float]
_lib.coda_col_partial_blocks.restype = _i64
_lib.coda_col_partial_blocks.argtypes = [_i64]
_lib.coda_col_finalize.restype = ctypes.c_int
_lib.coda_col_finalize.argtypes = [_vp, _vp, _i64, _i64, _vp]
_lib.coda_lse_finalize.restype = ctypes.c_int
_lib.coda_lse_finalize.argtypes = [_vp, _vp, _vp, _i64, _i64, _vp, _vp, _vp]
_lib.coda_row_sumsq.restype = ctypes.c_int
_lib.coda_row_sumsq.argtypes = [_vp, ctypes.POINTER(coda_mat), _vp]
_lib.coda_fold_gamma.restype = ctypes.c_int
_lib.coda_fold_gamma.argtypes = [_vp, ctypes.POINTER(coda_mat), _vp, _vp, _i64]
_lib.coda_interleave_pairs.restype = ctypes.c_int
_lib.coda_interleave_pairs.argtypes = [_vp, ctypes.POINTER(coda_mat), ctypes.POINTER(coda_mat), _vp, _i64]
_lib.coda_status_string.restype = ctypes.c_char_p
_lib.coda_status_string.argtypes = [ctypes.c_int]
_lib.coda_last_hip_error.restype = ctypes.c_int
_lib.coda_last_hip_error.argtypes = []
_blib.coda_unfused_rmsnorm_apply.restype = ctypes.c_int
_blib.coda_unfused_rmsnorm_apply.argtypes = [_vp, _vp, _i64, _vp, _vp, _i64, _i64, _vp, _i64]
_blib.coda_unfused_swiglu_fwd.restype = ctypes.c_int
_blib.coda_unfused_swiglu_fwd.argtypes = [_vp, _vp, _i64, _i64, _i64, _vp, _i64]
_blib.coda_unfused_swiglu_bwd.restype = ctypes.c_int
_blib.coda_unfused_swiglu_bwd.argtypes = [_vp, _vp, _i64, _vp, _i64, _i64, _i64, _vp, _i64]
_blib.coda_unfused_add_sumsq.restype = ctypes.c_int
_blib.coda_unfused_add_sumsq.argtypes = [_vp, _vp, _i64, _vp, _i64, _i64, _i64, _vp, _i64, _vp]
_blib.coda_unfused_accumulate.restype = ctypes.c_int
_blib.coda_unfused_accumulate.argtypes = [_vp, _vp, _i64, _i64, _i64, _vp, _i64]
_blib.coda_calib_mfma_loop.restype = ctypes.c_int
_blib.coda_calib_mfma_loop.argtypes = [_vp, _vp, _vp, _i64, _i64, _vp]
_blib.coda_calib_mfma_loop16.restype = ctypes.c_int
_blib.coda_calib_mfma_loop16.argtypes = [_vp, _vp, _vp, _i64, _i64, _vp]


class CodaError(RuntimeError):
    def __init__(self, status):
        self.status = status
        msg = _lib.coda_status_string(status).decode()
        if status == CODA_ERR_LAUNCH:
            msg += " (hipError %d)" % _lib.coda_last_hip_error()
        super().__init__("coda status %d: %s" % (status, msg))


def _check(status):
    if status != CODA_OK:
        raise CodaError(status)


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _ld(t):
    return 0 if t is None else (t.stride(0) if t.dim() == 2 else 0)


def mat(t, trans=False):
    """coda_mat describing a 2-D torch tensor as stored (row-major, unit column stride)."""
    import torch
    assert t.dim() == 2 and (t.shape[1] <= 1 or t.stride(1) == 1), "row-major 2-D tensor expected"
    if t.dtype == torch.bfloat16:
        dt = CODA_BF16
    elif t.dtype in (torch.uint8, torch.float8_e4m3fn):     # raw OCP E4M3 bytes
        dt = CODA_F8E4M3
    else:
        dt = CODA_F32
    return coda_mat(t.data_ptr(), t.shape[0], t.shape[1], t.stride(0), 1 if trans else 0, dt)


def _op(kind, flags=0, in_=None, out=None, out2=None, in2=None, in3=None, in4=None, out3=None, i0=0, i1=0):
    op = coda_epi_op(kind, flags, _ptr(in_), _ptr(out), _ptr(out2), _ld(in_), _ld(out), _ptr(in2), _ptr(in3),
                     _ptr(in4), _ptr(out3), i0, i1)
    op._keep = (in_, out, out2, in2, in3, in4, out3)     # the op owns a reference, so a temporary passed inline survives
    return op


# --- epilogue op constructors (each op holds its tensors for as long as the op object lives) ---
def row_scale(r):
    return _op(CODA_EPI_ROW_SCALE, in_=r)


def col_scale_side(gamma, out):
    return _op(CODA_EPI_COL_SCALE_SIDE, in_=gamma, out=out)


def rope(cos, sin, pos, head_dim, rope_cols):
    """cos / sin: f32 [T x head_dim/2] dense tables; pos: int32 [M]."""
    op = _op(CODA_EPI_ROPE, in_=cos, in2=sin, in3=pos, i0=head_dim, i1=rope_cols)
    op.ld_in = cos.shape[0]     # T: rows of the tables
    return op


def rmsnorm_bwd(C, r, z, gamma, c_out=None, dgamma_out=None, atomic=False, z_sum_over=0):
    """z: f32 [M] row statistic; with z_sum_over = d > 0 it holds the raw row sums and the kernel divides by d."""
    return _op(CODA_EPI_RMSNORM_BWD, CODA_REDUCE_ATOMIC if atomic else CODA_REDUCE_PARTIALS, in_=C, in2=r, in3=z,
               in4=gamma, out=c_out, out2=dgamma_out, i0=z_sum_over)


def lse_partial(y, pmax, psum, ztgt):
    """y: int32 [M] targets; pmax, psum: f32 [nblk x M]; ztgt: f32 [M]."""
    op = coda_epi_op(CODA_EPI_LSE_PARTIAL, 0, None, _ptr(pmax), _ptr(psum), 0, 0, None, _ptr(y), None, _ptr(ztgt), 0, 0)
    op._keep = (y, pmax, psum, ztgt)
    return op


def add_tile(C):
    return _op(CODA_EPI_ADD_TILE, in_=C)


def swiglu_fwd(preact_out=None):
    return _op(CODA_EPI_SWIGLU_FWD, out=preact_out)


def swiglu_bwd(Z, act_out=None, stat_out=None, atomic=False):
    return _op(CODA_EPI_SWIGLU_BWD, CODA_REDUCE_ATOMIC if atomic else CODA_REDUCE_PARTIALS, in_=Z,
               out=act_out, out2=stat_out)


def row_sumsq(out, atomic=False):
    return _op(CODA_EPI_ROW_SUMSQ, CODA_REDUCE_ATOMIC if atomic else CODA_REDUCE_PARTIALS, out=out)


def store(out, f32=False):
    return _op(CODA_EPI_STORE, CODA_STORE_F32 if f32 else 0, out=out)


def accum_f32(G):
    return _op(CODA_EPI_ACCUM_F32, out=G)


def _prog(ops):
    arr = (coda_epi_op * max(1, len(ops)))(*ops)
    return arr, len(ops)


# --- entry points -------------------------------------------------------------------------------
def coda_gemm_raw(stream, M, N, K, A, B, ops, workspace=None, workspace_bytes=0):
    """Forward coda_mat / coda_epi_op values unchanged; returns the status code."""
    arr, n = _prog(ops)
    return _lib.coda_gemm(stream, M, N, K, ctypes.byref(A) if A is not None else None,
                          ctypes.byref(B) if B is not None else None, arr if ops is not None else None, n,
                          workspace, workspace_bytes)


def coda_gemm(A, B, ops, transA=False, transB=False, stream=None, workspace=None):
    """D = op(A) op(B), then the epilogue ops in order.  A, B: 2-D bf16 CUDA tensors as stored.
    workspace: optional device tensor of at least coda_gemm_workspace_bytes(...) bytes (enables split-K)."""
    a, b = mat(A, transA), mat(B, transB)
    M, K = (A.shape[1], A.shape[0]) if transA else (A.shape[0], A.shape[1])
    N = B.shape[0] if transB else B.shape[1]
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(coda_gemm_raw(_stream(stream), M, N, K, a, b, list(ops), ws_ptr, ws_bytes))


def coda_gemm_static_ws_raw(stream, M, N, K, A, B, ops):
    arr, n = _prog(ops)
    return _lib.coda_gemm_static_ws(stream, M, N, K, ctypes.byref(A) if A is not None else None,
                                    ctypes.byref(B) if B is not None else None, arr if ops is not None else None, n)


def coda_gemm_static_ws(A, B, ops, transA=False, transB=False, stream=None):
    """coda_gemm with the library's static split-K scratch instead of a caller workspace (allocates nothing)."""
    a, b = mat(A, transA), mat(B, transB)
    M, K = (A.shape[1], A.shape[0]) if transA else (A.shape[0], A.shape[1])
    N = B.shape[0] if transB else B.shape[1]
    _check(coda_gemm_static_ws_raw(_stream(stream), M, N, K, a, b, list(ops)))


CODA_STATIC_WS_BYTES = 32 * 1024 * 1024 + 1024


def coda_gemm_workspace_bytes(M, N, K, ops):
    arr, n = _prog(list(ops))
    return _lib.coda_gemm_workspace_bytes(M, N, K, arr, n)


def coda_row_partial_blocks(N, ops=None):
    if ops is None:
        return _lib.coda_row_partial_blocks(N, None, 0)
    arr, n = _prog(list(ops))
    return _lib.coda_row_partial_blocks(N, arr, n)


def coda_row_finalize(partials, M, nblk, sum_out=None, rstd_out=None, d=1, eps=0.0, stream=None):
    _check(_lib.coda_row_finalize(_stream(stream), _ptr(partials), M, nblk, _ptr(sum_out), _ptr(rstd_out), d, eps))


def coda_lse_finalize(pmax, psum, M, nblk, ztgt=None, lse_out=None, loss_out=None, stream=None):
    _check(_lib.coda_lse_finalize(_stream(stream), _ptr(pmax), _ptr(psum), M, nblk, _ptr(ztgt), _ptr(lse_out), _ptr(loss_out)))


def coda_col_partial_blocks(M):
    return _lib.coda_col_partial_blocks(M)


def coda_col_finalize(partials, N, nblk, out, stream=None):
    _check(_lib.coda_col_finalize(_stream(stream), _ptr(partials), N, nblk, _ptr(out)))


def coda_row_sumsq(X, sum_out, stream=None):
    m = mat(X)
    _check(_lib.coda_row_sumsq(_stream(stream), ctypes.byref(m), _ptr(sum_out)))


def coda_fold_gamma(W, gamma, W_out, stream=None):
    m = mat(W)
    _check(_lib.coda_fold_gamma(_stream(stream), ctypes.byref(m), _ptr(gamma), _ptr(W_out), W_out.stride(0)))


def coda_interleave_pairs(Wa, Wb, W_out, stream=None):
    a, b = mat(Wa), mat(Wb)
    _check(_lib.coda_interleave_pairs(_stream(stream), ctypes.byref(a), ctypes.byref(b), _ptr(W_out), W_out.stride(0)))


def coda_status_string(status):
    return _lib.coda_status_string(status).decode()


def coda_last_hip_error():
    return _lib.coda_last_hip_error()


# --- unfused baseline kernels (include/coda_unfused.h) -----------------------------------------
def coda_unfused_rmsnorm_apply(X, r, gamma, Xn, stream=None):
    _check(_blib.coda_unfused_rmsnorm_apply(_stream(stream), _ptr(X), X.stride(0), _ptr(r), _ptr(gamma),
                                           X.shape[0], X.shape[1], _ptr(Xn), Xn.stride(0)))


def coda_unfused_swiglu_fwd(Z, H, stream=None):
    _check(_blib.coda_unfused_swiglu_fwd(_stream(stream), _ptr(Z), Z.stride(0), H.shape[0], H.shape[1],
                                        _ptr(H), H.stride(0)))


def coda_unfused_swiglu_bwd(dH, Z, dZ, stream=None):
    _check(_blib.coda_unfused_swiglu_bwd(_stream(stream), _ptr(dH), dH.stride(0), _ptr(Z), Z.stride(0),
                                        dH.shape[0], dH.shape[1], _ptr(dZ), dZ.stride(0)))


def coda_unfused_add_sumsq(D, R, Y, ss=None, stream=None):
    _check(_blib.coda_unfused_add_sumsq(_stream(stream), _ptr(D), D.stride(0), _ptr(R), R.stride(0),
                                       D.shape[0], D.shape[1], _ptr(Y), Y.stride(0), _ptr(ss)))


def coda_unfused_accumulate(T, G, stream=None):
    _check(_blib.coda_unfused_accumulate(_stream(stream), _ptr(T), T.stride(0), T.shape[0], T.shape[1],
                                        _ptr(G), G.stride(0)))


# --- measurement calibration (include/coda_calib.h) ----------------------------------------------
def _calib(fn, out_elems, a_frags, b_frags, n_blocks, iters, out, stream):
    need_a, need_b = n_blocks * 4 * 512 * 8, n_blocks * 2 * 512 * 8
    if a_frags.numel() < need_a or b_frags.numel() < need_b or a_frags.element_size() != 2 or b_frags.element_size() != 2:
        raise ValueError("fragment buffers too small: need %d and %d 16-bit elements" % (need_a, need_b))
    if out is not None and (out.numel() < out_elems or out.element_size() != 4):
        raise ValueError("out must hold %d fp32 values" % out_elems)
    _check(fn(_stream(stream), _ptr(a_frags), _ptr(b_frags), n_blocks, iters, _ptr(out)))


def coda_calib_mfma_loop(a_frags, b_frags, n_blocks, iters, out=None, stream=None):
    _calib(_blib.coda_calib_mfma_loop, 8 * 8 * 16 * 64, a_frags, b_frags, n_blocks, iters, out, stream)


def coda_calib_mfma_loop16(a_frags, b_frags, n_blocks, iters, out=None, stream=None):
    _calib(_blib.coda_calib_mfma_loop16, 8 * 8 * 4 * 64, a_frags, b_frags, n_blocks, iters, out, stream)
