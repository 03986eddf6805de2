"""ctypes marshalling for coda_oracle.c (test infrastructure; see the C file's header).

bf16 tensors travel as numpy uint16 arrays holding the raw bits; fp32 as float32;
everything the oracle returns is float64.  Matrices are row-major; `trans=True`
means "stored as the transpose of the operand the GEMM uses".
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "coda_oracle.c")
_LIB = os.path.join(_HERE, "libcoda_oracle.so")
_lib = None

__all__ = [
    "build", "lib_path", "num_threads", "bf16_bits_to_f64", "row_sumsq", "rstd", "rstd_from_sumsq",
    "gemm_rowscale", "gemm_rowscale_lse", "gemm_rowscale_rope", "gemm_rowscale_swiglu", "gemm_residual_sumsq", "gemm_swiglu_bwd",
    "gemm_accumulate", "gemm_rmsnorm_bwd", "rmsnorm_linear_unfused", "rmsnorm_linear_reparam", "mlp_block",
    "fold_gamma", "interleave_pairs", "swiglu_fwd_points", "swiglu_bwd_points", "f8e4m3_to_bf16_bits",
]


def lib_path():
    return _LIB


def build(force=False):
    """Compile the oracle with gcc (fp contraction off, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c99",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def num_threads():
    """Threads the OpenMP runtime will use for the contraction."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n.split(",")[0])
    return len(os.sched_getaffinity(0))


def bf16_bits_to_f64(bits):
    """Exact widening of raw bf16 bits (uint16 array) to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


_i64 = ctypes.c_int64
_int = ctypes.c_int
_dbl = ctypes.c_double


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u16(a):
    a = np.asarray(a)
    assert a.dtype == np.uint16 and a.ndim == 2 and a.strides[1] == 2, "bf16 bits, row-major 2-D"
    return a


def _ld(a):
    return a.strides[0] // a.itemsize


def _f64(a, n=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float64)
    if n is not None:
        assert a.shape == (n,), (a.shape, n)
    return a


def _rows(rows, M):
    if rows is None:
        return None, M
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < M))
    return rows, rows.size


def _check(rc):
    if rc != 0:
        raise RuntimeError("coda_oracle error code %d" % rc)


def _opshape(X, trans):
    r, c = X.shape
    return (c, r) if trans else (r, c)


def _mnk(A, transA, B, transB):
    M, K = _opshape(A, transA)
    K2, N = _opshape(B, transB)
    assert K == K2, "contraction sizes differ: %d vs %d" % (K, K2)
    return M, N, K


def row_sumsq(X, rows=None):
    X = _u16(X)
    M, d = X.shape
    rows, R = _rows(rows, M)
    out = np.empty(R, np.float64)
    _check(_load().coda_oracle_row_sumsq(_p(X), _i64(M), _i64(d), _i64(_ld(X)), _p(rows), _i64(R), _p(out)))
    return out


def rstd(X, eps, rows=None):
    X = _u16(X)
    M, d = X.shape
    rows, R = _rows(rows, M)
    out = np.empty(R, np.float64)
    _check(_load().coda_oracle_rstd(_p(X), _i64(M), _i64(d), _i64(_ld(X)), _dbl(eps), _p(rows), _i64(R), _p(out)))
    return out


def rstd_from_sumsq(ss, d, eps):
    ss = _f64(ss)
    out = np.empty_like(ss)
    _check(_load().coda_oracle_rstd_from_sumsq(_p(ss), _i64(ss.size), _i64(d), _dbl(eps), _p(out)))
    return out


def gemm_rowscale(A, B, r=None, transA=False, transB=False, rows=None):
    """Kernel 5 / plain GEMM: O = (op(A) op(B)) * r[:, None]."""
    A, B = _u16(A), _u16(B)
    M, N, K = _mnk(A, transA, B, transB)
    r = _f64(r, M)
    rows, R = _rows(rows, M)
    O = np.empty((R, N), np.float64)
    _check(_load().coda_oracle_gemm_rowscale(
        _p(A), _i64(_ld(A)), _int(transA), _p(B), _i64(_ld(B)), _int(transB), _i64(M), _i64(N), _i64(K),
        _p(r), _p(rows), _i64(R), _p(O)))
    return O


def gemm_rowscale_lse(A, B, y, r=None, transA=False, transB=False, rows=None):
    """Kernels 3 / 8: returns (Z [R x N], z_tgt [R], lse [R]); the per-token loss is lse - z_tgt."""
    A, B = _u16(A), _u16(B)
    M, N, K = _mnk(A, transA, B, transB)
    r = _f64(r, M)
    y = np.ascontiguousarray(y, dtype=np.int32)
    assert y.shape == (M,)
    rows, R = _rows(rows, M)
    Z = np.empty((R, N), np.float64)
    zt = np.empty(R, np.float64)
    lse = np.empty(R, np.float64)
    _check(_load().coda_oracle_gemm_rowscale_lse(
        _p(A), _i64(_ld(A)), _int(transA), _p(B), _i64(_ld(B)), _int(transB), _i64(M), _i64(N), _i64(K),
        _p(r), _p(y), _p(rows), _i64(R), _p(Z), _p(zt), _p(lse)))
    return Z, zt, lse


def gemm_rowscale_rope(A, B, cos, sin, pos, head_dim, rope_cols, r=None, transA=False, transB=False, rows=None):
    """Kernels 1 / 7: O = RoPE((op(A) op(B)) * r[:, None]) on adjacent pairs of the first rope_cols columns."""
    A, B = _u16(A), _u16(B)
    M, N, K = _mnk(A, transA, B, transB)
    r = _f64(r, M)
    cos = np.ascontiguousarray(cos, dtype=np.float32)
    sin = np.ascontiguousarray(sin, dtype=np.float32)
    assert cos.shape == sin.shape and cos.ndim == 2 and cos.shape[1] * 2 == head_dim
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    assert pos.shape == (M,)
    rows, R = _rows(rows, M)
    O = np.empty((R, N), np.float64)
    _check(_load().coda_oracle_gemm_rowscale_rope(
        _p(A), _i64(_ld(A)), _int(transA), _p(B), _i64(_ld(B)), _int(transB), _i64(M), _i64(N), _i64(K),
        _p(r), _p(cos), _p(sin), _i64(cos.shape[0]), _p(pos), _i64(head_dim), _i64(rope_cols),
        _p(rows), _i64(R), _p(O)))
    return O


def gemm_rowscale_swiglu(A, B, r=None, transA=False, transB=False, rows=None, want_preact=False):
    """Kernel 6 / Kernel 2: returns O [R x N/2] (and D' [R x N] if want_preact)."""
    A, B = _u16(A), _u16(B)
    M, N, K = _mnk(A, transA, B, transB)
    r = _f64(r, M)
    rows, R = _rows(rows, M)
    O = np.empty((R, N // 2), np.float64)
    Dp = np.empty((R, N), np.float64) if want_preact else None
    _check(_load().coda_oracle_gemm_rowscale_swiglu(
        _p(A), _i64(_ld(A)), _int(transA), _p(B), _i64(_ld(B)), _int(transB), _i64(M), _i64(N), _i64(K),
        _p(r), _p(rows), _i64(R), _p(O), _p(Dp)))
    return (O, Dp) if want_preact else O


def gemm_residual_sumsq(A, B, r=None, C=None, gamma=None, transA=False, transB=False, rows=None,
                        want_scaled=False):
    """Kernel 4 with optional leading row scale: D = (AB)*r + C, ss = rowsum(D^2), O = D*gamma."""
    A, B = _u16(A), _u16(B)
    M, N, K = _mnk(A, transA, B, transB)
    r = _f64(r, M)
    gamma = _f64(gamma, N)
    if C is not None:
        C = _u16(C)
        assert C.shape == (M, N)
    rows, R = _rows(rows, M)
    D = np.empty((R, N), np.float64)
    ss = np.empty(R, np.float64)
    O = np.empty((R, N), np.float64) if want_scaled else None
    _check(_load().coda_oracle_gemm_residual_sumsq(
        _p(A), _i64(_ld(A)), _int(transA), _p(B), _i64(_ld(B)), _int(transB), _i64(M), _i64(N), _i64(K),
        _p(r), _p(C), _i64(_ld(C) if C is not None else 0), _p(gamma), _p(rows), _i64(R), _p(D), _p(ss), _p(O)))
    return (D, ss, O) if want_scaled else (D, ss)


def gemm_swiglu_bwd(A, B, Z, transA=False, transB=False, rows=None):
    """Kernel 10: returns dZ [R x 2N], O [R x N], stat [R]."""
    A, B, Z = _u16(A), _u16(B), _u16(Z)
    M, N, K = _mnk(A, transA, B, transB)
    assert Z.shape == (M, 2 * N)
    rows, R = _rows(rows, M)
    dZ = np.empty((R, 2 * N), np.float64)
    O = np.empty((R, N), np.float64)
    stat = np.empty(R, np.float64)
    _check(_load().coda_oracle_gemm_swiglu_bwd(
        _p(A), _i64(_ld(A)), _int(transA), _p(B), _i64(_ld(B)), _int(transB), _i64(M), _i64(N), _i64(K),
        _p(Z), _i64(_ld(Z)), _p(rows), _i64(R), _p(dZ), _p(O), _p(stat)))
    return dZ, O, stat


def gemm_accumulate(A, B, Gin=None, transA=False, transB=False, rows=None):
    """Weight gradient with fp32 accumulation: G_out = G_in + op(A) op(B) (returned in fp64)."""
    A, B = _u16(A), _u16(B)
    M, N, K = _mnk(A, transA, B, transB)
    if Gin is not None:
        Gin = np.asarray(Gin)
        assert Gin.dtype == np.float32 and Gin.shape == (M, N) and Gin.strides[1] == 4
    rows, R = _rows(rows, M)
    G = np.empty((R, N), np.float64)
    _check(_load().coda_oracle_gemm_accumulate(
        _p(A), _i64(_ld(A)), _int(transA), _p(B), _i64(_ld(B)), _int(transB), _i64(M), _i64(N), _i64(K),
        _p(Gin), _i64(_ld(Gin) if Gin is not None else 0), _p(rows), _i64(R), _p(G)))
    return G


def gemm_rmsnorm_bwd(A, B, C, r, z, gamma, Oin=None, transA=False, transB=False, rows=None):
    """Kernel 9: returns (O_out [R x N], C_out [R x N], dgamma [N] summed over the selected rows)."""
    A, B, C = _u16(A), _u16(B), _u16(C)
    M, N, K = _mnk(A, transA, B, transB)
    assert C.shape == (M, N)
    r, z, gamma = _f64(r, M), _f64(z, M), _f64(gamma, N)
    if Oin is not None:
        Oin = _u16(Oin)
        assert Oin.shape == (M, N)
    rows, R = _rows(rows, M)
    Oout = np.empty((R, N), np.float64)
    Cout = np.empty((R, N), np.float64)
    dg = np.empty(N, np.float64)
    _check(_load().coda_oracle_gemm_rmsnorm_bwd(
        _p(A), _i64(_ld(A)), _int(transA), _p(B), _i64(_ld(B)), _int(transB), _i64(M), _i64(N), _i64(K),
        _p(C), _i64(_ld(C)), _p(r), _p(z), _p(gamma), _p(Oin), _i64(_ld(Oin) if Oin is not None else 0),
        _p(rows), _i64(R), _p(Oout), _p(Cout), _p(dg)))
    return Oout, Cout, dg


def _rms_linear(fn, X, gamma, eps, W, R, transW, rows):
    X, W = _u16(X), _u16(W)
    M, d = X.shape
    d2, N = _opshape(W, transW)
    assert d == d2
    gamma = _f64(gamma, d)
    if R is not None:
        R = _u16(R)
        assert R.shape == (M, N)
    rows, nR = _rows(rows, M)
    Y = np.empty((nR, N), np.float64)
    ss = np.empty(nR, np.float64)
    _check(fn(_p(X), _i64(_ld(X)), _p(gamma), _dbl(eps), _p(W), _i64(_ld(W)), _int(transW),
              _p(R), _i64(_ld(R) if R is not None else 0), _i64(M), _i64(N), _i64(d),
              _p(rows), _i64(nR), _p(Y), _p(ss)))
    return Y, ss


def rmsnorm_linear_unfused(X, gamma, eps, W, R=None, transW=False, rows=None):
    """Canonical chain: Y = RMSNorm(X, gamma) W + R; returns (Y, rowsum(Y^2))."""
    return _rms_linear(_load().coda_oracle_rmsnorm_linear_unfused, X, gamma, eps, W, R, transW, rows)


def rmsnorm_linear_reparam(X, gamma, eps, W, R=None, transW=False, rows=None):
    """Reparameterised: Y = diag(r) (X (diag(gamma) W)) + R; returns (Y, rowsum(Y^2))."""
    return _rms_linear(_load().coda_oracle_rmsnorm_linear_reparam, X, gamma, eps, W, R, transW, rows)


def mlp_block(X, gamma, eps, W1, W2, R=None, reparam=False, rows=None):
    """RMSNorm -> W1 -> SwiGLU -> W2 -> + R, no intermediate rounding; returns (Y, rowsum(Y^2))."""
    X, W1, W2 = _u16(X), _u16(W1), _u16(W2)
    M, d = X.shape
    assert W1.shape[0] == d and W1.shape[1] % 2 == 0
    F = W1.shape[1] // 2
    assert W2.shape[0] == F
    d2 = W2.shape[1]
    gamma = _f64(gamma, d)
    if R is not None:
        R = _u16(R)
        assert R.shape == (M, d2)
    rows, nR = _rows(rows, M)
    Y = np.empty((nR, d2), np.float64)
    ss = np.empty(nR, np.float64)
    _check(_load().coda_oracle_mlp_block(
        _p(X), _i64(_ld(X)), _p(gamma), _dbl(eps), _p(W1), _i64(_ld(W1)), _p(W2), _i64(_ld(W2)),
        _p(R), _i64(_ld(R) if R is not None else 0), _i64(M), _i64(d), _i64(F), _i64(d2),
        _int(1 if reparam else 0), _p(rows), _i64(nR), _p(Y), _p(ss)))
    return Y, ss


def fold_gamma(W, gamma):
    W = _u16(W)
    K, N = W.shape
    gamma = _f64(gamma, K)
    out = np.empty((K, N), np.float64)
    _check(_load().coda_oracle_fold_gamma(_p(W), _i64(_ld(W)), _p(gamma), _i64(K), _i64(N), _p(out)))
    return out


def interleave_pairs(Wa, Wb):
    Wa, Wb = _u16(Wa), _u16(Wb)
    assert Wa.shape == Wb.shape
    K, N = Wa.shape
    out = np.empty((K, 2 * N), np.uint16)
    _check(_load().coda_oracle_interleave_pairs(_p(Wa), _i64(_ld(Wa)), _p(Wb), _i64(_ld(Wb)), _i64(K), _i64(N), _p(out)))
    return out


def swiglu_fwd_points(g, u):
    g, u = _f64(g), _f64(u)
    o = np.empty_like(g)
    _check(_load().coda_oracle_swiglu_fwd_points(_p(g), _p(u), _i64(g.size), _p(o)))
    return o


def swiglu_bwd_points(d, g, u):
    d, g, u = _f64(d), _f64(g), _f64(u)
    dG, dU = np.empty_like(g), np.empty_like(g)
    _check(_load().coda_oracle_swiglu_bwd_points(_p(d), _p(g), _p(u), _i64(g.size), _p(dG), _p(dU)))
    return dG, dU


def f8e4m3_to_bf16_bits(bits):
    """OCP E4M3 bytes (uint8 array, any shape) -> the bf16 bit patterns of the same values (exact); the result can be
    passed to every gemm_* function above in place of a bf16 operand."""
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    out = np.empty(bits.shape, np.uint16)
    _check(_load().coda_oracle_f8e4m3_to_bf16(_p(bits), _i64(bits.size), _p(out)))
    return out
