"""Pins for the CPU oracle: each test checks it against something other than itself
(brute force, an independent library routine, a closed form, an identity of the paper,
finite differences), chosen so that a dropped term, a wrong sign or index, or a
transposed operand fails at least one of them.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from paper_2605_19269_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def wide(b):
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- bf16 bit format
def test_bf16_bit_patterns(oracle):
    b = np.array([[0x3F80, 0xBF80, 0x4000, 0x3F00, 0x0000, 0x3FC0, 0x4049]], dtype=np.uint16)
    want = np.array([1.0, -1.0, 2.0, 0.5, 0.0, 1.5, 3.140625])
    assert np.array_equal(oracle.bf16_bits_to_f64(b)[0], want)
    # the oracle's own widening, exercised through a 1x1 "GEMM" with B = [[1]]
    one = np.array([[0x3F80]], dtype=np.uint16)
    for v, w in zip(b[0], want):
        got = oracle.gemm_rowscale(np.array([[v]], dtype=np.uint16), one)
        assert got[0, 0] == w


def test_input_rounding_is_rne():
    # 1 + 2^-8 is a tie between 1.0 (even mantissa) and 1 + 2^-7: RNE picks 1.0;
    # 1 + 3*2^-8 is a tie between 1+2^-7 (odd) and 1+2^-6 (even): RNE picks 1+2^-6.
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    assert wide(synth.f32_to_bf16_bits(x)).tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]


# ---------------------------------------------------------------- contraction
def brute_gemm(A, B):
    M, K = A.shape
    N = B.shape[1]
    out = [[0.0] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            s = 0.0
            for k in range(K):
                s += float(A[i, k]) * float(B[k, j])
            out[i][j] = s
    return np.array(out)


@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, False), (True, True)])
def test_gemm_brute_force_tiny(oracle, transA, transB):
    g = rng(1)
    M, N, K = 5, 7, 6
    A = synth.normal_bf16(g, (M, K), 1.0)
    B = synth.normal_bf16(g, (K, N), 1.0)
    want = brute_gemm(wide(A), wide(B))
    As = np.ascontiguousarray(A.T) if transA else A
    Bs = np.ascontiguousarray(B.T) if transB else B
    got = oracle.gemm_rowscale(As, Bs, transA=transA, transB=transB)
    assert np.array_equal(got, want)  # same products, same order -> bit-identical


@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, False)])
def test_gemm_vs_library_matmul(oracle, transA, transB):
    g = rng(2)
    M, N, K = 64, 96, 80
    A = synth.normal_bf16(g, (M, K), 1.0)
    B = synth.normal_bf16(g, (K, N), 0.5)
    want = torch.from_numpy(wide(A)) @ torch.from_numpy(wide(B))
    As = np.ascontiguousarray(A.T) if transA else A
    Bs = np.ascontiguousarray(B.T) if transB else B
    got = oracle.gemm_rowscale(As, Bs, transA=transA, transB=transB)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-12)


def test_gemm_leading_dimension_and_row_selection(oracle):
    g = rng(3)
    big = synth.normal_bf16(g, (40, 50), 1.0)
    A = big[3:23, 5:35]          # 20 x 30 view, ld = 50
    B = synth.normal_bf16(g, (30, 12), 1.0)
    rows = np.array([19, 0, 7], dtype=np.int64)
    want = (wide(np.ascontiguousarray(A)) @ wide(B))[rows]
    got = oracle.gemm_rowscale(A, B, rows=rows)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


def test_gemm_one_hot_picks_the_right_operand_entry(oracle):
    # A = e_i e_k^T, B = e_k' e_j^T: product is nonzero only if k == k'; catches index swaps.
    M, K, N = 4, 5, 6
    for (i, k, kp, j) in [(1, 2, 2, 3), (3, 4, 1, 0)]:
        A = np.zeros((M, K), np.float32); A[i, k] = 2.0
        B = np.zeros((K, N), np.float32); B[kp, j] = 3.0
        got = oracle.gemm_rowscale(bits(A), bits(B))
        want = np.zeros((M, N)); want[i, j] = 6.0 if k == kp else 0.0
        assert np.array_equal(got, want)


def test_row_scale_is_per_row_not_per_column(oracle):
    g = rng(4)
    A = synth.normal_bf16(g, (6, 8), 1.0)
    B = synth.normal_bf16(g, (8, 6), 1.0)
    r = np.array([1.0, 2.0, 3.0, 4.0, 5.0, 6.0])
    got = oracle.gemm_rowscale(A, B, r=r)
    want = (wide(A) @ wide(B)) * r[:, None]
    np.testing.assert_allclose(got, want, rtol=1e-14)
    sel = oracle.gemm_rowscale(A, B, r=r, rows=np.array([4, 2]))
    np.testing.assert_allclose(sel, want[[4, 2]], rtol=1e-14)   # r indexed by original row


# ---------------------------------------------------------------- rstd / RMSNorm
def test_rstd_closed_form_constant_rows(oracle):
    d = 64
    X = np.stack([np.full(d, c, np.float32) for c in (0.5, -2.0, 0.0, 1.0)])
    eps = 1e-6
    got = oracle.rstd(bits(X), eps)
    want = [1.0 / math.sqrt(c * c + eps) for c in (0.5, -2.0, 0.0, 1.0)]
    np.testing.assert_allclose(got, want, rtol=1e-15)
    assert abs(got[2] - 1000.0) < 1e-9          # zero row: 1/sqrt(eps)


def test_rstd_vs_library_rmsnorm(oracle):
    g = rng(5)
    X = synth.normal_bf16(g, (9, 48), 1.0)
    Xd = torch.from_numpy(wide(X))
    eps = 1e-6
    normed = torch.nn.functional.rms_norm(Xd, (48,), weight=None, eps=eps).numpy()
    got = oracle.rstd(X, eps)
    np.testing.assert_allclose(wide(X) * got[:, None], normed, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(oracle.rstd_from_sumsq(oracle.row_sumsq(X), 48, eps), got, rtol=1e-15)


def test_row_sumsq_one_hot_rows_exact(oracle):
    X = np.zeros((5, 16), np.float32)
    X[0, 3] = 3.0; X[1, 0] = -4.0; X[2, 15] = 2.0; X[2, 14] = 1.0; X[4, :] = 1.0
    assert oracle.row_sumsq(bits(X)).tolist() == [9.0, 16.0, 5.0, 0.0, 16.0]


def torch_chain(X, gamma, eps, W, R):
    Xd = torch.from_numpy(wide(X))
    Y = torch.nn.functional.rms_norm(Xd, (Xd.shape[1],), weight=torch.from_numpy(gamma), eps=eps) @ torch.from_numpy(wide(W))
    if R is not None:
        Y = Y + torch.from_numpy(wide(R))
    return Y.numpy()


def test_unfused_chain_vs_library_ops(oracle):
    c = synth.tiny_rmsnorm_gemm(seed=7, M=12, K=40, N=24)
    gamma = c["gamma"].astype(np.float64)
    Y, ss = oracle.rmsnorm_linear_unfused(c["X"], gamma, c["eps"], c["W"], c["R"])
    want = torch_chain(c["X"], gamma, c["eps"], c["W"], c["R"])
    np.testing.assert_allclose(Y, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ss, (want ** 2).sum(1), rtol=1e-12)


@pytest.mark.parametrize("shape", [(8, 12, 16), (256, 256, 512)])
def test_reparameterisation_identity(oracle, shape):
    # Section 3.2.1: r commutes with the second GEMM and gamma folds into W.
    M, K, N = shape
    c = synth.tiny_rmsnorm_gemm(seed=0, M=M, K=K, N=N)
    gamma = c["gamma"].astype(np.float64)
    Yu, su = oracle.rmsnorm_linear_unfused(c["X"], gamma, c["eps"], c["W"], c["R"])
    Yr, sr = oracle.rmsnorm_linear_reparam(c["X"], gamma, c["eps"], c["W"], c["R"])
    scale = np.abs(Yu).max()
    assert np.abs(Yu - Yr).max() <= 1e-12 * scale
    np.testing.assert_allclose(su, sr, rtol=1e-12)
    # and the pieces the GPU path is built from compose to the same thing
    r = oracle.rstd(c["X"], c["eps"])
    Wp = oracle.fold_gamma(c["W"], gamma)
    Yc = (wide(c["X"]) @ Wp) * r[:, None] + wide(c["R"])
    assert np.abs(Yu - Yc).max() <= 1e-12 * scale


def test_fused_kernel_form_matches_chain_when_gamma_is_one(oracle):
    # gamma == 1: W' == W exactly, so Kernel 4 with a leading row scale IS the chain.
    c = synth.tiny_rmsnorm_gemm(seed=3, M=10, K=32, N=20)
    ones = np.ones(32)
    Yu, su = oracle.rmsnorm_linear_unfused(c["X"], ones, c["eps"], c["W"], c["R"])
    r = oracle.rstd(c["X"], c["eps"])
    D, ss = oracle.gemm_residual_sumsq(c["X"], c["W"], r=r, C=c["R"])
    np.testing.assert_allclose(D, Yu, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ss, su, rtol=1e-12)


def test_kernel4_pieces(oracle):
    g = rng(8)
    A = synth.normal_bf16(g, (6, 10), 1.0); B = synth.normal_bf16(g, (10, 8), 1.0)
    C = synth.normal_bf16(g, (6, 8), 1.0); gamma = g.random(8) + 0.5
    D, ss, O = oracle.gemm_residual_sumsq(A, B, C=C, gamma=gamma, want_scaled=True)
    want = wide(A) @ wide(B) + wide(C)
    np.testing.assert_allclose(D, want, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(ss, (want ** 2).sum(1), rtol=1e-13)      # reduces the UNSCALED D
    np.testing.assert_allclose(O, want * gamma[None, :], rtol=1e-13, atol=1e-14)
    D0, ss0 = oracle.gemm_residual_sumsq(A, B)                            # no residual: plain GEMM
    np.testing.assert_allclose(D0, wide(A) @ wide(B), rtol=1e-13, atol=1e-14)


def test_mlp_block_unfused_equals_reparam_and_library(oracle):
    g = rng(9)
    M, d, F = 6, 24, 16
    X = synth.normal_bf16(g, (M, d), 1.0)
    gamma = (g.random(d) + 0.5)
    W1 = synth.normal_bf16(g, (d, 2 * F), 0.2)
    W2 = synth.normal_bf16(g, (F, d), 0.2)
    Yu, su = oracle.mlp_block(X, gamma, 1e-6, W1, W2, R=X, reparam=False)
    Yr, sr = oracle.mlp_block(X, gamma, 1e-6, W1, W2, R=X, reparam=True)
    assert np.abs(Yu - Yr).max() <= 1e-12 * np.abs(Yu).max()
    Z = torch.from_numpy(torch_chain(X, gamma, 1e-6, W1, None))
    H = torch.nn.functional.silu(Z[:, 0::2]) * Z[:, 1::2]
    want = (H @ torch.from_numpy(wide(W2)) + torch.from_numpy(wide(X))).numpy()
    np.testing.assert_allclose(Yu, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(su, (want ** 2).sum(1), rtol=1e-12)


# ---------------------------------------------------------------- SwiGLU forward
def golden_points():
    pts = []
    with open(os.path.join(GOLDEN, "swiglu_closed_form.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a, frac = line.split()
            num, den = frac.split("/")
            pts.append((math.log(float(a)), float(num) / float(den)))
    return pts


def test_swiglu_forward_closed_form(oracle):
    for g, sig in golden_points():
        for u in (1.0, -2.5):
            got = oracle.swiglu_fwd_points(np.array([g]), np.array([u]))[0]
            assert abs(got - g * sig * u) <= 1e-15 * max(1.0, abs(got))
    big = oracle.swiglu_fwd_points(np.array([40.0, -40.0, 0.0, -800.0]), np.array([3.0, 3.0, 3.0, 3.0]))
    assert abs(big[0] - 120.0) < 1e-12 and abs(big[1]) < 1e-15 and big[2] == 0.0 and big[3] == 0.0


def test_swiglu_forward_pair_order_and_library(oracle):
    # even column = gate, odd column = up.  A = I picks rows of B, so D' = B exactly.
    g = rng(10)
    N = 12
    B = synth.normal_bf16(g, (8, N), 1.0)
    A = bits(np.eye(8, dtype=np.float32))
    O, Dp = oracle.gemm_rowscale_swiglu(A, B, want_preact=True)
    Bd = torch.from_numpy(wide(B))
    want = (torch.nn.functional.silu(Bd[:, 0::2]) * Bd[:, 1::2]).numpy()
    np.testing.assert_allclose(O, want, rtol=1e-13, atol=1e-15)
    assert np.array_equal(Dp, wide(B))
    # row scale applies BEFORE the split (Kernel 6)
    r = g.random(8) + 0.5
    O2 = oracle.gemm_rowscale_swiglu(A, B, r=r)
    Bs = Bd * torch.from_numpy(r)[:, None]
    want2 = (torch.nn.functional.silu(Bs[:, 0::2]) * Bs[:, 1::2]).numpy()
    np.testing.assert_allclose(O2, want2, rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- SwiGLU backward
def test_swiglu_backward_closed_form_points(oracle):
    for g, sig in golden_points():
        silu = g * sig
        dsilu = sig * (1.0 + g * (1.0 - sig))
        d, u = 0.7, -1.3
        dG, dU = oracle.swiglu_bwd_points(np.array([d]), np.array([g]), np.array([u]))
        assert abs(dU[0] - d * silu) <= 1e-15
        assert abs(dG[0] - d * u * dsilu) <= 1e-15
    dG, _ = oracle.swiglu_bwd_points(np.array([1.0]), np.array([0.0]), np.array([1.0]))
    assert dG[0] == 0.5                                   # silu'(0) = 1/2


def test_swiglu_backward_vs_autodiff_and_finite_differences(oracle):
    g = rng(11)
    n = 200
    gv, uv, dv = g.standard_normal(n) * 2, g.standard_normal(n), g.standard_normal(n)
    dG, dU = oracle.swiglu_bwd_points(dv, gv, uv)
    tg = torch.tensor(gv, requires_grad=True); tu = torch.tensor(uv, requires_grad=True)
    (torch.nn.functional.silu(tg) * tu * torch.tensor(dv)).sum().backward()
    np.testing.assert_allclose(dG, tg.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dU, tu.grad.numpy(), rtol=1e-12, atol=1e-14)
    h = 1e-6
    f = lambda a, b: oracle.swiglu_fwd_points(a, b)
    fdG = dv * (f(gv + h, uv) - f(gv - h, uv)) / (2 * h)
    fdU = dv * (f(gv, uv + h) - f(gv, uv - h)) / (2 * h)
    assert np.abs(fdG - dG).max() <= 1e-8 and np.abs(fdU - dU).max() <= 1e-8


def test_kernel10_layout_and_statistic(oracle):
    g = rng(12)
    M, N, K = 7, 10, 9
    A = synth.normal_bf16(g, (M, K), 1.0)
    Bt = synth.normal_bf16(g, (N, K), 1.0)        # stored [N x K], used transposed (D = A B^T)
    Z = synth.normal_bf16(g, (M, 2 * N), 1.0)
    dZ, O, stat = oracle.gemm_swiglu_bwd(A, Bt, Z, transB=True)
    D = wide(A) @ wide(Bt).T
    Zd = wide(Z)
    G, U = Zd[:, 0::2], Zd[:, 1::2]
    dGp, dUp = oracle.swiglu_bwd_points(D.ravel(), G.ravel(), U.ravel())
    np.testing.assert_allclose(dZ[:, 0::2], dGp.reshape(M, N), rtol=1e-13, atol=1e-15)   # even = dG
    np.testing.assert_allclose(dZ[:, 1::2], dUp.reshape(M, N), rtol=1e-13, atol=1e-15)   # odd  = dU
    np.testing.assert_allclose(O, oracle.swiglu_fwd_points(G.ravel(), U.ravel()).reshape(M, N), rtol=1e-14)
    np.testing.assert_allclose(stat, (Zd * dZ).sum(1), rtol=1e-12, atol=1e-14)           # sum Z*dZ
    # whole-kernel autodiff check: loss = <D, silu(G)*U> differentiated w.r.t. Z
    tz = torch.tensor(Zd, requires_grad=True)
    (torch.from_numpy(D) * torch.nn.functional.silu(tz[:, 0::2]) * tz[:, 1::2]).sum().backward()
    np.testing.assert_allclose(dZ, tz.grad.numpy(), rtol=1e-12, atol=1e-14)
    sel = oracle.gemm_swiglu_bwd(A, Bt, Z, transB=True, rows=np.array([5, 1]))
    np.testing.assert_allclose(sel[0], dZ[[5, 1]], rtol=0, atol=0)


def test_rmsnorm_backward_statistic_moves_across_the_gemm(oracle):
    # Section 3.2.1 (backward): sum_cols(grad_h2 * h2) == sum_cols(grad_y * y) with
    # y = h2 W1 and grad_h2 = grad_y W1^T.  Both sides via the oracle's contraction.
    g = rng(13)
    M, d, N = 5, 12, 9
    h2 = synth.normal_bf16(g, (M, d), 1.0)
    W1 = synth.normal_bf16(g, (d, N), 0.5)
    gy = synth.normal_bf16(g, (M, N), 1.0)
    y = oracle.gemm_rowscale(h2, W1)
    gh2 = oracle.gemm_rowscale(gy, W1, transB=True)
    lhs = (gh2 * wide(h2)).sum(1)
    rhs = (wide(gy) * y).sum(1)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- weight gradient
def test_weight_gradient_linearity_and_finite_differences(oracle):
    g = rng(14)
    T, F, d = 11, 6, 5                                # tokens, in-features, out-features
    H = synth.normal_bf16(g, (T, F), 1.0)
    dY = synth.normal_bf16(g, (T, d), 1.0)
    Gin = synth.normal_f32(g, (F, d), 1.0)
    base = oracle.gemm_accumulate(H, dY, None, transA=True)               # G_in = 0 -> H^T dY
    np.testing.assert_allclose(base, wide(H).T @ wide(dY), rtol=1e-13, atol=1e-14)
    acc = oracle.gemm_accumulate(H, dY, Gin, transA=True)
    np.testing.assert_allclose(acc - Gin.astype(np.float64), base, rtol=1e-12, atol=1e-13)
    dY2 = bits(2.0 * wide(dY).astype(np.float32))                         # doubling is exact in bf16
    np.testing.assert_allclose(oracle.gemm_accumulate(H, dY2, None, transA=True), 2.0 * base, rtol=1e-14)
    # d/dW <dY, H W> = H^T dY, by central differences on a few entries (the form is linear in W)
    Hd, dYd = wide(H), wide(dY)
    W = g.standard_normal((F, d))
    for (a, b) in [(0, 0), (3, 4), (5, 2)]:
        E = np.zeros_like(W); E[a, b] = 1e-3
        fd = ((dYd * (Hd @ (W + E))).sum() - (dYd * (Hd @ (W - E))).sum()) / 2e-3
        assert abs(fd - base[a, b]) <= 1e-9 * max(1.0, abs(base[a, b]))
    sel = oracle.gemm_accumulate(H, dY, Gin, transA=True, rows=np.array([4, 0]))
    np.testing.assert_allclose(sel, acc[[4, 0]], rtol=0, atol=0)


# ---------------------------------------------------------------- weight preparation
def test_weight_preparation_definitions(oracle):
    g = rng(15)
    Wa = synth.normal_bf16(g, (4, 6), 1.0); Wb = synth.normal_bf16(g, (4, 6), 1.0)
    W = oracle.interleave_pairs(Wa, Wb)
    assert np.array_equal(W[:, 0::2], Wa) and np.array_equal(W[:, 1::2], Wb)
    gamma = g.random(4) + 0.5
    np.testing.assert_allclose(oracle.fold_gamma(Wa, gamma), gamma[:, None] * wide(Wa), rtol=1e-15)


# ---------------------------------------------------------------- RoPE (Kernels 1 and 7)
def _rope_case(seed, M=9, K=6, heads=3, hd=8, extra=4, T=32):
    g = rng(seed)
    N = heads * hd + extra
    A = synth.normal_bf16(g, (M, K), 1.0)
    B = synth.normal_bf16(g, (K, N), 1.0)
    pos = g.integers(0, T, size=M).astype(np.int32)
    cos, sin = synth.rope_tables(T, hd)
    return A, B, pos, cos, sin, hd, heads * hd, N


def test_rope_vs_library_complex_multiplication(oracle):
    A, B, pos, cos, sin, hd, rc, N = _rope_case(16)
    got = oracle.gemm_rowscale_rope(A, B, cos, sin, pos, hd, rc)
    D = torch.from_numpy(wide(A) @ wide(B))
    z = torch.view_as_complex(D[:, :rc].reshape(len(pos), rc // hd, hd // 2, 2).contiguous())
    w = torch.complex(torch.from_numpy(cos[pos].astype(np.float64)), torch.from_numpy(sin[pos].astype(np.float64)))
    want = torch.view_as_real(z * w[:, None, :]).reshape(len(pos), rc)
    np.testing.assert_allclose(got[:, :rc], want.numpy(), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(got[:, rc:], D[:, rc:].numpy(), rtol=0, atol=0)          # pass-through columns


def test_rope_invariants(oracle):
    A, B, pos, cos, sin, hd, rc, N = _rope_case(17)
    M = len(pos)
    r = rng(18).random(M) + 0.5
    plain = oracle.gemm_rowscale(A, B, r=r)
    rot = oracle.gemm_rowscale_rope(A, B, cos, sin, pos, hd, rc, r=r)
    # a rotation preserves the norm of every pair (cos/sin are fp32 table values: c^2+s^2 = 1 to ~1e-7)
    n0 = plain[:, :rc].reshape(M, -1, 2)
    n1 = rot[:, :rc].reshape(M, -1, 2)
    np.testing.assert_allclose((n1 ** 2).sum(-1), (n0 ** 2).sum(-1), rtol=1e-6)
    # position 0 is the identity
    same = oracle.gemm_rowscale_rope(A, B, cos, sin, np.zeros(M, np.int32), hd, rc, r=r)
    np.testing.assert_allclose(same, plain, rtol=0, atol=0)
    # row selection and row scale indexed by the original row
    sel = oracle.gemm_rowscale_rope(A, B, cos, sin, pos, hd, rc, r=r, rows=np.array([7, 2]))
    np.testing.assert_allclose(sel, rot[[7, 2]], rtol=0, atol=0)
    # the sign convention: one-hot x0 = 1 at angle theta gives (cos, +sin)
    e = np.zeros((1, 2), np.float32); e[0, 0] = 1.0
    I2 = bits(np.eye(2, dtype=np.float32))
    c1, s1 = np.array([[0.6]], np.float32), np.array([[0.8]], np.float32)
    out = oracle.gemm_rowscale_rope(bits(e), I2, c1, s1, np.zeros(1, np.int32), 2, 2)
    np.testing.assert_allclose(out[0], [np.float32(0.6), np.float32(0.8)], rtol=1e-15)


def test_rope_relative_position_property(oracle):
    # <RoPE(q, m), RoPE(k, n)> depends on m - n only (exact-angle tables in fp64 would make this exact;
    # with fp32 tables it holds to ~1e-6)
    g = rng(19)
    hd, T = 16, 64
    cos, sin = synth.rope_tables(T, hd)
    I = bits(np.eye(hd, dtype=np.float32))
    q = synth.normal_bf16(g, (1, hd), 1.0); k = synth.normal_bf16(g, (1, hd), 1.0)
    def dot(m, n):
        a = oracle.gemm_rowscale_rope(q, I, cos, sin, np.array([m], np.int32), hd, hd)
        b = oracle.gemm_rowscale_rope(k, I, cos, sin, np.array([n], np.int32), hd, hd)
        return float((a * b).sum())
    assert abs(dot(5, 2) - dot(23, 20)) < 1e-5 and abs(dot(40, 47) - dot(3, 10)) < 1e-5
    assert abs(dot(5, 2) - dot(5, 3)) > 1e-3            # and it does depend on the offset


# ---------------------------------------------------------------- RMSNorm backward (Kernel 9)
def test_kernel9_vs_autodiff_of_library_rmsnorm(oracle):
    g = rng(20)
    M, d = 7, 24
    h1 = synth.normal_bf16(g, (M, d), 1.0)
    G2 = synth.normal_bf16(g, (M, d), 1.0)            # gradient w.r.t. the normalised activation
    Oin = synth.normal_bf16(g, (M, d), 1.0)
    gamma = g.random(d) + 0.5
    eps = 1e-6
    I = bits(np.eye(d, dtype=np.float32))
    th = torch.tensor(wide(h1), requires_grad=True)
    tg = torch.tensor(gamma, requires_grad=True)
    h2 = torch.nn.functional.rms_norm(th, (d,), weight=tg, eps=eps)
    (h2 * torch.from_numpy(wide(G2))).sum().backward()
    r = oracle.rstd(h1, eps)
    z = (wide(G2) * h2.detach().numpy()).sum(1) / d      # the row statistic, from the library's h2
    Oout, Cout, dg = oracle.gemm_rmsnorm_bwd(G2, I, h1, r, z, gamma, Oin=Oin)
    np.testing.assert_allclose(Oout - wide(Oin), th.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dg, tg.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(Cout, h2.detach().numpy(), rtol=1e-13, atol=1e-15)
    O2, _, dg2 = oracle.gemm_rmsnorm_bwd(G2, I, h1, r, z, gamma, rows=np.array([5, 1]))
    np.testing.assert_allclose(O2, (Oout - wide(Oin))[[5, 1]], rtol=1e-13, atol=1e-14)
    want = (wide(G2) * wide(h1) * r[:, None])[[5, 1]].sum(0)
    np.testing.assert_allclose(dg2, want, rtol=1e-13, atol=1e-14)


def test_kernel9_uses_the_gemm_result_with_transposed_weight(oracle):
    # D = grad_y W1^T: against an end-to-end autodiff through RMSNorm -> Linear
    g = rng(21)
    M, d, N = 6, 16, 10
    h1 = synth.normal_bf16(g, (M, d), 1.0)
    W1 = synth.normal_bf16(g, (d, N), 0.3)
    gy = synth.normal_bf16(g, (M, N), 1.0)
    gamma = g.random(d) + 0.5
    th = torch.tensor(wide(h1), requires_grad=True)
    y = torch.nn.functional.rms_norm(th, (d,), weight=torch.from_numpy(gamma), eps=1e-6) @ torch.from_numpy(wide(W1))
    (y * torch.from_numpy(wide(gy))).sum().backward()
    r = oracle.rstd(h1, 1e-6)
    z = (wide(gy) * y.detach().numpy()).sum(1) / d        # statistic taken AFTER the GEMM (Section 3.2.4 identity)
    Oout, _, _ = oracle.gemm_rmsnorm_bwd(gy, W1, h1, r, z, gamma, transB=True)
    np.testing.assert_allclose(Oout, th.grad.numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- cross-entropy pieces (Kernels 3 and 8)
def test_lse_kernel_vs_library_cross_entropy(oracle):
    g = rng(22)
    M, K, N = 9, 12, 40
    A = synth.normal_bf16(g, (M, K), 1.0)
    B = synth.normal_bf16(g, (K, N), 1.0)
    y = g.integers(0, N, size=M).astype(np.int32)
    r = g.random(M) + 0.5
    Z, zt, lse = oracle.gemm_rowscale_lse(A, B, y, r=r)
    Zt = torch.from_numpy((wide(A) @ wide(B)) * r[:, None])
    np.testing.assert_allclose(Z, Zt.numpy(), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse, torch.logsumexp(Zt, dim=1).numpy(), rtol=1e-13)
    np.testing.assert_allclose(zt, Zt.numpy()[np.arange(M), y], rtol=0, atol=0)
    loss = torch.nn.functional.cross_entropy(Zt, torch.from_numpy(y.astype(np.int64)), reduction="none").numpy()
    np.testing.assert_allclose(lse - zt, loss, rtol=1e-12, atol=1e-13)          # Section 3.2.3: l_i = -h_{i,y_i} + log sum exp
    sel = oracle.gemm_rowscale_lse(A, B, y, r=r, rows=np.array([8, 3]))
    np.testing.assert_allclose(sel[2], lse[[8, 3]], rtol=0, atol=0)
    np.testing.assert_allclose(sel[1], zt[[8, 3]], rtol=0, atol=0)


def test_lse_closed_forms(oracle):
    # all logits equal c  ->  lse = c + log N ; huge logits do not overflow ; one dominant logit -> lse ~ that logit
    N = 64
    I = bits(np.eye(N, dtype=np.float32))
    rowc = bits(np.full((1, N), 3.0, np.float32))
    y0 = np.zeros(1, np.int32)
    _, zt, lse = oracle.gemm_rowscale_lse(rowc, I, y0)
    assert abs(lse[0] - (3.0 + math.log(N))) < 1e-14 and zt[0] == 3.0
    big = np.full((1, N), -1000.0, np.float32); big[0, 7] = 900.0
    _, zt, lse = oracle.gemm_rowscale_lse(bits(big), I, np.array([7], np.int32))
    assert lse[0] == 900.0 and zt[0] == 900.0            # exp(-1900) underflows to exactly 0
    # scaling the row by r scales every logit: lse(r*z) for r = 2 on the constant row
    _, _, lse2 = oracle.gemm_rowscale_lse(rowc, I, y0, r=np.array([2.0]))
    assert abs(lse2[0] - (6.0 + math.log(N))) < 1e-14


# ---- 8-bit operands (OCP E4M3) --------------------------------------------------------------------------------
def test_f8e4m3_decoder_named_values(oracle):
    """Values the OFP8 specification names for E4M3: bias 7, max normal 448 (0x7E), min normal 2^-6 (0x08), max
    subnormal 0.875 * 2^-6 (0x07), min subnormal 2^-9 (0x01), no infinities, S.1111.111 = NaN, signed zeros."""
    dec = lambda codes: oracle.bf16_bits_to_f64(oracle.f8e4m3_to_bf16_bits(np.array(codes, dtype=np.uint8)))
    named = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 0.875 * 2.0 ** -6, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125, 0x3C: 1.5,
             0x40: 2.0, 0x77: 240.0, 0x78: 256.0, 0x7E: 448.0, 0xB8: -1.0, 0xC0: -2.0, 0xFE: -448.0}
    got = dec(list(named.keys()))
    assert np.array_equal(got, np.array(list(named.values())))
    assert np.isnan(dec([0x7F, 0xFF])).all()
    assert np.signbit(dec([0x80]))[0] and dec([0x80])[0] == 0.0
    pos = dec(list(range(0x7F)))
    assert (np.diff(pos) > 0).all(), "codes 0x00..0x7E must be strictly increasing"
    assert np.array_equal(dec(list(range(0x80, 0xFF))), -pos)


def test_f8e4m3_decoder_vs_library_all_codes(oracle):
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.bf16_bits_to_f64(oracle.f8e4m3_to_bf16_bits(codes))
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(lib))
    ok = ~np.isnan(lib)
    assert np.array_equal(got[ok], lib[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(lib[ok]))


def test_f8e4m3_input_rounding_is_rne_and_round_trips(oracle):
    """The seeded generator's storage rounding: every finite code survives decode -> encode, ties go to the even
    mantissa, values beyond 448 saturate, and the rounding agrees with a library conversion on random draws."""
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    vals = oracle.bf16_bits_to_f64(oracle.f8e4m3_to_bf16_bits(codes))
    assert np.array_equal(synth.f32_to_f8e4m3_bits(vals.astype(np.float32)), codes)
    ties = np.array([1.0625, 1.1875, -1.0625, 2.0 ** -10, 3 * 2.0 ** -10], dtype=np.float32)   # midpoints of neighbours
    assert list(synth.f32_to_f8e4m3_bits(ties)) == [0x38, 0x3A, 0xB8, 0x00, 0x02]
    assert list(synth.f32_to_f8e4m3_bits(np.array([449.0, 1e6, -1e6], dtype=np.float32))) == [0x7E, 0x7E, 0xFE]
    x = (np.random.Generator(np.random.PCG64(3)).standard_normal(100000) * 2.5).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(synth.f32_to_f8e4m3_bits(x), lib)


def test_gemm_on_f8e4m3_operands_is_the_gemm_of_their_values(oracle):
    g = np.random.Generator(np.random.PCG64(4))
    A8, B8 = synth.normal_f8e4m3(g, (24, 40), 1.0), synth.normal_f8e4m3(g, (16, 40), 1.0)
    got = oracle.gemm_rowscale(oracle.f8e4m3_to_bf16_bits(A8), oracle.f8e4m3_to_bf16_bits(B8), transB=True)
    Af = torch.from_numpy(A8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    Bf = torch.from_numpy(B8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_allclose(got, Af @ Bf.T, rtol=1e-13, atol=1e-13)
