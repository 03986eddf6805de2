"""GPU parity: every entry point of libcoda.so, called through the C ABI, against the CPU
oracle on the same seeded inputs, element by element.  Sizes span several 256x256x64 tiles
plus ragged tails in every dimension; outputs sit in sentinel-guarded buffers."""
import numpy as np
import pytest
import torch

from paper_2605_19269_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

coda = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global coda
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_19269_amd import coda as _c
    coda = _c
    yield
    torch.cuda.synchronize()


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def operands(g, M, N, K, transA, transB, a_std=1.0, b_std=0.5):
    """Random bf16 operands as stored for the requested layout; returns (A_bits, B_bits)."""
    A = synth.normal_bf16(g, (K, M) if transA else (M, K), a_std)
    B = synth.normal_bf16(g, (N, K) if transB else (K, N), b_std)
    return A, B


SHAPES = [(256, 256, 64), (512, 768, 192), (520, 776, 200), (8, 8, 8), (264, 40, 72)]
LAYOUTS = [(False, False), (False, True), (True, False), (True, True)]


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_plain_gemm_store_bf16(oracle, M, N, K, transA, transB):
    g = rng(100 + M + N + K)
    A, B = operands(g, M, N, K, transA, transB)
    out = G.Guarded(M, N, torch.bfloat16)
    dA, dB = G.dev_bf16(A), G.dev_bf16(B)
    coda.coda_gemm(dA, dB, [coda.store(out.t)], transA=transA, transB=transB)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale(A, B, transA=transA, transB=transB)
    out.check_guards(); out.written()
    G.assert_bf16_close(G.host_f64(out.t), ref, "plain gemm")


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("K", [128, 192, 256, 320, 384, 448, 512, 640, 704])
def test_k_loop_lengths_whole_tiles(oracle, K, transA, transB):
    """K-step counts 4 .. 22 on whole tiles: the ring fill alone, the run-dry steps alone, and one to several trips of the
    steady loop with its waves a phase apart, in all four layouts; fp32 output, so no rounding hides a dropped K-step."""
    M, N = 256, 512
    g = rng(7000 + K)
    A, B = operands(g, M, N, K, transA, transB)
    out = G.Guarded(M, N, torch.float32, pad_cols=4)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.store(out.t, f32=True)], transA=transA, transB=transB)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale(A, B, transA=transA, transB=transB)
    out.check_guards(); out.written()
    got = G.host_f64(out.t)
    scale = np.sqrt(K) * 0.5
    assert np.abs(got - ref).max() <= 2e-5 * scale * 8, "max |delta| %.3g" % np.abs(got - ref).max()


def _random_ragged_cases(n, seed):
    """Seeded shapes around the tile boundaries: M any (a multiple of 8 when A is stored transposed), N and K multiples
    of 8; K below, at and just past multiples of the 32 / 64-element K-steps; one layout and one pitch padding each."""
    g = np.random.Generator(np.random.PCG64(seed))
    cases = []
    for i in range(n):
        transA, transB = bool(g.integers(2)), bool(g.integers(2))
        M = int(g.choice([1, 7, 8, 255, 256, 257, 300, 511, 520]))
        if transA:
            M = max(8, M // 8 * 8)
        N = int(g.choice([8, 24, 248, 256, 264, 504, 520]))
        K = int(g.choice([8, 24, 32, 40, 56, 64, 72, 120, 128, 136, 184, 192, 200, 320, 328]))
        cases.append((M, N, K, transA, transB, int(g.choice([0, 8, 24]))))
    return cases


@pytest.mark.parametrize("M,N,K,transA,transB,pad", _random_ragged_cases(28, seed=2024))
def test_ragged_shapes_residual_sumsq(oracle, M, N, K, transA, transB, pad):
    """Ragged M / N / K through the one mainloop (clamped edge fetches, zero-filled K tail), padded operand pitches,
    guarded outputs: row scale + residual + row sum of squares against the oracle."""
    g = rng(4000 + 7 * M + 3 * N + K + 2 * transA + transB)
    a_shape, b_shape = ((K, M) if transA else (M, K)), ((N, K) if transB else (K, N))
    Ap = synth.normal_bf16(g, (a_shape[0], a_shape[1] + pad), 1.0)
    Bp = synth.normal_bf16(g, (b_shape[0], b_shape[1] + pad), 0.3)
    A, B = np.ascontiguousarray(Ap[:, :a_shape[1]]), np.ascontiguousarray(Bp[:, :b_shape[1]])
    dA, dB = G.dev_bf16(Ap)[:, :a_shape[1]], G.dev_bf16(Bp)[:, :b_shape[1]]      # pitch > width
    C = synth.normal_bf16(g, (M, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    Y = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dr, dC = G.dev_f32(r), G.dev_bf16(C)
    coda.coda_gemm(dA, dB, [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y.t)],
                   transA=transA, transB=transB)
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
    torch.cuda.synchronize()
    refD, refss = oracle.gemm_residual_sumsq(A, B, r=r.astype(np.float64), C=C, transA=transA, transB=transB)[:2]
    Y.check_guards(); Y.written()
    G.assert_bf16_close(G.host_f64(Y.t), refD, "ragged row scale + residual")
    G.assert_sumsq_close(G.host_f64(ss), refss, "ragged row sum of squares")


@pytest.mark.parametrize("transA,transB", [(False, False), (True, False)])
def test_plain_gemm_store_f32(oracle, transA, transB):
    M, N, K = 520, 264, 136
    g = rng(7)
    A, B = operands(g, M, N, K, transA, transB)
    out = G.Guarded(M, N, torch.float32, pad_cols=4)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.store(out.t, f32=True)], transA=transA, transB=transB)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale(A, B, transA=transA, transB=transB)
    out.check_guards(); out.written()
    G.assert_f32_signed_close(G.host_f64(out.t), ref, "f32 store")


@pytest.mark.parametrize("M,N,K", [(512, 512, 128), (520, 776, 200)])
@pytest.mark.parametrize("transB", [False, True])
def test_kernel5_row_scale(oracle, M, N, K, transB):
    g = rng(11)
    A, B = operands(g, M, N, K, False, transB)
    r = synth.uniform_f32(g, (M,), 0.25, 2.0)
    out = G.Guarded(M, N, torch.bfloat16)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.row_scale(G.dev_f32(r)), coda.store(out.t)], transB=transB)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale(A, B, r=r.astype(np.float64), transB=transB)
    out.check_guards(); out.written()
    G.assert_bf16_close(G.host_f64(out.t), ref, "row scale")


@pytest.mark.parametrize("M,N,K", [(512, 512, 128), (520, 776, 200)])
@pytest.mark.parametrize("with_r,with_preact", [(True, False), (False, True), (True, True)])
def test_kernel6_swiglu_forward(oracle, M, N, K, with_r, with_preact):
    g = rng(12)
    A, B = operands(g, M, N, K, False, False, b_std=0.2)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5) if with_r else None
    H = G.Guarded(M, N // 2, torch.bfloat16)
    Z = G.Guarded(M, N, torch.bfloat16) if with_preact else None
    ops = ([coda.row_scale(dr := G.dev_f32(r))] if with_r else []) + \
          [coda.swiglu_fwd(Z.t if Z else None), coda.store(H.t)]
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), ops)
    torch.cuda.synchronize()
    refH, refZ = oracle.gemm_rowscale_swiglu(A, B, r=None if r is None else r.astype(np.float64), want_preact=True)
    H.check_guards(); H.written()
    G.assert_bf16_close(G.host_f64(H.t), refH, "swiglu fwd")
    if Z:
        Z.check_guards(); Z.written()
        G.assert_bf16_close(G.host_f64(Z.t), refZ, "pre-activation side output")


@pytest.mark.parametrize("M,N,K", [(512, 512, 128), (520, 776, 200)])
@pytest.mark.parametrize("atomic", [False, True])
@pytest.mark.parametrize("transB", [False, True])
def test_kernel4_residual_sumsq_gamma(oracle, M, N, K, atomic, transB):
    g = rng(13)
    A, B = operands(g, M, N, K, False, transB, b_std=0.1)
    C = synth.normal_bf16(g, (M, N), 1.0)
    gamma = synth.uniform_f32(g, (N,), 0.5, 1.5)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    Y = G.Guarded(M, N, torch.bfloat16)
    O = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    red = torch.zeros(M, dtype=torch.float32, device="cuda") if atomic else \
        torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dr, dC, dg = G.dev_f32(r), G.dev_bf16(C), G.dev_f32(gamma)
    ops = [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(red, atomic=atomic),
           coda.col_scale_side(dg, O.t), coda.store(Y.t)]
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), ops, transB=transB)
    if atomic:
        ss = red
    else:
        ss = torch.empty(M, dtype=torch.float32, device="cuda")
        coda.coda_row_finalize(red, M, nblk, sum_out=ss, d=N, eps=0.0)
    torch.cuda.synchronize()
    refD, refss, refO = oracle.gemm_residual_sumsq(A, B, r=r.astype(np.float64), C=C, gamma=gamma.astype(np.float64),
                                                   transB=transB, want_scaled=True)
    Y.check_guards(); Y.written(); O.check_guards(); O.written()
    G.assert_bf16_close(G.host_f64(Y.t), refD, "residual output")
    G.assert_bf16_close(G.host_f64(O.t), refO, "gamma-scaled side output")
    G.assert_sumsq_close(G.host_f64(ss), refss, "row sum of squares")


@pytest.mark.parametrize("M,N,K", [(512, 256, 128), (520, 264, 200)])
@pytest.mark.parametrize("extras", [False, True])
def test_kernel10_swiglu_backward(oracle, M, N, K, extras):
    g = rng(14)
    A = synth.normal_bf16(g, (M, K), 1e-2)
    Bt = synth.normal_bf16(g, (N, K), 0.02)          # W_down stored [F x d], used transposed
    Z = synth.normal_bf16(g, (M, 2 * N), 1.0)
    dZ = G.Guarded(M, 2 * N, torch.bfloat16)
    O = G.Guarded(M, N, torch.bfloat16) if extras else None
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda") if extras else None
    dZin = G.dev_bf16(Z)
    ops = [coda.swiglu_bwd(dZin, act_out=O.t if O else None, stat_out=part), coda.store(dZ.t)]
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(Bt), ops, transB=True)
    torch.cuda.synchronize()
    refdZ, refO, refstat = oracle.gemm_swiglu_bwd(A, Bt, Z, transB=True)
    dZ.check_guards(); dZ.written()
    G.assert_bf16_close(G.host_f64(dZ.t), refdZ, "dZ")
    if extras:
        O.check_guards(); O.written()
        G.assert_bf16_close(G.host_f64(O.t), refO, "recomputed activation")
        stat = torch.empty(M, dtype=torch.float32, device="cuda")
        coda.coda_row_finalize(part, M, nblk, sum_out=stat, d=1, eps=0.0)
        torch.cuda.synchronize()
        G.assert_f32_signed_close(G.host_f64(stat), refstat, "row statistic")


@pytest.mark.parametrize("M,N,K", [(512, 256, 256), (264, 520, 200)])
def test_weight_gradient_accumulate(oracle, M, N, K):
    g = rng(15)
    H = synth.normal_bf16(g, (K, M), 1.0)             # activations [tokens x in], used transposed
    dY = synth.normal_bf16(g, (K, N), 1e-2)
    Gin = synth.normal_f32(g, (M, N), 1e-3)
    buf = G.Guarded(M, N, torch.float32, pad_cols=4)
    buf.t.copy_(torch.from_numpy(Gin))
    buf.ref = buf.full.clone()
    coda.coda_gemm(G.dev_bf16(H), G.dev_bf16(dY), [coda.accum_f32(buf.t)], transA=True)
    torch.cuda.synchronize()
    ref = oracle.gemm_accumulate(H, dY, Gin, transA=True)
    buf.check_guards()
    G.assert_f32_signed_close(G.host_f64(buf.t), ref, "accumulated weight gradient")
    # second accumulation on top of the first (in-place semantics)
    coda.coda_gemm(G.dev_bf16(H), G.dev_bf16(dY), [coda.accum_f32(buf.t)], transA=True)
    torch.cuda.synchronize()
    ref2 = ref + oracle.gemm_accumulate(H, dY, None, transA=True)
    G.assert_f32_signed_close(G.host_f64(buf.t), ref2, "second accumulation")


def test_tiny_rmsnorm_gemm_configuration(oracle):
    """The tiny configuration end to end on the GPU: row_sumsq -> finalize(rstd) ; fold_gamma ;
    GEMM with [row scale, residual add, sum of squares, store]; against the canonical
    RMSNorm -> GEMM -> residual chain of the oracle."""
    c = synth.tiny_rmsnorm_gemm(seed=0)
    M, K = c["X"].shape
    N = c["W"].shape[1]
    X, W, R, gamma = G.dev_bf16(c["X"]), G.dev_bf16(c["W"]), G.dev_bf16(c["R"]), G.dev_f32(c["gamma"])
    ssx = torch.empty(M, dtype=torch.float32, device="cuda")
    rstd = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_sumsq(X, ssx)
    coda.coda_row_finalize(ssx.view(1, M), M, 1, rstd_out=rstd, d=K, eps=c["eps"])
    Wp = torch.empty_like(W)
    coda.coda_fold_gamma(W, gamma, Wp)
    Y = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.empty((nblk, M), dtype=torch.float32, device="cuda")
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_gemm(X, Wp, [coda.row_scale(rstd), coda.add_tile(R), coda.row_sumsq(part), coda.store(Y.t)])
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
    torch.cuda.synchronize()
    refY, refss = oracle.rmsnorm_linear_unfused(c["X"], c["gamma"].astype(np.float64), c["eps"], c["W"], c["R"])
    Y.check_guards(); Y.written()
    G.assert_sumsq_close(G.host_f64(rstd), oracle.rstd(c["X"], c["eps"]), "rstd")
    G.assert_bf16_close(G.host_f64(Y.t), refY, "Y")
    G.assert_sumsq_close(G.host_f64(ss), refss, "sum of squares of Y")


def test_mlp_block_chain(oracle):
    """RMSNorm -> up-projection+SwiGLU -> down-projection+residual+sum of squares, three fused
    launches plus the auxiliary reductions, against the unfused fp64 operator chain."""
    g = rng(21)
    M, d, F = 384, 256, 512
    Xb = synth.normal_bf16(g, (M, d), 1.0)
    gamma = synth.uniform_f32(g, (d,), 0.5, 1.5)
    W1 = synth.normal_bf16(g, (d, 2 * F), 0.08)
    W2 = synth.normal_bf16(g, (F, d), 0.08)
    X, dW1, dW2, dg = G.dev_bf16(Xb), G.dev_bf16(W1), G.dev_bf16(W2), G.dev_f32(gamma)
    ssx = torch.empty(M, dtype=torch.float32, device="cuda")
    rstd = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_sumsq(X, ssx)
    coda.coda_row_finalize(ssx.view(1, M), M, 1, rstd_out=rstd, d=d, eps=1e-6)
    W1p = torch.empty_like(dW1)
    coda.coda_fold_gamma(dW1, dg, W1p)
    H = torch.empty((M, F), dtype=torch.bfloat16, device="cuda")
    coda.coda_gemm(X, W1p, [coda.row_scale(rstd), coda.swiglu_fwd(), coda.store(H)])
    Y = torch.empty((M, d), dtype=torch.bfloat16, device="cuda")
    nblk = coda.coda_row_partial_blocks(d)
    part = torch.empty((nblk, M), dtype=torch.float32, device="cuda")
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_gemm(H, dW2, [coda.add_tile(X), coda.row_sumsq(part), coda.store(Y)])
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=d, eps=0.0)
    torch.cuda.synchronize()
    refY, refss = oracle.mlp_block(Xb, gamma.astype(np.float64), 1e-6, W1, W2, R=Xb, reparam=False)
    # two bf16 intermediates (folded weight, H) lie between the input and Y: chain tolerance
    G.assert_chain_close(G.host_f64(Y), refY, "block output")
    # the row statistic inherits the chain error of Y (about 0.3% rms per element, partly
    # correlated along a row through rstd and the folded weight): 1e-2 relative
    rel = np.abs(G.host_f64(ss) - refss) / refss
    assert rel.max() <= 1e-2, "block sum of squares: max relative error %.3g" % rel.max()


def test_mlp_block_chain_stage_by_stage(oracle):
    """The same three launches, each held to the single-kernel bar: every stage's oracle gets the bytes that the GPU
    stage before it actually stored (the fp32 rstd, the folded bf16 weight, the bf16 H), so no rounding of an earlier
    stage is left for the tolerance to absorb."""
    g = rng(21)
    M, d, F = 384, 256, 512
    Xb = synth.normal_bf16(g, (M, d), 1.0)
    gamma = synth.uniform_f32(g, (d,), 0.5, 1.5)
    W1 = synth.normal_bf16(g, (d, 2 * F), 0.08)
    W2 = synth.normal_bf16(g, (F, d), 0.08)
    X, dW1, dW2, dg = G.dev_bf16(Xb), G.dev_bf16(W1), G.dev_bf16(W2), G.dev_f32(gamma)
    ssx = torch.empty(M, dtype=torch.float32, device="cuda")
    rstd = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_sumsq(X, ssx)
    coda.coda_row_finalize(ssx.view(1, M), M, 1, rstd_out=rstd, d=d, eps=1e-6)
    W1p = torch.empty_like(dW1)
    coda.coda_fold_gamma(dW1, dg, W1p)
    H = G.Guarded(M, F, torch.bfloat16)
    coda.coda_gemm(X, W1p, [coda.row_scale(rstd), coda.swiglu_fwd(), coda.store(H.t)])
    Y = G.Guarded(M, d, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(d)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_gemm(H.t, dW2, [coda.add_tile(X), coda.row_sumsq(part), coda.store(Y.t)])
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=d, eps=0.0)
    torch.cuda.synchronize()
    H.check_guards(); H.written(); Y.check_guards(); Y.written()
    # stage 1: the row statistic
    G.assert_sumsq_close(G.host_f64(rstd), oracle.rstd(Xb, 1e-6), "stage rstd")
    # stage 2: the folded weight, one rounding of the exact product
    W1p_bits = G.host_bits(W1p)
    G.assert_bf16_close(G.bits_to_f64(W1p_bits), oracle.fold_gamma(W1, gamma.astype(np.float64)), "stage folded weight")
    # stage 3: up-projection on the GPU's own rstd and folded weight
    refH = oracle.gemm_rowscale_swiglu(Xb, W1p_bits, r=G.host_f64(rstd))
    G.assert_bf16_close(G.host_f64(H.t), refH, "stage H")
    # stage 4: down-projection on the GPU's own stored H
    refY, refss = oracle.gemm_residual_sumsq(np.ascontiguousarray(G.host_bits(H.t)), W2, C=Xb)[:2]
    G.assert_bf16_close(G.host_f64(Y.t), refY, "stage Y")
    G.assert_sumsq_close(G.host_f64(ss), refss, "stage sum of squares")


@pytest.mark.parametrize("atomic", [False, True])
def test_backward_chain_kernel10_statistic_into_kernel9(oracle, atomic):
    """Kernel 10's row statistic feeds Kernel 9 end to end: dY W_down^T with SwiGLU backward leaves dZ and the row sums
    sum_j (g dG + u dU); the auxiliary combine adds the tile partials; Kernel 9 (dZ W1^T with the local RMSNorm backward)
    reads those raw sums and divides by the hidden size itself.  The oracle takes the same chain in fp64, with the
    GPU's stored dZ as Kernel 9's operand so that the second stage is held to the single-kernel bar."""
    g = rng(83)
    M, dm, F = 520, 264, 256
    dYb = synth.normal_bf16(g, (M, dm), 0.5)
    Wd = synth.normal_bf16(g, (F, dm), 0.1)              # down-projection weight [F x d], used transposed
    Zb = synth.normal_bf16(g, (M, 2 * F), 1.0)
    W1 = synth.normal_bf16(g, (dm, 2 * F), 0.1)          # up-projection weight [d x 2F], used transposed
    h1 = synth.normal_bf16(g, (M, dm), 1.0)              # the RMSNorm input
    Oin = synth.normal_bf16(g, (M, dm), 0.5)
    gamma = synth.uniform_f32(g, (dm,), 0.5, 1.5)
    r = oracle.rstd(h1, 1e-6).astype(np.float32)
    # Kernel 10
    dZ = G.Guarded(M, 2 * F, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(F)
    stat = torch.zeros(M, dtype=torch.float32, device="cuda") if atomic else \
        torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dZz = G.dev_bf16(Zb)
    coda.coda_gemm(G.dev_bf16(dYb), G.dev_bf16(Wd), [coda.swiglu_bwd(dZz, stat_out=stat, atomic=atomic), coda.store(dZ.t)], transB=True)
    if atomic:
        zsum = stat
    else:
        zsum = torch.empty(M, dtype=torch.float32, device="cuda")
        coda.coda_row_finalize(stat, M, nblk, sum_out=zsum, d=1, eps=0.0)
    # Kernel 9 on the stored dZ, z = zsum / d formed in the kernel
    Oout, Cout = G.Guarded(M, dm, torch.bfloat16), G.Guarded(M, dm, torch.bfloat16)
    nb2 = coda.coda_col_partial_blocks(M)
    dgp = torch.full((nb2, dm), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dgam = torch.empty(dm, dtype=torch.float32, device="cuda")
    dh1, dr, dgm, dO = G.dev_bf16(h1), G.dev_f32(r), G.dev_f32(gamma), G.dev_bf16(Oin)
    coda.coda_gemm(dZ.t, G.dev_bf16(W1),
                   [coda.rmsnorm_bwd(dh1, dr, zsum, dgm, c_out=Cout.t, dgamma_out=dgp, z_sum_over=dm), coda.add_tile(dO), coda.store(Oout.t)],
                   transB=True)
    coda.coda_col_finalize(dgp, dm, nb2, dgam)
    torch.cuda.synchronize()
    for t in (dZ, Oout, Cout):
        t.check_guards(); t.written()
    refdZ, _, refstat = oracle.gemm_swiglu_bwd(dYb, Wd, Zb, transB=True)
    G.assert_bf16_close(G.host_f64(dZ.t), refdZ, "chain dZ")
    G.assert_f32_signed_close(G.host_f64(zsum), refstat, "chain row statistic")
    dZ_bits = np.ascontiguousarray(G.host_bits(dZ.t))
    refO, refC, refdg = oracle.gemm_rmsnorm_bwd(dZ_bits, W1, h1, r.astype(np.float64), refstat / dm, gamma.astype(np.float64),
                                                Oin=Oin, transB=True)
    G.assert_bf16_close(G.host_f64(Oout.t), refO, "chain O_out")
    G.assert_bf16_close(G.host_f64(Cout.t), refC, "chain C_out")
    G.assert_f32_signed_close(G.host_f64(dgam), refdg, "chain dgamma")


def test_aux_kernels(oracle):
    g = rng(31)
    M, K = 37, 264
    Xb = synth.normal_bf16(g, (M, K + 8), 1.0)[:, :K]    # pitch > width
    X = G.dev_bf16(np.ascontiguousarray(synth.normal_bf16(g, (M, K + 8), 1.0)))
    Xv = X[:, :K]
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_sumsq(Xv, ss)
    torch.cuda.synchronize()
    G.assert_sumsq_close(G.host_f64(ss), oracle.row_sumsq(np.ascontiguousarray(G.host_bits(Xv))), "row_sumsq")
    # finalize over several blocks
    nblk = 5
    part = synth.uniform_f32(g, (nblk, M), 0.0, 4.0)
    s_out = torch.empty(M, dtype=torch.float32, device="cuda")
    r_out = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(G.dev_f32(part), M, nblk, sum_out=s_out, rstd_out=r_out, d=K, eps=1e-6)
    torch.cuda.synchronize()
    tot = part.astype(np.float64).sum(0)
    G.assert_sumsq_close(G.host_f64(s_out), tot, "finalize sum")
    G.assert_sumsq_close(G.host_f64(r_out), oracle.rstd_from_sumsq(tot, K, 1e-6), "finalize rstd")
    # weight preparation
    Wa, Wb = synth.normal_bf16(g, (24, 40), 1.0), synth.normal_bf16(g, (24, 40), 1.0)
    out = G.Guarded(24, 80, torch.bfloat16)
    coda.coda_interleave_pairs(G.dev_bf16(Wa), G.dev_bf16(Wb), out.t)
    torch.cuda.synchronize()
    out.check_guards()
    assert np.array_equal(G.host_bits(out.t), oracle.interleave_pairs(Wa, Wb))       # bit-exact
    gamma = synth.uniform_f32(g, (24,), 0.5, 1.5)
    fo = G.Guarded(24, 40, torch.bfloat16)
    coda.coda_fold_gamma(G.dev_bf16(Wa), G.dev_f32(gamma), fo.t)
    torch.cuda.synchronize()
    fo.check_guards()
    want = synth.f32_to_bf16_bits(oracle.fold_gamma(Wa, gamma.astype(np.float64)).astype(np.float32))
    # product of a bf16 and an fp32 value is exact in fp64 and needs <= 32 significant bits, so
    # rounding it through fp32 first can differ from direct rounding only at double-rounding ties
    got = G.host_bits(fo.t)
    assert (got != want).mean() < 1e-3
    G.assert_bf16_close(G.bits_to_f64(got), oracle.fold_gamma(Wa, gamma.astype(np.float64)), "fold_gamma")
    del Xb


def test_degenerate_sizes(oracle):
    g = rng(41)
    # K == 0: the program runs on D = 0  ->  Y = R, ss = rowsum(R^2)
    M, N = 264, 264
    A = torch.empty((M, 0), dtype=torch.bfloat16, device="cuda")
    B = torch.empty((0, N), dtype=torch.bfloat16, device="cuda")
    Rb = synth.normal_bf16(g, (M, N), 1.0)
    Y = G.Guarded(M, N, torch.bfloat16)
    ss = torch.zeros(M, dtype=torch.float32, device="cuda")
    st = coda.coda_gemm_raw(0, M, N, 0, coda.coda_mat(A.data_ptr(), M, 0, 8, 0, 0), coda.coda_mat(B.data_ptr(), 0, N, N, 0, 0),
                            [coda.add_tile(dR := G.dev_bf16(Rb)), coda.row_sumsq(ss, atomic=True), coda.store(Y.t)])
    assert st == coda.CODA_OK
    torch.cuda.synchronize()
    Y.check_guards(); Y.written()
    assert np.array_equal(G.host_bits(Y.t), Rb)
    G.assert_sumsq_close(G.host_f64(ss), (G.bits_to_f64(Rb) ** 2).sum(1), "K=0 sumsq")
    # M == 0 and N == 0 are no-ops that still validate
    out = torch.empty((8, 8), dtype=torch.bfloat16, device="cuda")
    a0 = coda.coda_mat(out.data_ptr(), 0, 8, 8, 0, 0)
    b0 = coda.coda_mat(out.data_ptr(), 8, 8, 8, 0, 0)
    assert coda.coda_gemm_raw(0, 0, 8, 8, a0, b0, [coda.store(out)]) == coda.CODA_OK


def test_unfused_baseline_kernels(oracle):
    """The stand-alone kernels of the unfused chain (measurement baseline) against the same
    definitions of the oracle (GEMM replaced by an identity so the oracle's epilogue is isolated)."""
    g = rng(51)
    M, F = 70, 264
    Zb = synth.normal_bf16(g, (M, 2 * F), 1.0)
    dHb = synth.normal_bf16(g, (M, F), 1e-2)
    eyeF = synth.f32_to_bf16_bits(np.eye(F, dtype=np.float32))
    # forward: Z -> H   (oracle: Kernel 2 with A = Z, B = I)
    H = G.Guarded(M, F, torch.bfloat16)
    coda.coda_unfused_swiglu_fwd(G.dev_bf16(Zb), H.t)
    eye2F = synth.f32_to_bf16_bits(np.eye(2 * F, dtype=np.float32))
    refH = oracle.gemm_rowscale_swiglu(Zb, eye2F)
    # backward: (dH, Z) -> dZ   (oracle: Kernel 10 with A = dH, B = I)
    dZ = G.Guarded(M, 2 * F, torch.bfloat16)
    coda.coda_unfused_swiglu_bwd(G.dev_bf16(dHb), G.dev_bf16(Zb), dZ.t)
    refdZ, _, _ = oracle.gemm_swiglu_bwd(dHb, eyeF, Zb)
    # residual add + sum of squares   (oracle: Kernel 4 with A = D, B = I)
    Db, Rb = synth.normal_bf16(g, (M, F), 1.0), synth.normal_bf16(g, (M, F), 1.0)
    Y = G.Guarded(M, F, torch.bfloat16)
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_unfused_add_sumsq(G.dev_bf16(Db), G.dev_bf16(Rb), Y.t, ss)
    refY, refss = oracle.gemm_residual_sumsq(Db, eyeF, C=Rb)
    # RMSNorm apply: Xn = X * r * gamma   (oracle: Kernel 5 on X diag(gamma) is not bf16-exact, so
    # compare against the exact product formed from the oracle's widened inputs)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5); gamma = synth.uniform_f32(g, (F,), 0.5, 1.5)
    Xn = G.Guarded(M, F, torch.bfloat16)
    coda.coda_unfused_rmsnorm_apply(G.dev_bf16(Db), G.dev_f32(r), G.dev_f32(gamma), Xn.t)
    refXn = oracle.gemm_rowscale(Db, eyeF, r=r.astype(np.float64)) * gamma.astype(np.float64)[None, :]
    # fp32 accumulate
    T, G0 = synth.normal_f32(g, (M, F), 1.0), synth.normal_f32(g, (M, F), 1.0)
    Gd = G.dev_f32(G0)
    coda.coda_unfused_accumulate(G.dev_f32(T), Gd)
    torch.cuda.synchronize()
    for buf in (H, dZ, Y, Xn):
        buf.check_guards(); buf.written()
    G.assert_bf16_close(G.host_f64(H.t), refH, "unfused swiglu fwd")
    G.assert_bf16_close(G.host_f64(dZ.t), refdZ, "unfused swiglu bwd")
    G.assert_bf16_close(G.host_f64(Y.t), refY, "unfused add")
    G.assert_sumsq_close(G.host_f64(ss), refss, "unfused sumsq")
    G.assert_bf16_close(G.host_f64(Xn.t), refXn, "unfused rmsnorm apply")
    assert np.array_equal(Gd.cpu().numpy(), G0 + T)          # one fp32 add: bit-exact


@pytest.mark.parametrize("M,N,K,hd,rc", [(512, 768, 128, 64, 512), (520, 776, 200, 16, 768), (256, 256, 64, 128, 256)])
@pytest.mark.parametrize("with_r,f32", [(True, False), (False, False), (True, True)])
def test_kernel7_rope(oracle, M, N, K, hd, rc, with_r, f32):
    """Kernels 1 / 7: row scale, RoPE on adjacent pairs of the first rc columns, store."""
    g = rng(61)
    A, B = operands(g, M, N, K, False, False, b_std=0.2)
    T = 96
    cos, sin = synth.rope_tables(T, hd)
    pos = g.integers(0, T, size=M).astype(np.int32)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5) if with_r else None
    out = G.Guarded(M, N, torch.float32 if f32 else torch.bfloat16)
    dcos, dsin, dpos = G.dev_f32(cos), G.dev_f32(sin), torch.from_numpy(pos).cuda()
    ops = ([coda.row_scale(dr := G.dev_f32(r))] if with_r else []) + \
          [coda.rope(dcos, dsin, dpos, hd, rc), coda.store(out.t, f32=f32)]
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), ops)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale_rope(A, B, cos, sin, pos, hd, rc, r=None if r is None else r.astype(np.float64))
    out.check_guards(); out.written()
    if f32:
        G.assert_f32_signed_close(G.host_f64(out.t), ref, "rope f32")
    else:
        G.assert_bf16_close(G.host_f64(out.t), ref, "rope")


@pytest.mark.parametrize("M,N,K,hd", [(512, 768, 128, 64), (264, 256, 72, 16)])
@pytest.mark.parametrize("f32", [False, True])
def test_rope_positions_outside_the_table_are_clamped(oracle, M, N, K, hd, f32):
    """A position below 0 or at / beyond the table length T reads the nearest table row (never outside the table):
    the result equals the oracle's on the clamped positions.  The tables sit between sentinel rows that would poison
    the output if a row outside [0, T) were read.  Both RoPE paths (LDS-staged tables, per-unit gathers) are covered."""
    g = rng(67)
    A, B = operands(g, M, N, K, False, False, b_std=0.2)
    T = 40
    cos, sin = synth.rope_tables(T, hd)
    pos = g.integers(0, T, size=M).astype(np.int32)
    pos[::7] = -1 - g.integers(0, 1000, size=pos[::7].size).astype(np.int32)
    pos[3::7] = T + g.integers(0, 1 << 20, size=pos[3::7].size).astype(np.int32)
    pos[5] = np.iinfo(np.int32).min
    pos[6] = np.iinfo(np.int32).max
    pad = np.full((64, hd // 2), 1e30, np.float32)
    dcos = G.dev_f32(np.concatenate([pad, cos, pad]))[64:64 + T]
    dsin = G.dev_f32(np.concatenate([pad, sin, pad]))[64:64 + T]
    out = G.Guarded(M, N, torch.float32 if f32 else torch.bfloat16)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.rope(dcos, dsin, torch.from_numpy(pos).cuda(), hd, N), coda.store(out.t, f32=f32)])
    torch.cuda.synchronize()
    out.check_guards(); out.written()
    ref = oracle.gemm_rowscale_rope(A, B, cos, sin, np.clip(pos, 0, T - 1).astype(np.int32), hd, N)
    if f32:
        G.assert_f32_signed_close(G.host_f64(out.t), ref, "rope clamp f32")
    else:
        G.assert_bf16_close(G.host_f64(out.t), ref, "rope clamp")


@pytest.mark.parametrize("M,N,K", [(512, 512, 128), (520, 264, 200)])
@pytest.mark.parametrize("with_oin,atomic,transB", [(True, False, True), (False, True, True), (True, False, False)])
def test_kernel9_rmsnorm_backward(oracle, M, N, K, with_oin, atomic, transB):
    """Kernel 9: D = A op(B); O_out = O_in + (D*gamma - C*r*z)*r; C_out = C*r*gamma; dgamma = colsum(D*C*r)."""
    g = rng(71)
    A, B = operands(g, M, N, K, False, transB, a_std=1.0, b_std=0.1)
    Cb = synth.normal_bf16(g, (M, N), 1.0)
    Oin = synth.normal_bf16(g, (M, N), 1.0) if with_oin else None
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    z = synth.normal_f32(g, (M,), 0.3)
    gamma = synth.uniform_f32(g, (N,), 0.5, 1.5)
    Oout = G.Guarded(M, N, torch.bfloat16)
    Cout = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_col_partial_blocks(M)
    dgp = torch.zeros(N, dtype=torch.float32, device="cuda") if atomic else \
        torch.full((nblk, N), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dC, dr, dz, dgm = G.dev_bf16(Cb), G.dev_f32(r), G.dev_f32(z), G.dev_f32(gamma)
    ops = [coda.rmsnorm_bwd(dC, dr, dz, dgm, c_out=Cout.t, dgamma_out=dgp, atomic=atomic)]
    if with_oin:
        dO = G.dev_bf16(Oin)
        ops.append(coda.add_tile(dO))
    ops.append(coda.store(Oout.t))
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), ops, transB=transB)
    if atomic:
        dg = dgp
    else:
        dg = torch.empty(N, dtype=torch.float32, device="cuda")
        coda.coda_col_finalize(dgp, N, nblk, dg)
    torch.cuda.synchronize()
    refO, refC, refdg = oracle.gemm_rmsnorm_bwd(A, B, Cb, r.astype(np.float64), z.astype(np.float64),
                                                gamma.astype(np.float64), Oin=Oin, transB=transB)
    Oout.check_guards(); Oout.written(); Cout.check_guards(); Cout.written()
    G.assert_bf16_close(G.host_f64(Oout.t), refO, "O_out")
    G.assert_bf16_close(G.host_f64(Cout.t), refC, "C_out")
    G.assert_f32_signed_close(G.host_f64(dg), refdg, "dgamma")


@pytest.mark.parametrize("M,N,K", [(512, 1024, 128), (520, 776, 200)])
@pytest.mark.parametrize("with_r,transB", [(True, False), (False, True)])
def test_kernel8_logits_lse_partials(oracle, M, N, K, with_r, transB):
    """Kernels 3 / 8: logits (materialised), target logit and per-tile (max, sum-exp) partials -> lse and loss."""
    g = rng(81)
    A, B = operands(g, M, N, K, False, transB, b_std=0.3)
    y = g.integers(0, N, size=M).astype(np.int32)
    y[:4] = [0, N - 1, 255 if N > 255 else 1, 256 if N > 256 else 2]        # tile-boundary targets
    r = synth.uniform_f32(g, (M,), 0.5, 1.5) if with_r else None
    Z = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    pmax = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    psum = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    zt = torch.full((M,), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dy = torch.from_numpy(y).cuda()
    ops = ([coda.row_scale(dr := G.dev_f32(r))] if with_r else []) + [coda.lse_partial(dy, pmax, psum, zt), coda.store(Z.t)]
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), ops, transB=transB)
    lse = torch.empty(M, dtype=torch.float32, device="cuda")
    loss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_lse_finalize(pmax, psum, M, nblk, ztgt=zt, lse_out=lse, loss_out=loss)
    torch.cuda.synchronize()
    refZ, refzt, reflse = oracle.gemm_rowscale_lse(A, B, y, r=None if r is None else r.astype(np.float64), transB=transB)
    Z.check_guards(); Z.written()
    G.assert_bf16_close(G.host_f64(Z.t), refZ, "logits")
    assert (pmax != G.SENTINEL_F32).all() and (psum != G.SENTINEL_F32).all() and (zt != G.SENTINEL_F32).all()
    G.assert_f32_signed_close(G.host_f64(zt), refzt, "target logit")
    d = np.abs(G.host_f64(lse) - reflse)
    assert (d <= 1e-3 * np.maximum(np.abs(reflse), 1.0)).all(), "lse max delta %.3g" % d.max()
    G.assert_f32_signed_close(G.host_f64(loss), reflse - refzt, "per-token loss")


# Gate pre-activations from deep saturation on both sides (where exp(-g) overflows or underflows fp32) through the
# linear region around zero: the kernels' sigmoid must go to exactly 0 / 1 there without producing NaN or Inf.
EXTREME_GATES = np.array([-1e4, -120.0, -100.0, -89.0, -88.0, -87.0, -60.0, -30.0, -17.0, -10.0, -1.0, -1e-3, -1e-30, 0.0,
                          1e-30, 1e-3, 1.0, 10.0, 17.0, 30.0, 60.0, 87.0, 88.0, 89.0, 100.0, 120.0, 1e4], np.float32)


def _extreme_pairs(g, rows, pairs):
    """[rows x 2*pairs] bf16 bits: even columns (gates) cycle through EXTREME_GATES, shifted per row; odd columns
    (up-projection values) are standard normal."""
    Z = G.bits_to_f64(synth.normal_bf16(g, (rows, 2 * pairs), 1.0)).astype(np.float32)
    idx = (np.arange(rows)[:, None] * 5 + np.arange(pairs)[None, :]) % EXTREME_GATES.size
    Z[:, 0::2] = EXTREME_GATES[idx]
    return synth.f32_to_bf16_bits(Z)


def test_logits_lse_with_row_scales_of_either_sign(oracle):
    """The log-sum-exp partials take the row maximum from the raw accumulators in the direction of the row scale's sign:
    negative, zero and positive row scales, and targets on the last valid column of a ragged tile."""
    g = rng(97)
    M, N, K = 300, 520, 136
    A, B = operands(g, M, N, K, False, False, b_std=0.3)
    r = synth.uniform_f32(g, (M,), -2.0, 2.0)
    r[::5] = 0.0
    r[1::5] = -np.abs(r[1::5])
    y = g.integers(0, N, size=M).astype(np.int32)
    y[:8] = N - 1
    y[8:16] = [0, 3, 4, 15, 16, 63, 64, 255]
    Z = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    pmax = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    psum = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    zt = torch.full((M,), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    lse = torch.empty(M, dtype=torch.float32, device="cuda")
    dy, dr = torch.from_numpy(y).cuda(), G.dev_f32(r)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.row_scale(dr), coda.lse_partial(dy, pmax, psum, zt), coda.store(Z.t)])
    coda.coda_lse_finalize(pmax, psum, M, nblk, lse_out=lse)
    torch.cuda.synchronize()
    Z.check_guards(); Z.written()
    assert int((pmax == G.SENTINEL_F32).sum().item()) == 0 and int((zt == G.SENTINEL_F32).sum().item()) == 0
    refZ, refzt, reflse = oracle.gemm_rowscale_lse(A, B, y, r=r.astype(np.float64))
    G.assert_bf16_close(G.host_f64(Z.t), refZ, "logits, signed row scales")
    G.assert_f32_signed_close(G.host_f64(zt), refzt, "target logit, signed row scales")
    d = np.abs(G.host_f64(lse) - reflse)
    assert (d <= 1e-3 * np.maximum(np.abs(reflse), 1.0)).all(), "lse max delta %.3g" % d.max()


def test_swiglu_forward_saturated_gates(oracle):
    M, N, K = 256, 512, 64
    g = rng(31)
    A = np.zeros((M, K), np.float32)
    A[np.arange(M), np.arange(M) % K] = 1.0             # one-hot rows: row i of A*B is row i % K of B, exactly
    A = synth.f32_to_bf16_bits(A)
    B = _extreme_pairs(g, K, N // 2)
    H = G.Guarded(M, N // 2, torch.bfloat16)
    Z = G.Guarded(M, N, torch.bfloat16)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.swiglu_fwd(Z.t), coda.store(H.t)])
    torch.cuda.synchronize()
    refH, refZ = oracle.gemm_rowscale_swiglu(A, B, want_preact=True)
    H.check_guards(); H.written(); Z.check_guards(); Z.written()
    got = G.host_f64(H.t)
    assert np.isfinite(got).all()
    assert (G.host_bits(Z.t) == B[np.arange(M) % K]).all(), "pre-activation must be the selected rows of B, bit for bit"
    G.assert_bf16_close(got, refH, "swiglu fwd, saturated gates")
    gates = G.bits_to_f64(B[np.arange(M) % K])[:, 0::2]
    assert (got[gates <= -100.0] == 0.0).all(), "deeply negative gates must give exactly zero"


@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (264, 200, 72)])
def test_swiglu_backward_saturated_gates(oracle, M, N, K):
    g = rng(32)
    A = synth.normal_bf16(g, (M, K), 0.125)
    Bt = synth.normal_bf16(g, (N, K), 1.0)
    Z = _extreme_pairs(g, M, N)
    dZ = G.Guarded(M, 2 * N, torch.bfloat16)
    O = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    ops = [coda.swiglu_bwd(G.dev_bf16(Z), act_out=O.t, stat_out=part), coda.store(dZ.t)]
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(Bt), ops, transB=True)
    stat = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=stat, d=1, eps=0.0)
    torch.cuda.synchronize()
    refdZ, refO, refstat = oracle.gemm_swiglu_bwd(A, Bt, Z, transB=True)
    dZ.check_guards(); dZ.written(); O.check_guards(); O.written()
    got, gotO = G.host_f64(dZ.t), G.host_f64(O.t)
    assert np.isfinite(got).all() and np.isfinite(gotO).all() and np.isfinite(G.host_f64(stat)).all()
    # elementwise against |ref| alone: the 1e4 gates would otherwise inflate an rms-based allowance
    d = np.abs(got - refdZ)
    assert (d <= 1e-2 + 1e-2 * np.abs(refdZ)).all(), "dZ: max delta %.3g" % d.max()
    d = np.abs(gotO - refO)
    assert (d <= 1e-2 + 1e-2 * np.abs(refO)).all(), "activation: max delta %.3g" % d.max()
    G.assert_f32_signed_close(G.host_f64(stat), refstat, "row statistic")


def test_repeat_launches_are_bitwise_identical_and_leave_inputs_alone():
    """With two-pass partials nothing depends on the order in which workgroups run: the same launch twice gives the same
    bits in every output (tile outputs, row partials, column partials), and no input buffer changes.  Atomic row sums may
    differ in the last bits between runs; their spread is bounded here."""
    M, N, K = 1024, 1280, 520
    g = rng(77)
    A, Bt = synth.normal_bf16(g, (M, K), 1.0), synth.normal_bf16(g, (N, K), 0.05)
    C, Z = synth.normal_bf16(g, (M, N), 1.0), synth.normal_bf16(g, (M, 2 * N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    dA, dB, dC, dZ, dr = G.dev_bf16(A), G.dev_bf16(Bt), G.dev_bf16(C), G.dev_bf16(Z), G.dev_f32(r)
    inputs = [dA, dB, dC, dZ, dr]
    before = [t.clone() for t in inputs]
    nblk = coda.coda_row_partial_blocks(N)

    def run_all():
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        part = torch.empty((nblk, M), dtype=torch.float32, device="cuda")
        coda.coda_gemm(dA, dB, [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y)], transB=True)
        H = torch.empty((M, N // 2), dtype=torch.bfloat16, device="cuda")
        coda.coda_gemm(dA, dB, [coda.row_scale(dr), coda.swiglu_fwd(), coda.store(H)], transB=True)
        dZo = torch.empty((M, 2 * N), dtype=torch.bfloat16, device="cuda")
        stat = torch.empty((nblk, M), dtype=torch.float32, device="cuda")
        coda.coda_gemm(dA, dB, [coda.swiglu_bwd(dZ, stat_out=stat), coda.store(dZo)], transB=True)
        ss_atomic = torch.zeros(M, dtype=torch.float32, device="cuda")
        Y2 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        coda.coda_gemm(dA, dB, [coda.add_tile(dC), coda.row_sumsq(ss_atomic, atomic=True), coda.store(Y2)], transB=True)
        torch.cuda.synchronize()
        return [Y, part, H, dZo, stat, Y2], ss_atomic

    first, at1 = run_all()
    second, at2 = run_all()
    for a, b in zip(first, second):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    for t, t0 in zip(inputs, before):
        assert torch.equal(t.view(torch.uint8), t0.view(torch.uint8)), "an input buffer was modified"
    rel = ((at1 - at2).abs() / at1.abs().clamp_min(1e-30)).max().item()
    assert rel <= 1e-5, "atomic row sums differ by %.3g between runs" % rel


def test_both_operands_k_contiguous_long_k_whole_tiles(oracle):
    """Whole tiles, A [M x K] and B [N x K], K long enough that every XCD starts its K loop at a different offset
    (12 tiles cover all eight start offsets): linear program and SwiGLU backward, element by element."""
    M, N, K = 1024, 768, 1024
    g = rng(88)
    A, Bt = synth.normal_bf16(g, (M, K), 1.0), synth.normal_bf16(g, (N, K), 0.05)
    C = synth.normal_bf16(g, (M, N), 1.0)
    Y = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dA, dB, dC = G.dev_bf16(A), G.dev_bf16(Bt), G.dev_bf16(C)
    coda.coda_gemm(dA, dB, [coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y.t)], transB=True)
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
    torch.cuda.synchronize()
    refD, refss = oracle.gemm_residual_sumsq(A, Bt, C=C, transB=True)[:2]
    Y.check_guards(); Y.written()
    G.assert_bf16_close(G.host_f64(Y.t), refD, "residual output")
    G.assert_sumsq_close(G.host_f64(ss), refss, "row sum of squares")
    # the K order of a tile depends on its position only: a second launch gives the same bits
    Y2 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    part2 = torch.empty_like(part)
    coda.coda_gemm(dA, dB, [coda.add_tile(dC), coda.row_sumsq(part2), coda.store(Y2)], transB=True)
    torch.cuda.synchronize()
    assert torch.equal(Y2.view(torch.int16), Y.t.contiguous().view(torch.int16)) and torch.equal(part2.view(torch.int32), part.view(torch.int32))
    A2 = synth.normal_bf16(g, (M, K), 1e-2)
    Z = synth.normal_bf16(g, (M, 2 * N), 1.0)
    dZ = G.Guarded(M, 2 * N, torch.bfloat16)
    dZin, dA2 = G.dev_bf16(Z), G.dev_bf16(A2)
    coda.coda_gemm(dA2, dB, [coda.swiglu_bwd(dZin), coda.store(dZ.t)], transB=True)
    torch.cuda.synchronize()
    refdZ = oracle.gemm_swiglu_bwd(A2, Bt, Z, transB=True)[0]
    dZ.check_guards(); dZ.written()
    G.assert_bf16_close(G.host_f64(dZ.t), refdZ, "dZ")


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("pad", [8, 40])
def test_whole_tiles_with_padded_operand_pitches(oracle, transA, transB, pad):
    """Whole-tile kernels on operands whose rows do not start on 128-byte boundaries (pitch = width + pad elements)."""
    M, N, K = 512, 512, 256
    g = rng(300 + pad)
    a_shape, b_shape = ((K, M) if transA else (M, K)), ((N, K) if transB else (K, N))
    Ap = synth.normal_bf16(g, (a_shape[0], a_shape[1] + pad), 1.0)
    Bp = synth.normal_bf16(g, (b_shape[0], b_shape[1] + pad), 0.3)
    dA, dB = G.dev_bf16(Ap)[:, :a_shape[1]], G.dev_bf16(Bp)[:, :b_shape[1]]
    out = G.Guarded(M, N, torch.bfloat16)
    coda.coda_gemm(dA, dB, [coda.store(out.t)], transA=transA, transB=transB)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale(np.ascontiguousarray(Ap[:, :a_shape[1]]), np.ascontiguousarray(Bp[:, :b_shape[1]]),
                               transA=transA, transB=transB)
    out.check_guards(); out.written()
    G.assert_bf16_close(G.host_f64(out.t), ref, "padded pitches")


@pytest.mark.parametrize("K", [64, 128, 192, 256, 320, 384, 448, 512, 640])
@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_whole_tiles_every_short_k(oracle, K, transA, transB):
    """One whole tile per workgroup, K-step counts 2 .. 20: prologue only, ring never full, first steady trips, run-dry
    steps (and with a K-contiguous A: pairs of K-steps in a ring of three pair slots)."""
    M, N = 256, 512
    g = rng(400 + K)
    A, B = operands(g, M, N, K, transA, transB)
    out = G.Guarded(M, N, torch.bfloat16)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.store(out.t)], transA=transA, transB=transB)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale(A, B, transA=transA, transB=transB)
    out.check_guards(); out.written()
    G.assert_bf16_close(G.host_f64(out.t), ref, "K = %d" % K)
