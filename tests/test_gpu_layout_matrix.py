"""GPU parity, layout x epilogue matrix: every epilogue mode of coda_gemm is instantiated once per operand
layout (A or A^T, B or B^T).  Each (layout, mode) pair is run on a shape of whole 256 x 256 x 64 tiles, on a shape
ragged in every dimension (clamped fetches, zero-filled K tail, bounds-checked epilogue) and on a shape ragged
in M and N only, against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2605_19269_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

LAYOUTS = [(False, False), (False, True), (True, False), (True, True)]
SHAPES = [(256, 512, 128), (264, 520, 72), (264, 520, 128)]   # whole tiles | ragged in every dimension | ragged in M and N only

coda = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global coda
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_19269_amd import coda as _c
    coda = _c
    yield
    torch.cuda.synchronize()


def operands(g, M, N, K, transA, transB, a_std=1.0, b_std=0.2):
    A = synth.normal_bf16(g, (K, M) if transA else (M, K), a_std)
    B = synth.normal_bf16(g, (N, K) if transB else (K, N), b_std)
    return A, B


def seed(M, transA, transB, salt):
    return 1000 * salt + 10 * M + 2 * int(transA) + int(transB)


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_linear_program_all_layouts(oracle, M, N, K, transA, transB):
    g = np.random.Generator(np.random.PCG64(seed(M, transA, transB, 1)))
    A, B = operands(g, M, N, K, transA, transB)
    C = synth.normal_bf16(g, (M, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    Y = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dr, dC = G.dev_f32(r), G.dev_bf16(C)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y.t)],
                   transA=transA, transB=transB)
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
    torch.cuda.synchronize()
    refD, refss = oracle.gemm_residual_sumsq(A, B, r=r.astype(np.float64), C=C, transA=transA, transB=transB)[:2]
    Y.check_guards(); Y.written()
    G.assert_bf16_close(G.host_f64(Y.t), refD, "row scale + residual")
    G.assert_sumsq_close(G.host_f64(ss), refss, "row sum of squares")


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_swiglu_forward_all_layouts(oracle, M, N, K, transA, transB):
    g = np.random.Generator(np.random.PCG64(seed(M, transA, transB, 2)))
    A, B = operands(g, M, N, K, transA, transB)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    H = G.Guarded(M, N // 2, torch.bfloat16)
    Z = G.Guarded(M, N, torch.bfloat16)
    dr = G.dev_f32(r)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.row_scale(dr), coda.swiglu_fwd(Z.t), coda.store(H.t)],
                   transA=transA, transB=transB)
    torch.cuda.synchronize()
    refH, refZ = oracle.gemm_rowscale_swiglu(A, B, r=r.astype(np.float64), transA=transA, transB=transB, want_preact=True)
    H.check_guards(); H.written(); Z.check_guards(); Z.written()
    G.assert_bf16_close(G.host_f64(H.t), refH, "swiglu forward")
    G.assert_bf16_close(G.host_f64(Z.t), refZ, "pre-activation")


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_swiglu_backward_all_layouts(oracle, M, N, K, transA, transB):
    g = np.random.Generator(np.random.PCG64(seed(M, transA, transB, 3)))
    A, B = operands(g, M, N, K, transA, transB, a_std=1e-2, b_std=0.05)
    Z = synth.normal_bf16(g, (M, 2 * N), 1.0)
    dZ = G.Guarded(M, 2 * N, torch.bfloat16)
    O = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dZin = G.dev_bf16(Z)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.swiglu_bwd(dZin, act_out=O.t, stat_out=part), coda.store(dZ.t)],
                   transA=transA, transB=transB)
    stat = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=stat, d=1, eps=0.0)
    torch.cuda.synchronize()
    refdZ, refO, refstat = oracle.gemm_swiglu_bwd(A, B, Z, transA=transA, transB=transB)
    dZ.check_guards(); dZ.written(); O.check_guards(); O.written()
    G.assert_bf16_close(G.host_f64(dZ.t), refdZ, "dZ")
    G.assert_bf16_close(G.host_f64(O.t), refO, "recomputed activation")
    G.assert_f32_signed_close(G.host_f64(stat), refstat, "row statistic")


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_accumulate_all_layouts(oracle, M, N, K, transA, transB):
    g = np.random.Generator(np.random.PCG64(seed(M, transA, transB, 4)))
    A, B = operands(g, M, N, K, transA, transB, b_std=1e-2)
    Gin = synth.normal_f32(g, (M, N), 1e-3)
    buf = G.Guarded(M, N, torch.float32, pad_cols=4)
    buf.t.copy_(torch.from_numpy(Gin))
    buf.ref = buf.full.clone()
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.accum_f32(buf.t)], transA=transA, transB=transB)
    torch.cuda.synchronize()
    ref = oracle.gemm_accumulate(A, B, Gin, transA=transA, transB=transB)
    buf.check_guards()
    G.assert_f32_signed_close(G.host_f64(buf.t), ref, "fp32 accumulate")


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_rmsnorm_backward_all_layouts(oracle, M, N, K, transA, transB):
    g = np.random.Generator(np.random.PCG64(seed(M, transA, transB, 5)))
    A, B = operands(g, M, N, K, transA, transB, b_std=0.1)
    Cb = synth.normal_bf16(g, (M, N), 1.0)
    Oin = synth.normal_bf16(g, (M, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    z = synth.normal_f32(g, (M,), 0.3)
    gamma = synth.uniform_f32(g, (N,), 0.5, 1.5)
    Oout, Cout = G.Guarded(M, N, torch.bfloat16), G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_col_partial_blocks(M)
    dgp = torch.full((nblk, N), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dC, dr, dz, dgm, dO = G.dev_bf16(Cb), G.dev_f32(r), G.dev_f32(z), G.dev_f32(gamma), G.dev_bf16(Oin)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B),
                   [coda.rmsnorm_bwd(dC, dr, dz, dgm, c_out=Cout.t, dgamma_out=dgp), coda.add_tile(dO), coda.store(Oout.t)],
                   transA=transA, transB=transB)
    dg = torch.empty(N, dtype=torch.float32, device="cuda")
    coda.coda_col_finalize(dgp, N, nblk, dg)
    torch.cuda.synchronize()
    refO, refC, refdg = oracle.gemm_rmsnorm_bwd(A, B, Cb, r.astype(np.float64), z.astype(np.float64), gamma.astype(np.float64),
                                                Oin=Oin, transA=transA, transB=transB)
    Oout.check_guards(); Oout.written(); Cout.check_guards(); Cout.written()
    G.assert_bf16_close(G.host_f64(Oout.t), refO, "O_out")
    G.assert_bf16_close(G.host_f64(Cout.t), refC, "C_out")
    G.assert_f32_signed_close(G.host_f64(dg), refdg, "dgamma")


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_rope_and_lse_all_layouts(oracle, M, N, K, transA, transB):
    g = np.random.Generator(np.random.PCG64(seed(M, transA, transB, 6)))
    A, B = operands(g, M, N, K, transA, transB)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    dr = G.dev_f32(r)
    # RoPE on the first 256 columns, head dimension 64
    hd, rc, T = 64, 256, 80
    cos, sin = synth.rope_tables(T, hd)
    pos = g.integers(0, T, size=M).astype(np.int32)
    out = G.Guarded(M, N, torch.bfloat16)
    dcos, dsin, dpos = G.dev_f32(cos), G.dev_f32(sin), torch.from_numpy(pos).cuda()
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.row_scale(dr), coda.rope(dcos, dsin, dpos, hd, rc), coda.store(out.t)],
                   transA=transA, transB=transB)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale_rope(A, B, cos, sin, pos, hd, rc, r=r.astype(np.float64), transA=transA, transB=transB)
    out.check_guards(); out.written()
    G.assert_bf16_close(G.host_f64(out.t), ref, "rope")
    # log-sum-exp partials with the target logit
    y = g.integers(0, N, size=M).astype(np.int32)
    Z = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    pmax = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    psum = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    zt = torch.full((M,), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dy = torch.from_numpy(y).cuda()
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.row_scale(dr), coda.lse_partial(dy, pmax, psum, zt), coda.store(Z.t)],
                   transA=transA, transB=transB)
    lse = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_lse_finalize(pmax, psum, M, nblk, ztgt=zt, lse_out=lse)
    torch.cuda.synchronize()
    refZ, refzt, reflse = oracle.gemm_rowscale_lse(A, B, y, r=r.astype(np.float64), transA=transA, transB=transB)
    Z.check_guards(); Z.written()
    G.assert_bf16_close(G.host_f64(Z.t), refZ, "logits")
    G.assert_f32_signed_close(G.host_f64(zt), refzt, "target logit")
    d = np.abs(G.host_f64(lse) - reflse)
    assert (d <= 1e-3 * np.maximum(np.abs(reflse), 1.0)).all(), "lse max delta %.3g" % d.max()
