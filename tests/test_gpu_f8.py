"""GPU parity of the 8-bit-operand variant (OCP E4M3 operands in all four storage layouts, fp32 accumulation, the same
epilogue programs) against the CPU oracle, which decodes the very same bytes by the format's definition and then applies
its ordinary GEMM definitions.  Covers the decoding of every finite code, every epilogue mode, ragged shapes, split-K,
and the layouts with an operand whose output index is contiguous (read through the 8-bit transposing LDS read)."""
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


def dev_u8(bits):
    return torch.from_numpy(np.ascontiguousarray(bits)).cuda()


def operands(oracle, g, M, N, K, a_std=1.0, b_std=1.0):
    """E4M3 bytes for the GPU and the bf16 bit patterns of the same values for the oracle."""
    A8, B8 = synth.normal_f8e4m3(g, (M, K), a_std), synth.normal_f8e4m3(g, (N, K), b_std)
    return A8, B8, oracle.f8e4m3_to_bf16_bits(A8), oracle.f8e4m3_to_bf16_bits(B8)


# whole tiles | ragged in M, N and K (K past a whole pair of 64-element K-steps by 16 and by 80 elements)
SHAPES = [(256, 256, 128), (512, 768, 384), (256, 512, 2048), (264, 520, 208), (200, 264, 144)]


def test_every_finite_code_is_decoded_as_e4m3(oracle):
    """B selects single elements of A (one 1.0 per row), so D holds A's decoded values themselves: exact in fp32."""
    M, N, K = 256, 256, 128
    codes = (np.arange(M * K, dtype=np.int64) % 256).astype(np.uint8).reshape(M, K)
    codes[(codes & 0x7F) == 0x7F] = 0                        # the two NaN codes are outside the contract
    B8 = np.zeros((N, K), np.uint8)
    B8[np.arange(N), np.arange(N) % K] = 0x38                # 1.0
    out = G.Guarded(M, N, torch.float32, pad_cols=4)
    coda.coda_gemm(dev_u8(codes), dev_u8(B8), [coda.store(out.t, f32=True)], transB=True)
    torch.cuda.synchronize()
    out.check_guards(); out.written()
    ref = oracle.gemm_rowscale(oracle.f8e4m3_to_bf16_bits(codes), oracle.f8e4m3_to_bf16_bits(B8), transB=True)
    got = G.host_f64(out.t)
    assert np.array_equal(got, ref), "max |delta| %.3g" % np.abs(got - ref).max()
    assert set(np.unique(codes)) >= set(c for c in range(256) if (c & 0x7F) != 0x7F)


# without a workspace | with one, on shapes the 8-bit plan splits 4-way and 2-way
@pytest.mark.parametrize("M,N,K,split", [(m, n, k, False) for m, n, k in SHAPES] + [(256, 256, 8192, True), (512, 512, 4096, True), (504, 264, 4304, True)] + [(8, 8, 16, False), (1, 256, 64, False)]
                         + [(256, 256, k, False) for k in (256, 512, 640, 768)])   # K-step counts 4, 8, 10, 12: ring fill and run-dry
def test_f8_linear_program(oracle, M, N, K, split):
    g = np.random.Generator(np.random.PCG64(1100 + M + K))
    A8, B8, A16, B16 = operands(oracle, g, M, N, K)
    C = synth.normal_bf16(g, (M, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.02, 0.06)               # carries the operands' dequantisation scales
    ws = None
    if split:
        need = coda.coda_gemm_workspace_bytes(M, N, K, [])
        assert need > 0
        ws = torch.empty(need, dtype=torch.uint8, device="cuda").fill_(0x5A)
    Y = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dr, dC = G.dev_f32(r), G.dev_bf16(C)
    coda.coda_gemm(dev_u8(A8), dev_u8(B8), [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y.t)],
                   transB=True, workspace=ws)
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
    torch.cuda.synchronize()
    refD, refss = oracle.gemm_residual_sumsq(A16, B16, r=r.astype(np.float64), C=C, transB=True)[:2]
    Y.check_guards(); Y.written()
    G.assert_bf16_close(G.host_f64(Y.t), refD, "f8 row scale + residual")
    G.assert_sumsq_close(G.host_f64(ss), refss, "f8 row sum of squares")


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_f8_swiglu_forward_and_backward(oracle, M, N, K):
    g = np.random.Generator(np.random.PCG64(1200 + M + K))
    A8, B8, A16, B16 = operands(oracle, g, M, N, K)
    r = synth.uniform_f32(g, (M,), 0.02, 0.06)
    H, Zs = G.Guarded(M, N // 2, torch.bfloat16), G.Guarded(M, N, torch.bfloat16)
    dr = G.dev_f32(r)
    coda.coda_gemm(dev_u8(A8), dev_u8(B8), [coda.row_scale(dr), coda.swiglu_fwd(Zs.t), coda.store(H.t)], transB=True)
    torch.cuda.synchronize()
    refH, refZ = oracle.gemm_rowscale_swiglu(A16, B16, r=r.astype(np.float64), transB=True, want_preact=True)
    H.check_guards(); H.written(); Zs.check_guards(); Zs.written()
    G.assert_bf16_close(G.host_f64(H.t), refH, "f8 swiglu forward")
    G.assert_bf16_close(G.host_f64(Zs.t), refZ, "f8 pre-activation")
    # backward on the same operands: D plays the incoming gradient (small values via small A)
    A8b = synth.normal_f8e4m3(g, (M, K), 0.05)
    A16b = oracle.f8e4m3_to_bf16_bits(A8b)
    Z = synth.normal_bf16(g, (M, 2 * N), 1.0)
    dZ, O = G.Guarded(M, 2 * N, torch.bfloat16), G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dZin = G.dev_bf16(Z)
    coda.coda_gemm(dev_u8(A8b), dev_u8(B8), [coda.swiglu_bwd(dZin, act_out=O.t, stat_out=part), coda.store(dZ.t)], transB=True)
    stat = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=stat, d=1, eps=0.0)
    torch.cuda.synchronize()
    refdZ, refO, refstat = oracle.gemm_swiglu_bwd(A16b, B16, Z, transB=True)
    dZ.check_guards(); dZ.written(); O.check_guards(); O.written()
    G.assert_bf16_close(G.host_f64(dZ.t), refdZ, "f8 dZ")
    G.assert_bf16_close(G.host_f64(O.t), refO, "f8 recomputed activation")
    G.assert_f32_signed_close(G.host_f64(stat), refstat, "f8 row statistic")


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_f8_accumulate_rmsnorm_backward_rope_lse(oracle, M, N, K):
    g = np.random.Generator(np.random.PCG64(1300 + M + K))
    A8, B8, A16, B16 = operands(oracle, g, M, N, K, a_std=0.25, b_std=0.25)
    dA, dB = dev_u8(A8), dev_u8(B8)
    # fp32 accumulate
    Gin = synth.normal_f32(g, (M, N), 1e-1)
    buf = G.Guarded(M, N, torch.float32, pad_cols=4)
    buf.t.copy_(torch.from_numpy(Gin))
    buf.ref = buf.full.clone()
    coda.coda_gemm(dA, dB, [coda.accum_f32(buf.t)], transB=True)
    torch.cuda.synchronize()
    buf.check_guards()
    G.assert_f32_signed_close(G.host_f64(buf.t), oracle.gemm_accumulate(A16, B16, Gin, transB=True), "f8 fp32 accumulate")
    # RMSNorm backward
    Cb, Oin = synth.normal_bf16(g, (M, N), 1.0), synth.normal_bf16(g, (M, N), 1.0)
    r, z = synth.uniform_f32(g, (M,), 0.5, 1.5), synth.normal_f32(g, (M,), 0.3)
    gamma = synth.uniform_f32(g, (N,), 0.5, 1.5)
    Oout, Cout = G.Guarded(M, N, torch.bfloat16), G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_col_partial_blocks(M)
    dgp = torch.full((nblk, N), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dC, dr, dz, dgm, dO = G.dev_bf16(Cb), G.dev_f32(r), G.dev_f32(z), G.dev_f32(gamma), G.dev_bf16(Oin)
    coda.coda_gemm(dA, dB, [coda.rmsnorm_bwd(dC, dr, dz, dgm, c_out=Cout.t, dgamma_out=dgp), coda.add_tile(dO), coda.store(Oout.t)],
                   transB=True)
    dg = torch.empty(N, dtype=torch.float32, device="cuda")
    coda.coda_col_finalize(dgp, N, nblk, dg)
    torch.cuda.synchronize()
    refO, refC, refdg = oracle.gemm_rmsnorm_bwd(A16, B16, Cb, r.astype(np.float64), z.astype(np.float64), gamma.astype(np.float64),
                                                Oin=Oin, transB=True)
    Oout.check_guards(); Oout.written(); Cout.check_guards(); Cout.written()
    G.assert_bf16_close(G.host_f64(Oout.t), refO, "f8 O_out")
    G.assert_bf16_close(G.host_f64(Cout.t), refC, "f8 C_out")
    G.assert_f32_signed_close(G.host_f64(dg), refdg, "f8 dgamma")
    # RoPE
    hd, rc, T = 64, 256, 80
    cos, sin = synth.rope_tables(T, hd)
    pos = g.integers(0, T, size=M).astype(np.int32)
    out = G.Guarded(M, N, torch.bfloat16)
    dcos, dsin, dpos = G.dev_f32(cos), G.dev_f32(sin), torch.from_numpy(pos).cuda()
    coda.coda_gemm(dA, dB, [coda.row_scale(dr), coda.rope(dcos, dsin, dpos, hd, rc), coda.store(out.t)], transB=True)
    torch.cuda.synchronize()
    out.check_guards(); out.written()
    G.assert_bf16_close(G.host_f64(out.t), oracle.gemm_rowscale_rope(A16, B16, cos, sin, pos, hd, rc, r=r.astype(np.float64), transB=True),
                        "f8 rope")
    # log-sum-exp partials
    y = g.integers(0, N, size=M).astype(np.int32)
    Zl = G.Guarded(M, N, torch.bfloat16)
    nb = coda.coda_row_partial_blocks(N)
    pmax = torch.full((nb, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    psum = torch.full((nb, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    zt = torch.full((M,), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dy = torch.from_numpy(y).cuda()
    rl = synth.uniform_f32(g, (M,), 0.05, 0.15)
    drl = G.dev_f32(rl)
    coda.coda_gemm(dA, dB, [coda.row_scale(drl), coda.lse_partial(dy, pmax, psum, zt), coda.store(Zl.t)], transB=True)
    lse = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_lse_finalize(pmax, psum, M, nb, ztgt=zt, lse_out=lse)
    torch.cuda.synchronize()
    refZ, refzt, reflse = oracle.gemm_rowscale_lse(A16, B16, y, r=rl.astype(np.float64), transB=True)
    Zl.check_guards(); Zl.written()
    G.assert_bf16_close(G.host_f64(Zl.t), refZ, "f8 logits")
    G.assert_f32_signed_close(G.host_f64(zt), refzt, "f8 target logit")
    d = np.abs(G.host_f64(lse) - reflse)
    assert (d <= 1e-3 * np.maximum(np.abs(reflse), 1.0)).all(), "lse max delta %.3g" % d.max()


# shapes for the layouts with an output-index-contiguous operand: that index in whole 16-byte chunks (N, and M when A is
# stored transposed, multiples of 16); whole tiles | ragged in M, N and K | one short and one long contraction
LAYOUT_SHAPES = [(256, 256, 128), (512, 768, 384), (272, 528, 208), (208, 272, 144), (256, 512, 2048), (16, 16, 16)]


@pytest.mark.parametrize("transA,transB", [(False, False), (True, False), (True, True)])
@pytest.mark.parametrize("M,N,K", LAYOUT_SHAPES)
def test_f8_other_operand_layouts(oracle, M, N, K, transA, transB):
    """A stored [K x M] and / or B stored [K x N] in E4M3 (forward weights kept [in x out], the weight-gradient form
    A^T B): row scale + residual + row sum of squares against the oracle on the decoded bytes."""
    g = np.random.Generator(np.random.PCG64(1300 + M + K + 2 * transA + transB))
    A8 = synth.normal_f8e4m3(g, (K, M) if transA else (M, K), 1.0)
    B8 = synth.normal_f8e4m3(g, (N, K) if transB else (K, N), 1.0)
    A16, B16 = oracle.f8e4m3_to_bf16_bits(A8), oracle.f8e4m3_to_bf16_bits(B8)
    C = synth.normal_bf16(g, (M, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.02, 0.06)
    Y = G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dr, dC = G.dev_f32(r), G.dev_bf16(C)
    coda.coda_gemm(dev_u8(A8), dev_u8(B8), [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y.t)],
                   transA=transA, transB=transB)
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
    torch.cuda.synchronize()
    refD, refss = oracle.gemm_residual_sumsq(A16, B16, r=r.astype(np.float64), C=C, transA=transA, transB=transB)[:2]
    Y.check_guards(); Y.written()
    G.assert_bf16_close(G.host_f64(Y.t), refD, "f8 layout (%d, %d): row scale + residual" % (transA, transB))
    G.assert_sumsq_close(G.host_f64(ss), refss, "f8 layout (%d, %d): row sum of squares" % (transA, transB))


@pytest.mark.parametrize("transA,transB", [(False, False), (True, False), (True, True)])
def test_f8_other_layouts_decode_every_code_exactly(oracle, transA, transB):
    """The transposing read hands every byte to the right lane and k position: B (or A) selects single elements of the
    other operand, which holds every finite code, so D holds the decoded values themselves: exact in fp32."""
    M, N, K = 256, 256, 128
    codes = (np.arange(M * K, dtype=np.int64) * 7 % 256).astype(np.uint8).reshape(M, K)
    codes[(codes & 0x7F) == 0x7F] = 0
    sel = np.zeros((N, K), np.uint8)
    sel[np.arange(N), (np.arange(N) * 5 + 3) % K] = 0x38                # 1.0 at one k per column
    A8 = np.ascontiguousarray(codes.T) if transA else codes
    B8 = sel if transB else np.ascontiguousarray(sel.T)
    out = G.Guarded(M, N, torch.float32, pad_cols=4)
    coda.coda_gemm(dev_u8(A8), dev_u8(B8), [coda.store(out.t, f32=True)], transA=transA, transB=transB)
    torch.cuda.synchronize()
    out.check_guards(); out.written()
    ref = oracle.gemm_rowscale(oracle.f8e4m3_to_bf16_bits(A8), oracle.f8e4m3_to_bf16_bits(B8), transA=transA, transB=transB)
    got = G.host_f64(out.t)
    assert np.array_equal(got, ref), "max |delta| %.3g" % np.abs(got - ref).max()


def test_f8_weight_gradient_and_forward_weight_layouts_with_their_programs(oracle):
    """The two uses the other layouts exist for: the forward up-projection with the weight kept [in x out] (row scale +
    SwiGLU), and the weight gradient A^T B accumulated in fp32 with a split contraction."""
    g = np.random.Generator(np.random.PCG64(1400))
    M, N, K = 272, 512, 464
    X8, W8 = synth.normal_f8e4m3(g, (M, K), 1.0), synth.normal_f8e4m3(g, (K, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.02, 0.06)
    H = G.Guarded(M, N // 2, torch.bfloat16)
    Z = G.Guarded(M, N, torch.bfloat16)
    dr = G.dev_f32(r)
    coda.coda_gemm(dev_u8(X8), dev_u8(W8), [coda.row_scale(dr), coda.swiglu_fwd(Z.t), coda.store(H.t)])
    torch.cuda.synchronize()
    refH, refZ = oracle.gemm_rowscale_swiglu(oracle.f8e4m3_to_bf16_bits(X8), oracle.f8e4m3_to_bf16_bits(W8), r=r.astype(np.float64),
                                             want_preact=True)
    for t in (H, Z):
        t.check_guards(); t.written()
    G.assert_bf16_close(G.host_f64(H.t), refH, "f8 forward weight [in x out]: H")
    G.assert_bf16_close(G.host_f64(Z.t), refZ, "f8 forward weight [in x out]: pre-activation")
    # weight gradient: H^T dY over 4096 tokens into an existing fp32 buffer, with and without the workspace
    T, F, d = 4096, 512, 272
    H8, dY8 = synth.normal_f8e4m3(g, (T, F), 1.0), synth.normal_f8e4m3(g, (T, d + 0), 1.0)
    G0 = synth.normal_f32(g, (F, d), 1.0)
    need = coda.coda_gemm_workspace_bytes(F, d, T, [])
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda").fill_(0x5A)
    ref = oracle.gemm_accumulate(oracle.f8e4m3_to_bf16_bits(H8), oracle.f8e4m3_to_bf16_bits(dY8), G0, transA=True)
    for w in (None, ws):
        Gb = G.dev_f32(G0)
        coda.coda_gemm(dev_u8(H8), dev_u8(dY8), [coda.accum_f32(Gb)], transA=True, workspace=w)
        torch.cuda.synchronize()
        G.assert_f32_signed_close(G.host_f64(Gb), ref, "f8 weight gradient (workspace %s)" % (w is not None))


def test_f8_argument_errors(oracle):
    M, N, K = 256, 256, 128
    A8 = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
    B8 = torch.zeros((N, K), dtype=torch.uint8, device="cuda")
    Bb = torch.zeros((N, K), dtype=torch.bfloat16, device="cuda")
    Bn = torch.zeros((K, N + 16), dtype=torch.uint8, device="cuda")
    out = G.Guarded(M, N, torch.bfloat16)
    for a, b, kw, status in [(A8, Bb, dict(transB=True), "CODA_ERR_DTYPE"),            # mixed operand types
                             (A8, Bn[:, :N + 8], dict(), "CODA_ERR_SHAPE"),             # N-contiguous B: N not a multiple of 16
                             (A8[:, :72], B8[:, :72], dict(transB=True), "CODA_ERR_SHAPE")]:   # K not a multiple of 16
        with pytest.raises(coda.CodaError) as ei:
            coda.coda_gemm(a, b, [coda.store(out.t)], **kw)
        assert ei.value.status == getattr(coda, status)
    torch.cuda.synchronize()
    out.check_guards()


def test_f8_full_size_up_and_down_projection_sampled_rows(oracle):
    """The 8-bit kernels at the benchmark's 1B shapes, launched as bench.py launches them, checked on sampled output rows
    (every epilogue here is row-local, so the oracle computes exactly those rows)."""
    g = np.random.Generator(np.random.PCG64(1400))
    M, d, F = 8192, 2048, 8192
    rows = synth.sample_rows(M, 32, seed=5)
    # up-projection: row scale + SwiGLU
    X8, W8 = synth.normal_f8e4m3(g, (M, d), 1.0), synth.normal_f8e4m3(g, (2 * F, d), 1.0)
    r = synth.uniform_f32(g, (M,), 0.01, 0.03)
    H = torch.empty((M, F), dtype=torch.bfloat16, device="cuda")
    dr = G.dev_f32(r)
    coda.coda_gemm(dev_u8(X8), dev_u8(W8), [coda.row_scale(dr), coda.swiglu_fwd(), coda.store(H)], transB=True)
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale_swiglu(oracle.f8e4m3_to_bf16_bits(X8), oracle.f8e4m3_to_bf16_bits(W8), r=r.astype(np.float64),
                                      transB=True, rows=rows)
    G.assert_bf16_close(G.host_f64(H[torch.from_numpy(rows).cuda()]), ref, "f8 1B up")
    del H
    # down-projection: row scale (dequantisation) + residual + row sum of squares
    H8, Wd8 = synth.normal_f8e4m3(g, (M, F), 1.0), synth.normal_f8e4m3(g, (d, F), 1.0)
    R = synth.normal_bf16(g, (M, d), 1.0)
    r2 = synth.uniform_f32(g, (M,), 0.005, 0.015)
    Y = torch.empty((M, d), dtype=torch.bfloat16, device="cuda")
    nblk = coda.coda_row_partial_blocks(d)
    part = torch.empty((nblk, M), dtype=torch.float32, device="cuda")
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    dr2, dR = G.dev_f32(r2), G.dev_bf16(R)
    coda.coda_gemm(dev_u8(H8), dev_u8(Wd8), [coda.row_scale(dr2), coda.add_tile(dR), coda.row_sumsq(part), coda.store(Y)], transB=True)
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=d, eps=0.0)
    torch.cuda.synchronize()
    refY, refss = oracle.gemm_residual_sumsq(oracle.f8e4m3_to_bf16_bits(H8), oracle.f8e4m3_to_bf16_bits(Wd8), r=r2.astype(np.float64),
                                             C=R, transB=True, rows=rows)[:2]
    G.assert_bf16_close(G.host_f64(Y[torch.from_numpy(rows).cuda()]), refY, "f8 1B down")
    G.assert_sumsq_close(ss.cpu().numpy()[rows], refss, "f8 1B down sumsq")
