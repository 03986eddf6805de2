"""GPU parity of split-K: shapes with few output tiles and a long contraction, run with the workspace that lets
several workgroups share a tile.  Results must match the oracle to the same bar as the unsplit kernels, must not
depend on which workgroup finishes last (bitwise equal across repeats), and the workspace rules of the C ABI hold."""
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


def workspace(M, N, K, poison=True):
    need = coda.coda_gemm_workspace_bytes(M, N, K, [])
    assert need > 0, "shape should be planned for split-K"
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    if poison:
        ws.fill_(0xA5)            # the library must not rely on the workspace's contents
    return ws


def operands(g, M, N, K, transA, transB, a_std=1.0, b_std=0.05):
    A = synth.normal_bf16(g, (K, M) if transA else (M, K), a_std)
    B = synth.normal_bf16(g, (N, K) if transB else (K, N), b_std)
    return A, B


# (M, N, K) -> parts: 4 tiles, K = 4096 -> 4;  1 tile, K = 8192 -> 8;  2 tiles, K = 3072 -> 3;
# 1 tile, K = 6272 (196 K-steps of 32) -> 6 parts of 32 or 34 steps;
# 2 x 2 tiles with a ragged edge in M and N, K = 4096 -> 4; the same with a ragged K = 4168 (132 K-steps) -> 4 parts of 32 or 34
SHAPES = [(512, 512, 4096), (256, 256, 8192), (256, 512, 3072), (256, 256, 6272), (504, 264, 4096), (504, 264, 4168)]


@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, False)])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_splitk_linear_program(oracle, M, N, K, transA, transB):
    g = np.random.Generator(np.random.PCG64(900 + M + K + 2 * transA + transB))
    A, B = operands(g, M, N, K, transA, transB)
    C = synth.normal_bf16(g, (M, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    nblk = coda.coda_row_partial_blocks(N)
    dA, dB, dr, dC = G.dev_bf16(A), G.dev_bf16(B), G.dev_f32(r), G.dev_bf16(C)
    ws = workspace(M, N, K)
    outs = []
    for rep in range(2):
        Y = G.Guarded(M, N, torch.bfloat16)
        part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
        coda.coda_gemm(dA, dB, [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y.t)],
                       transA=transA, transB=transB, workspace=ws)
        ss = torch.empty(M, dtype=torch.float32, device="cuda")
        coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
        torch.cuda.synchronize()
        Y.check_guards(); Y.written()
        outs.append((Y.t.clone(), ss.clone()))
    refD, refss = oracle.gemm_residual_sumsq(A, B, r=r.astype(np.float64), C=C, transA=transA, transB=transB)[:2]
    G.assert_bf16_close(G.host_f64(outs[0][0]), refD, "split-K row scale + residual")
    G.assert_sumsq_close(G.host_f64(outs[0][1]), refss, "split-K row sum of squares")
    assert torch.equal(outs[0][0].view(torch.int16), outs[1][0].view(torch.int16)), "repeat differs: order-dependent sum"
    assert torch.equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_splitk_swiglu_forward_and_backward(oracle, M, N, K):
    g = np.random.Generator(np.random.PCG64(950 + M + K))
    A, B = operands(g, M, N, K, False, False)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    ws = workspace(M, N, K)
    H = G.Guarded(M, N // 2, torch.bfloat16)
    Zs = G.Guarded(M, N, torch.bfloat16)
    dr = G.dev_f32(r)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.row_scale(dr), coda.swiglu_fwd(Zs.t), coda.store(H.t)], workspace=ws)
    torch.cuda.synchronize()
    refH, refZ = oracle.gemm_rowscale_swiglu(A, B, r=r.astype(np.float64), want_preact=True)
    H.check_guards(); H.written(); Zs.check_guards(); Zs.written()
    G.assert_bf16_close(G.host_f64(H.t), refH, "split-K swiglu forward")
    G.assert_bf16_close(G.host_f64(Zs.t), refZ, "split-K pre-activation")
    # backward: dY [M x K] W^T with W stored [N x K]
    A2 = synth.normal_bf16(g, (M, K), 1e-2)
    Bt = synth.normal_bf16(g, (N, K), 0.02)
    Z = synth.normal_bf16(g, (M, 2 * N), 1.0)
    dZ = G.Guarded(M, 2 * N, torch.bfloat16)
    nblk = coda.coda_row_partial_blocks(N)
    part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dZin = G.dev_bf16(Z)
    coda.coda_gemm(G.dev_bf16(A2), G.dev_bf16(Bt), [coda.swiglu_bwd(dZin, stat_out=part), coda.store(dZ.t)], transB=True, workspace=ws)
    stat = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_finalize(part, M, nblk, sum_out=stat, d=1, eps=0.0)
    torch.cuda.synchronize()
    refdZ, _, refstat = oracle.gemm_swiglu_bwd(A2, Bt, Z, transB=True)
    dZ.check_guards(); dZ.written()
    G.assert_bf16_close(G.host_f64(dZ.t), refdZ, "split-K dZ")
    G.assert_f32_signed_close(G.host_f64(stat), refstat, "split-K row statistic")


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_splitk_accumulate_and_rmsnorm_backward(oracle, M, N, K):
    g = np.random.Generator(np.random.PCG64(970 + M + K))
    ws = workspace(M, N, K)
    # weight gradient: A^T B with A stored [K x M]
    A, B = operands(g, M, N, K, True, False, b_std=1e-2)
    Gin = synth.normal_f32(g, (M, N), 1e-3)
    buf = G.Guarded(M, N, torch.float32, pad_cols=4)
    buf.t.copy_(torch.from_numpy(Gin))
    buf.ref = buf.full.clone()
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B), [coda.accum_f32(buf.t)], transA=True, workspace=ws)
    torch.cuda.synchronize()
    buf.check_guards()
    G.assert_f32_signed_close(G.host_f64(buf.t), oracle.gemm_accumulate(A, B, Gin, transA=True), "split-K fp32 accumulate")
    # RMSNorm backward on A B^T
    A, B = operands(g, M, N, K, False, True, b_std=0.05)
    Cb, Oin = synth.normal_bf16(g, (M, N), 1.0), synth.normal_bf16(g, (M, N), 1.0)
    r, z = synth.uniform_f32(g, (M,), 0.5, 1.5), synth.normal_f32(g, (M,), 0.3)
    gamma = synth.uniform_f32(g, (N,), 0.5, 1.5)
    Oout, Cout = G.Guarded(M, N, torch.bfloat16), G.Guarded(M, N, torch.bfloat16)
    nblk = coda.coda_col_partial_blocks(M)
    dgp = torch.full((nblk, N), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    dC, dr, dz, dgm, dO = G.dev_bf16(Cb), G.dev_f32(r), G.dev_f32(z), G.dev_f32(gamma), G.dev_bf16(Oin)
    coda.coda_gemm(G.dev_bf16(A), G.dev_bf16(B),
                   [coda.rmsnorm_bwd(dC, dr, dz, dgm, c_out=Cout.t, dgamma_out=dgp), coda.add_tile(dO), coda.store(Oout.t)],
                   transB=True, workspace=ws)
    dg = torch.empty(N, dtype=torch.float32, device="cuda")
    coda.coda_col_finalize(dgp, N, nblk, dg)
    torch.cuda.synchronize()
    refO, refC, refdg = oracle.gemm_rmsnorm_bwd(A, B, Cb, r.astype(np.float64), z.astype(np.float64), gamma.astype(np.float64),
                                                Oin=Oin, transB=True)
    Oout.check_guards(); Oout.written(); Cout.check_guards(); Cout.written()
    G.assert_bf16_close(G.host_f64(Oout.t), refO, "split-K O_out")
    G.assert_bf16_close(G.host_f64(Cout.t), refC, "split-K C_out")
    G.assert_f32_signed_close(G.host_f64(dg), refdg, "split-K dgamma")


def test_splitk_workspace_rules(oracle):
    M, N, K = 512, 512, 4096
    g = np.random.Generator(np.random.PCG64(991))
    A, B = operands(g, M, N, K, False, False)
    dA, dB = G.dev_bf16(A), G.dev_bf16(B)
    need = coda.coda_gemm_workspace_bytes(M, N, K, [])
    assert need == 1024 + 4 * 4 * 256 * 256 * 4          # counters + tiles x parts x one fp32 tile
    # shapes that are not split ask for nothing: whole rounds of tiles, a short K
    assert coda.coda_gemm_workspace_bytes(8192, 8192, 8192, []) == 0
    assert coda.coda_gemm_workspace_bytes(512, 512, 1024, []) == 0
    assert coda.coda_gemm_workspace_bytes(520, 512, 4096, []) == 1024 + 6 * 4 * 256 * 256 * 4   # ragged M: 3 x 2 tiles
    out = G.Guarded(M, N, torch.bfloat16)
    small = torch.empty(need - 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(coda.CodaError) as ei:
        coda.coda_gemm(dA, dB, [coda.store(out.t)], workspace=small)
    assert ei.value.status == coda.CODA_ERR_WORKSPACE
    out.check_guards()                                      # nothing was enqueued
    # a workspace on a shape that is not split is accepted and ignored
    A2, B2 = operands(g, 264, 520, 72, False, False)
    o2 = G.Guarded(264, 520, torch.bfloat16)
    coda.coda_gemm(G.dev_bf16(A2), G.dev_bf16(B2), [coda.store(o2.t)], workspace=small)
    # split and unsplit runs of the same problem agree to fp32 summation-order noise
    ws = workspace(M, N, K)
    o_split, o_plain = G.Guarded(M, N, torch.float32, pad_cols=4), G.Guarded(M, N, torch.float32, pad_cols=4)
    coda.coda_gemm(dA, dB, [coda.store(o_split.t, f32=True)], workspace=ws)
    coda.coda_gemm(dA, dB, [coda.store(o_plain.t, f32=True)])
    torch.cuda.synchronize()
    o2.check_guards(); o2.written()
    G.assert_bf16_close(G.host_f64(o2.t), oracle.gemm_rowscale(A2, B2), "workspace ignored on a ragged shape")
    ref = oracle.gemm_rowscale(A, B)
    G.assert_f32_signed_close(G.host_f64(o_split.t), ref, "split-K f32 store")
    G.assert_f32_signed_close(G.host_f64(o_plain.t), ref, "unsplit f32 store")


@pytest.mark.parametrize("transB", [False, True])
def test_splitk_last_round_only(oracle, transB):
    """320 output tiles: the 256 tiles of the first round run whole, the 64 of the last round are shared by 4 workgroups
    each.  Checked on sampled rows of every tile row (the program is row-local), against the oracle and against the
    unsplit run of the same shape, and bitwise across repeats."""
    M, N, K = 5120, 4096, 4096
    g = np.random.Generator(np.random.PCG64(990 + transB))
    A, B = operands(g, M, N, K, False, transB, b_std=0.02)
    C = synth.normal_bf16(g, (M, N), 1.0)
    rows = np.sort(np.concatenate([np.arange(0, M, 256) + 3, np.arange(0, M, 256) + 250]))
    nblk = coda.coda_row_partial_blocks(N)
    dA, dB, dC = G.dev_bf16(A), G.dev_bf16(B), G.dev_bf16(C)
    ws = workspace(M, N, K)
    assert ws.numel() == 1024 + 64 * 4 * 256 * 256 * 4
    outs = []
    for w in (ws, ws, None):
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        part = torch.empty((nblk, M), dtype=torch.float32, device="cuda")
        ss = torch.empty(M, dtype=torch.float32, device="cuda")
        coda.coda_gemm(dA, dB, [coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y)], transB=transB, workspace=w)
        coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
        torch.cuda.synchronize()
        outs.append((Y, ss))
    refD, refss = oracle.gemm_residual_sumsq(A, B, C=C, transB=transB, rows=rows)[:2]
    idx = torch.from_numpy(rows).cuda()
    G.assert_bf16_close(G.host_f64(outs[0][0][idx]), refD, "last-round split-K residual")
    G.assert_sumsq_close(G.host_f64(outs[0][1][idx]), refss, "last-round split-K row sum of squares")
    assert torch.equal(outs[0][0].view(torch.int16), outs[1][0].view(torch.int16)), "repeat differs: order-dependent sum"
    assert torch.equal(outs[0][1], outs[1][1])
    # against the unsplit kernel: same products, different fp32 summation order in the shared tiles only
    d = (outs[0][0].float() - outs[2][0].float()).abs().max().item()
    assert d <= 0.0625, d          # at most one bf16 step of values of magnitude ~4
    eq = (outs[0][0].view(torch.int16) == outs[2][0].view(torch.int16)).view(M // 256, 256, N // 256, 256)
    same_tiles = eq.all(dim=3).all(dim=1).sum().item()
    assert same_tiles >= 256, "the tiles of the first round must run whole (bitwise equal to the unsplit launch): %d" % same_tiles


@pytest.mark.parametrize("M,N,K,transA", [(2560, 1024, 8192, False), (2500, 1000, 8200, False), (2560, 1024, 8192, True)])
def test_balanced_round_with_ranges_that_straddle_tiles(oracle, M, N, K, transA):
    """40 output tiles with a long contraction: 8 parts each would need 320 workgroups, so the K-steps of all tiles, laid end
    to end, are cut into 256 equal ranges; most ranges end in one tile and begin in the next (a workgroup then runs two
    work items), and a tile is finished by whichever of its up to 8 contributors arrives last.  Whole and ragged shapes,
    both A layouts; sampled rows of every tile row against the oracle, bitwise equal across repeats."""
    g = np.random.Generator(np.random.PCG64(1200 + M + K + transA))
    A, B = operands(g, M, N, K, transA, False, b_std=0.02)
    C = synth.normal_bf16(g, (M, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    need = coda.coda_gemm_workspace_bytes(M, N, K, [])
    tiles = -(-M // 256) * -(-N // 256)
    assert tiles == 40 and need > 1024 + tiles * 7 * 256 * 256 * 4, "expected the straddling plan (more slots than equal parts)"
    ws = torch.empty(need, dtype=torch.uint8, device="cuda").fill_(0xA5)
    dA, dB, dC, dr = G.dev_bf16(A), G.dev_bf16(B), G.dev_bf16(C), G.dev_f32(r)
    nblk = coda.coda_row_partial_blocks(N)
    outs = []
    for rep in range(2):
        Y = G.Guarded(M, N, torch.bfloat16)
        part = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
        ss = torch.empty(M, dtype=torch.float32, device="cuda")
        coda.coda_gemm(dA, dB, [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y.t)], transA=transA, workspace=ws)
        coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
        torch.cuda.synchronize()
        Y.check_guards(); Y.written()
        assert int((part == G.SENTINEL_F32).sum().item()) == 0
        outs.append((Y.t.clone(), ss.clone()))
    rows = synth.sample_rows_per_tile(M, 2, seed=77)
    refD, refss = oracle.gemm_residual_sumsq(A, B, r=r.astype(np.float64), C=C, transA=transA, rows=rows)[:2]
    idx = torch.from_numpy(rows).cuda()
    G.assert_bf16_close(G.host_f64(outs[0][0][idx]), refD, "balanced round: row scale + residual")
    G.assert_sumsq_close(G.host_f64(outs[0][1][idx]), refss, "balanced round: row sum of squares")
    assert torch.equal(outs[0][0].view(torch.int16), outs[1][0].view(torch.int16)), "repeat differs: order-dependent sum"
    assert torch.equal(outs[0][1], outs[1][1])
