"""Full-size parity: the benchmark workloads at their real shapes, launched exactly as bench.py launches
them (same programs, same layouts, whole-tile kernel instantiation), checked on a deterministic sample of output rows
that the oracle computes one by one.  Every epilogue on the path is row-local, so sampled rows are exact; the
weight gradient is sampled over its own output rows.  The sample holds rows of EVERY 256-row tile (two per tile at the
1B shapes, one at the 8B shapes, plus the tile-boundary rows), and every output buffer starts out filled with a sentinel
that must be gone afterwards, so a tile that was never written or was written by the wrong workgroup cannot hide between
sampled rows."""
import numpy as np
import pytest
import torch

from paper_2605_19269_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu
coda = None
PER_TILE = 2          # sampled rows per 256-row tile (1B shapes); the 8B shapes take one


def sentinel_bf16(shape):
    t = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    t.view(torch.int16).fill_(int(np.uint16(G.SENTINEL_BF16).view(np.int16)))
    return t


def sentinel_f32(shape):
    return torch.full(shape, G.SENTINEL_F32, dtype=torch.float32, device="cuda")


def assert_all_written(t, what):
    """No sentinel survives anywhere in the output (checked on the device over the whole tensor)."""
    if t.dtype == torch.bfloat16:
        left = int((t.view(torch.int16) == int(np.uint16(G.SENTINEL_BF16).view(np.int16))).sum().item())
    else:
        left = int((t == G.SENTINEL_F32).sum().item())
    assert left == 0, "%s: %d elements were never written" % (what, left)


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global coda
    assert torch.cuda.is_available()
    from paper_2605_19269_amd import coda as _c
    coda = _c
    yield
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


def rows_of(t, rows):
    return G.host_f64(t[torch.from_numpy(rows).cuda()])


def gpu_rstd(X, eps=1e-6):
    M, d = X.shape
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    r = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_row_sumsq(X, ss)
    coda.coda_row_finalize(ss.view(1, M), M, 1, rstd_out=r, d=d, eps=eps)
    return r


def check_up(oracle, Xb, Wb, tag, per_tile=PER_TILE):
    M, N = Xb.shape[0], Wb.shape[1]
    rows = synth.sample_rows_per_tile(M, per_tile, seed=3)
    X, W = G.dev_bf16(Xb), G.dev_bf16(Wb)
    r = gpu_rstd(X)
    H = sentinel_bf16((M, N // 2))
    coda.coda_gemm(X, W, [coda.row_scale(r), coda.swiglu_fwd(), coda.store(H)])
    torch.cuda.synchronize()
    assert_all_written(H, tag + " H")
    r_host = r.cpu().numpy()
    G.assert_sumsq_close(r_host[rows], oracle.rstd(Xb, 1e-6, rows=rows), tag + " rstd")
    ref = oracle.gemm_rowscale_swiglu(Xb, Wb, r=r_host.astype(np.float64), rows=rows)   # same fp32 r bytes as the GPU
    G.assert_bf16_close(rows_of(H, rows), ref, tag + " H")


def check_down(oracle, Hb, Wb, Rb, tag, per_tile=PER_TILE):
    M, N = Hb.shape[0], Wb.shape[1]
    rows = synth.sample_rows_per_tile(M, per_tile, seed=4)
    Y = sentinel_bf16((M, N))
    nblk = coda.coda_row_partial_blocks(N)
    part = sentinel_f32((nblk, M))
    ss = sentinel_f32((M,))
    dR = G.dev_bf16(Rb)
    coda.coda_gemm(G.dev_bf16(Hb), G.dev_bf16(Wb), [coda.add_tile(dR), coda.row_sumsq(part), coda.store(Y)])
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=N, eps=0.0)
    torch.cuda.synchronize()
    assert_all_written(Y, tag + " Y"); assert_all_written(part, tag + " partials"); assert_all_written(ss, tag + " sumsq")
    refY, refss = oracle.gemm_residual_sumsq(Hb, Wb, C=Rb, rows=rows)
    G.assert_bf16_close(rows_of(Y, rows), refY, tag + " Y")
    G.assert_sumsq_close(ss.cpu().numpy()[rows], refss, tag + " sumsq")


def test_llama1b_up_projection(oracle):
    c = synth.up_projection(seed=0)
    check_up(oracle, c["X"], c["W"], "1B up")


def test_llama1b_down_projection(oracle):
    c = synth.down_projection(seed=1)
    check_down(oracle, c["H"], c["W"], c["R"], "1B down")


def test_llama1b_mlp_backward(oracle):
    c = synth.mlp_backward(seed=2)
    M, d = c["dY"].shape
    F = c["W"].shape[0]
    dY, W, Z, H = G.dev_bf16(c["dY"]), G.dev_bf16(c["W"]), G.dev_bf16(c["Z"]), G.dev_bf16(c["H"])
    dZ = sentinel_bf16((M, 2 * F))
    coda.coda_gemm(dY, W, [coda.swiglu_bwd(Z), coda.store(dZ)], transB=True)
    Gb = torch.from_numpy(c["G"]).cuda()
    G0 = Gb.clone()
    coda.coda_gemm(H, dY, [coda.accum_f32(Gb)], transA=True)
    torch.cuda.synchronize()
    assert_all_written(dZ, "1B dZ")
    # the accumulate works in place: every element must have moved (increments are ~N(0, 0.9) on values ~1e-3)
    assert int((Gb == G0).sum().item()) <= 2, "1B dW accumulate left elements untouched"
    del G0
    rows = synth.sample_rows_per_tile(M, PER_TILE, seed=5)
    refdZ, _, _ = oracle.gemm_swiglu_bwd(c["dY"], c["W"], c["Z"], transB=True, rows=rows)
    G.assert_bf16_close(rows_of(dZ, rows), refdZ, "1B dZ")
    wrows = synth.sample_rows_per_tile(F, PER_TILE, seed=6)
    refG = oracle.gemm_accumulate(c["H"], c["dY"], c["G"], transA=True, rows=wrows)
    G.assert_f32_signed_close(rows_of(Gb, wrows), refG, "1B dW accumulate")


def test_llama8b_block_shapes(oracle):
    """LLaMA-3-8B-style shapes: QKV projection with row scale, up-projection with SwiGLU, down-projection with
    residual add and sum of squares (M = 16384, d = 4096, F = 14336)."""
    c = synth.block_8b(seed=7)
    M = c["X"].shape[0]
    rows = synth.sample_rows_per_tile(M, 1, seed=8)
    X = G.dev_bf16(c["X"])
    r = gpu_rstd(X)
    r_host = r.cpu().numpy().astype(np.float64)
    Q = sentinel_bf16((M, c["Wqkv"].shape[1]))
    coda.coda_gemm(X, G.dev_bf16(c["Wqkv"]), [coda.row_scale(r), coda.store(Q)])
    torch.cuda.synchronize()
    assert_all_written(Q, "8B qkv")
    G.assert_bf16_close(rows_of(Q, rows), oracle.gemm_rowscale(c["X"], c["Wqkv"], r=r_host, rows=rows), "8B qkv")
    # the same projection with RoPE on the query and key heads (32 + 8 heads of 128; value heads pass through)
    Q.view(torch.int16).fill_(int(np.uint16(G.SENTINEL_BF16).view(np.int16)))
    hd, rc, T = 128, 5120, 2048
    cos, sin = synth.rope_tables(T, hd)
    pos = (np.arange(M) % T).astype(np.int32)
    dcos, dsin, dpos = G.dev_f32(cos), G.dev_f32(sin), torch.from_numpy(pos).cuda()
    coda.coda_gemm(X, G.dev_bf16(c["Wqkv"]), [coda.row_scale(r), coda.rope(dcos, dsin, dpos, hd, rc), coda.store(Q)])
    torch.cuda.synchronize()
    assert_all_written(Q, "8B qkv + rope")
    G.assert_bf16_close(rows_of(Q, rows), oracle.gemm_rowscale_rope(c["X"], c["Wqkv"], cos, sin, pos, hd, rc, r=r_host, rows=rows),
                        "8B qkv + rope")
    del Q
    check_up(oracle, c["X"], c["Wup"], "8B up", per_tile=1)
    check_down(oracle, c["H"], c["Wdown"], c["R"], "8B down", per_tile=1)


def test_llama8b_rmsnorm_backward(oracle):
    """Kernel 9 at the 8B QKV-projection backward shape: D = dY[M x 6144] Wqkv^T -> [M x 4096], with residual-gradient
    accumulation, the recomputed normalised activation and the dgamma column partials.  O_out / C_out are checked on
    sampled rows; dgamma (a reduction over ALL rows) on sampled columns, by giving the oracle the column-sliced
    weight, C, gamma and O_in (every quantity of the kernel is column-local once D is formed)."""
    g = np.random.Generator(np.random.PCG64(9))
    M, N, K = 16384, 4096, 6144
    dY = synth.normal_bf16(g, (M, K), 1e-2)
    W = synth.normal_bf16(g, (N, K), 0.02)            # forward weight [d x 6144], used transposed
    Cb = synth.normal_bf16(g, (M, N), 1.0)
    Oin = synth.normal_bf16(g, (M, N), 1e-2)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    z = synth.normal_f32(g, (M,), 1e-3)
    gamma = synth.uniform_f32(g, (N,), 0.5, 1.5)
    Oout, Cout = sentinel_bf16((M, N)), sentinel_bf16((M, N))
    nblk = coda.coda_col_partial_blocks(M)
    part = sentinel_f32((nblk, N))
    dg = torch.empty(N, dtype=torch.float32, device="cuda")
    dC, dr, dz, dgm, dO = G.dev_bf16(Cb), G.dev_f32(r), G.dev_f32(z), G.dev_f32(gamma), G.dev_bf16(Oin)
    coda.coda_gemm(G.dev_bf16(dY), G.dev_bf16(W),
                   [coda.rmsnorm_bwd(dC, dr, dz, dgm, c_out=Cout, dgamma_out=part), coda.add_tile(dO), coda.store(Oout)], transB=True)
    coda.coda_col_finalize(part, N, nblk, dg)
    torch.cuda.synchronize()
    assert_all_written(Oout, "8B O_out"); assert_all_written(Cout, "8B C_out"); assert_all_written(part, "8B dgamma partials")
    rows = synth.sample_rows_per_tile(M, 1, seed=10)
    r64, z64, g64 = r.astype(np.float64), z.astype(np.float64), gamma.astype(np.float64)
    refO, refC, _ = oracle.gemm_rmsnorm_bwd(dY, W, Cb, r64, z64, g64, Oin=Oin, transB=True, rows=rows)
    G.assert_bf16_close(rows_of(Oout, rows), refO, "8B O_out")
    G.assert_bf16_close(rows_of(Cout, rows), refC, "8B C_out")
    cols = np.sort(g.choice(N, size=24, replace=False))
    _, _, refdg = oracle.gemm_rmsnorm_bwd(dY, np.ascontiguousarray(W[cols]), np.ascontiguousarray(Cb[:, cols]), r64, z64,
                                          g64[cols], Oin=None, transB=True)
    G.assert_f32_signed_close(dg.cpu().numpy()[cols].astype(np.float64), refdg, "8B dgamma")


def test_lm_head_logits_lse(oracle):
    """Kernel 8 at an LM-head shape (tokens 8192, hidden 4096, vocabulary 32768): logits, target logit, lse, loss."""
    g = np.random.Generator(np.random.PCG64(11))
    M, K, N = 8192, 4096, 32768
    Xb = synth.normal_bf16(g, (M, K), 1.0)
    Wb = synth.normal_bf16(g, (K, N), 0.02)
    y = g.integers(0, N, size=M).astype(np.int32)
    X = G.dev_bf16(Xb)
    r = gpu_rstd(X)
    Z = sentinel_bf16((M, N))
    nblk = coda.coda_row_partial_blocks(N)
    pmax, psum = sentinel_f32((nblk, M)), sentinel_f32((nblk, M))
    zt, lse, loss = (sentinel_f32((M,)) for _ in range(3))
    dy = torch.from_numpy(y).cuda()
    coda.coda_gemm(X, G.dev_bf16(Wb), [coda.row_scale(r), coda.lse_partial(dy, pmax, psum, zt), coda.store(Z)])
    coda.coda_lse_finalize(pmax, psum, M, nblk, ztgt=zt, lse_out=lse, loss_out=loss)
    torch.cuda.synchronize()
    for t, what in ((Z, "logits"), (pmax, "max partials"), (psum, "sum-exp partials"), (zt, "target logit"), (lse, "lse"), (loss, "loss")):
        assert_all_written(t, "LM-head " + what)
    rows = synth.sample_rows_per_tile(M, 1, seed=12)
    refZ, refzt, reflse = oracle.gemm_rowscale_lse(Xb, Wb, y, r=r.cpu().numpy().astype(np.float64), rows=rows)
    G.assert_bf16_close(rows_of(Z, rows), refZ, "LM-head logits")
    G.assert_f32_signed_close(zt.cpu().numpy()[rows].astype(np.float64), refzt, "LM-head target logit")
    d = np.abs(lse.cpu().numpy()[rows].astype(np.float64) - reflse)
    assert (d <= 1e-3 * np.maximum(np.abs(reflse), 1.0)).all(), "lse max delta %.3g" % d.max()
    G.assert_f32_signed_close(loss.cpu().numpy()[rows].astype(np.float64), reflse - refzt, "LM-head loss")


def test_llama1b_forward_gemms_on_f8e4m3_operands(oracle):
    """The 8-bit-operand variant at the step's forward shapes, launched as bench.py launches it, on sampled rows:
    up-projection (row scale carrying rstd times a quantisation scale, SwiGLU) and down-projection (row scale,
    residual, sum of squares).  Operands ~ N(0,1) rounded to E4M3; the weights are stored [out x in]."""
    M, d, F = 8192, 2048, 8192
    g = np.random.Generator(np.random.PCG64(31))
    rows = synth.sample_rows_per_tile(M, 1, seed=5)
    X8, W8 = synth.normal_f8e4m3(g, (M, d), 1.0), synth.normal_f8e4m3(g, (2 * F, d), 1.0)
    r = synth.uniform_f32(g, (M,), 0.01, 0.03)
    dr = G.dev_f32(r)
    H = sentinel_bf16((M, F))
    coda.coda_gemm(torch.from_numpy(X8).cuda(), torch.from_numpy(W8).cuda(), [coda.row_scale(dr), coda.swiglu_fwd(), coda.store(H)],
                   transB=True)
    torch.cuda.synchronize()
    assert_all_written(H, "1B up, E4M3 operands")
    ref = oracle.gemm_rowscale_swiglu(oracle.f8e4m3_to_bf16_bits(X8), oracle.f8e4m3_to_bf16_bits(W8), r=r.astype(np.float64),
                                      transB=True, rows=rows)
    G.assert_bf16_close(rows_of(H, rows), ref, "1B up, E4M3 operands")
    del X8, W8, H
    H8, Wd8 = synth.normal_f8e4m3(g, (M, F), 1.0), synth.normal_f8e4m3(g, (d, F), 1.0)
    Rb = synth.normal_bf16(g, (M, d), 1.0)
    r2 = synth.uniform_f32(g, (M,), 0.005, 0.015)
    dr2, dR = G.dev_f32(r2), G.dev_bf16(Rb)
    Y = sentinel_bf16((M, d))
    nblk = coda.coda_row_partial_blocks(d)
    part = sentinel_f32((nblk, M))
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    coda.coda_gemm(torch.from_numpy(H8).cuda(), torch.from_numpy(Wd8).cuda(),
                   [coda.row_scale(dr2), coda.add_tile(dR), coda.row_sumsq(part), coda.store(Y)], transB=True)
    coda.coda_row_finalize(part, M, nblk, sum_out=ss, d=d, eps=0.0)
    torch.cuda.synchronize()
    assert_all_written(Y, "1B down, E4M3 operands"); assert_all_written(part, "1B down partials, E4M3 operands")
    refY, refss = oracle.gemm_residual_sumsq(oracle.f8e4m3_to_bf16_bits(H8), oracle.f8e4m3_to_bf16_bits(Wd8), r=r2.astype(np.float64),
                                             C=Rb, transB=True, rows=rows)[:2]
    G.assert_bf16_close(rows_of(Y, rows), refY, "1B down, E4M3 operands")
    G.assert_sumsq_close(ss.cpu().numpy()[rows], refss, "1B down sumsq, E4M3 operands")


def test_operands_and_outputs_beyond_4_gib(oracle):
    """Byte offsets past 2^32 in an operand (A: 140000 x 16384 bf16 = 4.6 GB) and in an output (140000 x 16384 bf16),
    with a ragged M: sampled rows, most of them past the 4 GiB mark, against the oracle on exactly those rows."""
    M = 140000
    gen = torch.Generator(device="cuda").manual_seed(11)
    rows = np.concatenate([[0, 1, 131071, 131072, M - 1],
                           np.random.Generator(np.random.PCG64(12)).integers(131072, M, size=19)]).astype(np.int64)
    drows = torch.from_numpy(rows).cuda()

    def bits(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

    # large A, narrow output
    K, N = 16384, 256
    A = torch.randn((M, K), generator=gen, device="cuda", dtype=torch.bfloat16)
    B = (torch.randn((K, N), generator=gen, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    r = torch.rand(M, generator=gen, device="cuda", dtype=torch.float32) + 0.5
    out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    coda.coda_gemm(A, B, [coda.row_scale(r), coda.store(out)])
    torch.cuda.synchronize()
    ref = oracle.gemm_rowscale(bits(A[drows]), bits(B), r=r[drows].cpu().numpy().astype(np.float64))
    G.assert_bf16_close(G.host_f64(out[drows]), ref, "A beyond 4 GiB")
    del A, out
    torch.cuda.empty_cache()
    # short contraction, large output (pairwise forward halves it: H is 140000 x 16384, its pre-activation twice that)
    K, N = 64, 32768
    A = torch.randn((M, K), generator=gen, device="cuda", dtype=torch.bfloat16)
    B = (torch.randn((K, N), generator=gen, device="cuda", dtype=torch.float32) * 0.2).to(torch.bfloat16)
    H = torch.empty((M, N // 2), dtype=torch.bfloat16, device="cuda")
    Z = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    coda.coda_gemm(A, B, [coda.row_scale(r), coda.swiglu_fwd(Z), coda.store(H)])
    torch.cuda.synchronize()
    refH, refZ = oracle.gemm_rowscale_swiglu(bits(A[drows]), bits(B), r=r[drows].cpu().numpy().astype(np.float64), want_preact=True)
    G.assert_bf16_close(G.host_f64(H[drows]), refH, "H beyond 4 GiB")
    G.assert_bf16_close(G.host_f64(Z[drows]), refZ, "Z beyond 4 GiB")


def test_transposed_operand_beyond_4_gib_with_k_tail(oracle):
    """A stored [K x M] with K = 140000 tokens (4.6 GB; K is not a multiple of the K-step): the weight-gradient form
    G += A^T B in fp32, checked on sampled output rows (= columns of the stored A)."""
    Kt, M, N = 140000, 16384, 256
    gen = torch.Generator(device="cuda").manual_seed(13)
    A = torch.randn((Kt, M), generator=gen, device="cuda", dtype=torch.bfloat16)
    B = (torch.randn((Kt, N), generator=gen, device="cuda", dtype=torch.float32) * 1e-2).to(torch.bfloat16)
    G0 = torch.randn((M, N), generator=gen, device="cuda", dtype=torch.float32) * 1e-3
    Gw = G0.clone()
    coda.coda_gemm(A, B, [coda.accum_f32(Gw)], transA=True)
    torch.cuda.synchronize()
    cols = np.concatenate([[0, 255, 256, M - 1], np.random.Generator(np.random.PCG64(14)).integers(0, M, size=12)]).astype(np.int64)
    dcols = torch.from_numpy(cols).cuda()

    def bits(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

    ref = oracle.gemm_accumulate(bits(A[:, dcols]), bits(B), G0[dcols].cpu().numpy(), transA=True)
    G.assert_f32_signed_close(G.host_f64(Gw[dcols]), ref, "A^T beyond 4 GiB")


def test_full_size_launches_repeat_bitwise_with_every_cu_busy():
    """The three mainloop layouts of the benchmark step at their real shapes, twenty launches each with every compute unit
    busy and several rounds of tiles: each repeat must reproduce the first launch bit for bit (a read of an LDS ring slot
    that races its refill, or a wait that is one load short, shows up as a difference here long before it shows in a
    sampled comparison), and the operands must be untouched."""
    dev = "cuda"
    g = torch.Generator(device=dev); g.manual_seed(31)
    def bf(shape, std):
        return (torch.randn(shape, generator=g, device=dev) * std).to(torch.bfloat16)
    M, d, F = 8192, 2048, 8192
    X, W = bf((M, d), 1.0), bf((d, 2 * F), 0.02)
    r = torch.rand(M, generator=g, device=dev) + 0.5
    dY, Wd = bf((M, d), 1e-2), bf((F, d), 0.02)          # dY * Wd^T: both K-contiguous
    Z = bf((M, 2 * F), 1.0)
    H = bf((M, F), 1.0)                                  # H^T dY: both token-major, contraction over tokens
    cases = [
        ("up-projection A*B", lambda out: coda.coda_gemm(X, W, [coda.row_scale(r), coda.swiglu_fwd(), coda.store(out)]), (M, F), torch.bfloat16, [X, W]),
        ("SwiGLU backward A*B^T", lambda out: coda.coda_gemm(dY, Wd, [coda.swiglu_bwd(Z), coda.store(out)], transB=True), (M, 2 * F), torch.bfloat16, [dY, Wd, Z]),
        ("weight gradient A^T*B", lambda out: coda.coda_gemm(H, dY, [coda.store(out, f32=True)], transA=True), (F, d), torch.float32, [H, dY]),
    ]
    for name, launch, shape, dt, inputs in cases:
        before = [t.clone() for t in inputs]
        first = torch.empty(shape, dtype=dt, device=dev)
        launch(first)
        torch.cuda.synchronize()
        again = torch.empty(shape, dtype=dt, device=dev)
        for rep in range(20):
            again.view(torch.uint8).fill_(0xA5)
            launch(again)
            torch.cuda.synchronize()
            assert torch.equal(again.view(torch.uint8), first.view(torch.uint8)), "%s: launch %d differs from the first" % (name, rep + 2)
        for t, t0 in zip(inputs, before):
            assert torch.equal(t.view(torch.uint8), t0.view(torch.uint8)), "%s: an operand was modified" % name
        del first, again, before
    torch.cuda.empty_cache()
