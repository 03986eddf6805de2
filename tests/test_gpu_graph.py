"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
sequence of its calls can be captured into a HIP graph.  Captured here: the tiny MLP chain (row statistics, up-projection
with SwiGLU, down-projection with residual and row sums of squares, SwiGLU backward, fp32 weight-gradient accumulation) and
a split-K launch whose ticket counters are re-zeroed by a kernel inside the captured sequence.  Every replay is compared
bit for bit with the eager run of the same calls, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2605_19269_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def test_captured_chain_replays_match_eager():
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2605_19269_amd import coda
    M, d, F = 520, 256, 384
    g = np.random.Generator(np.random.PCG64(99))
    X, Wup = G.dev_bf16(synth.normal_bf16(g, (M, d), 1.0)), G.dev_bf16(synth.normal_bf16(g, (d, 2 * F), 0.06))
    Wdn, R = G.dev_bf16(synth.normal_bf16(g, (F, d), 0.05)), G.dev_bf16(synth.normal_bf16(g, (M, d), 1.0))
    dY = G.dev_bf16(synth.normal_bf16(g, (M, d), 1e-2))
    G0 = G.dev_f32(synth.normal_f32(g, (F, d), 1e-3))
    # split-K case: 4 output tiles, long contraction
    Ms, Ns, Ks = 512, 512, 4096
    As, Bs = G.dev_bf16(synth.normal_bf16(g, (Ms, Ks), 1.0)), G.dev_bf16(synth.normal_bf16(g, (Ks, Ns), 0.02))
    need = coda.coda_gemm_workspace_bytes(Ms, Ns, Ks, [])
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    f32 = dict(dtype=torch.float32, device="cuda")
    b16 = dict(dtype=torch.bfloat16, device="cuda")
    nb_d = coda.coda_row_partial_blocks(d)

    def buffers():
        return dict(ssx=torch.empty(M, **f32), rstd=torch.empty(M, **f32), Z=torch.empty((M, 2 * F), **b16),
                    H=torch.empty((M, F), **b16), Y=torch.empty((M, d), **b16), part=torch.empty((nb_d, M), **f32),
                    ssy=torch.empty(M, **f32), dZ=torch.empty((M, 2 * F), **b16), Gw=G0.clone(), S=torch.empty((Ms, Ns), **b16),
                    ss_at=torch.empty(M, **f32))

    def chain(o):
        coda.coda_row_sumsq(X, o["ssx"])
        coda.coda_row_finalize(o["ssx"].view(1, M), M, 1, rstd_out=o["rstd"], d=d, eps=1e-6)
        coda.coda_gemm(X, Wup, [coda.row_scale(o["rstd"]), coda.swiglu_fwd(o["Z"]), coda.store(o["H"])])
        o["ss_at"].zero_()                                   # a fill kernel, not a memset node
        coda.coda_gemm(o["H"], Wdn, [coda.add_tile(R), coda.row_sumsq(o["part"]), coda.store(o["Y"])])
        coda.coda_row_finalize(o["part"], M, nb_d, sum_out=o["ssy"], d=d, eps=0.0)
        coda.coda_gemm(dY, Wdn, [coda.swiglu_bwd(o["Z"]), coda.store(o["dZ"])], transB=True)
        coda.coda_gemm(o["H"], dY, [coda.accum_f32(o["Gw"])], transA=True)
        coda.coda_gemm(As, Bs, [coda.store(o["S"])], workspace=ws)

    eager = buffers()
    chain(eager)
    torch.cuda.synchronize()

    cap = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain(cap)                                           # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        chain(cap)
    torch.cuda.synchronize()

    for replay in range(3):
        cap["Gw"].copy_(G0)                                  # the accumulate target is read-modify-write: restore it
        for k in ("H", "Y", "dZ", "S", "Z"):
            cap[k].fill_(float("nan"))                       # eager work between the replays; stale results cannot pass
        ws.fill_(0xA5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in eager:
            if k == "ss_at":
                continue
            assert torch.equal(cap[k].view(torch.uint8), eager[k].view(torch.uint8)), "replay %d: %s differs" % (replay, k)
