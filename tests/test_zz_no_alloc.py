"""The entry point that allocates nothing (coda_gemm_static_ws: split-K through the library's static device array) against
coda_gemm with a caller workspace: same results bit for bit, on two calls in a row, the second with a smaller input, so
that whatever the first call left in the array (partials, counters) must not leak into the second."""
import numpy as np
import pytest
import torch

from paper_2605_19269_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _run_pair(coda, oracle, M, N, K, seed, first_call_on_this_gpu=False):
    g = np.random.Generator(np.random.PCG64(seed))
    A = synth.normal_bf16(g, (M, K), 1.0)
    B = synth.normal_bf16(g, (K, N), 0.05)
    C = synth.normal_bf16(g, (M, N), 1.0)
    r = synth.uniform_f32(g, (M,), 0.5, 1.5)
    dA, dB, dC, dr = G.dev_bf16(A), G.dev_bf16(B), G.dev_bf16(C), G.dev_f32(r)
    nblk = coda.coda_row_partial_blocks(N)
    need = coda.coda_gemm_workspace_bytes(M, N, K, [])
    assert 0 < need <= coda.CODA_STATIC_WS_BYTES, "shape must be planned for split-K and fit the static array"

    def program(Y, part):
        return [coda.row_scale(dr), coda.add_tile(dC), coda.row_sumsq(part), coda.store(Y.t)]

    # existing entry point, caller workspace
    ws = torch.empty(need, dtype=torch.uint8, device="cuda").fill_(0xA5)
    Y0 = G.Guarded(M, N, torch.bfloat16)
    p0 = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    coda.coda_gemm(dA, dB, program(Y0, p0), workspace=ws)
    # the entry point under test: no workspace argument, no allocation inside
    Y1 = G.Guarded(M, N, torch.bfloat16)
    p1 = torch.full((nblk, M), G.SENTINEL_F32, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    coda.coda_gemm_static_ws(dA, dB, program(Y1, p1))
    torch.cuda.synchronize()
    if not first_call_on_this_gpu:     # the very first call may load the code object that holds the array
        assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated or freed during the call"
    Y1.check_guards(); Y1.written()
    assert torch.equal(Y0.t.contiguous().view(torch.int16), Y1.t.contiguous().view(torch.int16)), "outputs differ"
    assert torch.equal(p0, p1), "row partials differ"
    refD = oracle.gemm_residual_sumsq(A, B, r=r.astype(np.float64), C=C)[0]
    G.assert_bf16_close(G.host_f64(Y1.t), refD, "static-scratch split-K %dx%dx%d" % (M, N, K))


def test_static_scratch_matches_workspace_on_two_calls_in_a_row(oracle):
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2605_19269_amd import coda
    _run_pair(coda, oracle, 1024, 1024, 4096, seed=4100, first_call_on_this_gpu=True)   # 16 tiles in 4 parts: 16 MiB of partials, 16 counters
    _run_pair(coda, oracle, 504, 264, 4168, seed=4101)     # smaller, ragged in M, N and K: 4 tiles in 3 parts
    torch.cuda.synchronize()


def test_static_scratch_refuses_plans_beyond_its_size():
    from paper_2605_19269_amd import coda
    M = N = 2048
    K = 8192
    assert coda.coda_gemm_workspace_bytes(M, N, K, []) > coda.CODA_STATIC_WS_BYTES
    A = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    B = torch.zeros((K, N), dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    st = coda.coda_gemm_static_ws_raw(None, M, N, K, coda.mat(A), coda.mat(B), [coda.store(Y)])
    assert st == coda.CODA_ERR_WORKSPACE
    torch.cuda.synchronize()
