"""GPU check of the MFMA calibration loops (include/coda_calib.h): their accumulators must equal the matrix
product that the fragment layout of v_mfma_f32_32x32x16_bf16 / v_mfma_f32_16x16x32_bf16 defines, computed here in
fp64 with numpy.
(The loop is measurement infrastructure, not a step of the method, so there is no oracle function for it.)"""
import numpy as np
import pytest
import torch

from paper_2605_19269_amd import synth

pytestmark = pytest.mark.gpu


def bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_mfma_loop_matches_fragment_layout():
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2605_19269_amd import coda
    g = np.random.Generator(np.random.PCG64(7))
    n_blocks, iters = 3, 3
    a_bits = synth.normal_bf16(g, (n_blocks, 4, 512, 8), 1.0)
    b_bits = synth.normal_bf16(g, (n_blocks, 2, 512, 8), 0.5)
    a = torch.from_numpy(a_bits.view(np.int16)).view(torch.bfloat16).cuda()
    b = torch.from_numpy(b_bits.view(np.int16)).view(torch.bfloat16).cuda()
    out = torch.full((8, 8, 16, 64), float("nan"), dtype=torch.float32, device="cuda")
    coda.coda_calib_mfma_loop(a, b, n_blocks, iters, out=out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    af, bfv = bf16_to_f64(a_bits[0]), bf16_to_f64(b_bits[0])          # block 0: [4 or 2][512][8]
    k = np.arange(16)
    for wave in range(8):
        for i in range(4):
            for j in range(2):
                # operand matrices [32][16]: element (r, k) sits in lane r + 32*(k/8), slot k%8 of the wave's fragment
                P = np.stack([bfv[j, wave * 64 + r + 32 * (k // 8), k % 8] for r in range(32)])   # first operand (rows of D)
                Q = np.stack([af[i, wave * 64 + c + 32 * (k // 8), k % 8] for c in range(32)])    # second operand (columns of D)
                D = 2 * iters * (P @ Q.T)
                for e in range(16):
                    for half in range(2):
                        r = 8 * (e // 4) + 4 * half + e % 4
                        np.testing.assert_allclose(got[wave, i * 2 + j, e, half * 32:(half + 1) * 32], D[r, :],
                                                   rtol=1e-5, atol=1e-5)


def test_mfma_loop16_matches_fragment_layout():
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2605_19269_amd import coda
    g = np.random.Generator(np.random.PCG64(8))
    n_blocks, iters = 2, 3
    a_bits = synth.normal_bf16(g, (n_blocks, 4, 512, 8), 1.0)
    b_bits = synth.normal_bf16(g, (n_blocks, 2, 512, 8), 0.5)
    a = torch.from_numpy(a_bits.view(np.int16)).view(torch.bfloat16).cuda()
    b = torch.from_numpy(b_bits.view(np.int16)).view(torch.bfloat16).cuda()
    out = torch.full((8, 8, 4, 64), float("nan"), dtype=torch.float32, device="cuda")
    coda.coda_calib_mfma_loop16(a, b, n_blocks, iters, out=out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    af, bfv = bf16_to_f64(a_bits[0]), bf16_to_f64(b_bits[0])
    k = np.arange(32)
    for wave in range(8):
        for i in range(4):
            for j in range(2):
                # operand matrices [16][32]: element (r, k) sits in lane r + 16*(k/8), slot k%8 of the wave's fragment
                P = np.stack([bfv[j, wave * 64 + r + 16 * (k // 8), k % 8] for r in range(16)])   # first operand (rows of D)
                Q = np.stack([af[i, wave * 64 + c + 16 * (k // 8), k % 8] for c in range(16)])    # second operand (columns of D)
                D = 4 * iters * (P @ Q.T)
                for e in range(4):
                    for q in range(4):
                        np.testing.assert_allclose(got[wave, i * 2 + j, e, q * 16:(q + 1) * 16], D[4 * q + e, :],
                                                   rtol=1e-5, atol=1e-5)


def test_mfma_loop_argument_errors():
    from paper_2605_19269_amd import coda
    a = torch.zeros(4 * 512 * 8, dtype=torch.bfloat16, device="cuda")
    b = torch.zeros(2 * 512 * 8, dtype=torch.bfloat16, device="cuda")
    coda.coda_calib_mfma_loop(a, b, 0, 10)                     # no blocks: nothing launched
    with pytest.raises(ValueError):
        coda.coda_calib_mfma_loop(a, b, 2, 10)                 # buffers hold one block only
    with pytest.raises(RuntimeError):
        coda.coda_calib_mfma_loop(a, b, 1, -1)
    coda.coda_calib_mfma_loop16(a, b, 0, 10)
    with pytest.raises(ValueError):
        coda.coda_calib_mfma_loop16(a, b, 2, 10)
    with pytest.raises(RuntimeError):
        coda.coda_calib_mfma_loop16(a, b, 1, -1)
    torch.cuda.synchronize()
