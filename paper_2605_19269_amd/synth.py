"""Seeded synthetic inputs for the GEMM-plus-epilogue workloads.

This module only draws random tensors in the shapes, dtypes and value
distributions of the LLaMA-style workloads and rounds them to the storage
format; it contains none of the method's arithmetic.  Both the GPU library's
tests/benchmark and the CPU oracle read the very same bytes produced here.

bf16 tensors are numpy uint16 arrays holding raw bits (round-to-nearest-even from
the fp32 draw); fp32 tensors are float32 arrays.  The second parameter of a
normal draw is always the standard deviation.
"""
import numpy as np


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16, returned as raw uint16 bits (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def normal_bf16(rng, shape, std):
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(std))


def f32_to_f8e4m3_bits(x):
    """Round-to-nearest-even fp32 -> OCP E4M3 bytes (uint8), saturating at +-448 (finite inputs).  Storage rounding of
    synthetic inputs only: 8-bit operands are an input format of the GEMM, not part of its arithmetic."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    a = np.abs(x)
    # normal range (|x| >= 2^-6): round the 23-bit mantissa to 3 bits on the raw bits, then re-bias the exponent (127 -> 7)
    u = a.view(np.uint32)
    r = u + np.uint32(0x7FFFF) + ((u >> np.uint32(20)) & np.uint32(1))
    code = (r >> np.uint32(20)).astype(np.int32) - np.int32((127 - 7) << 3)
    # subnormal range: multiples of 2^-9; a value that rounds up to 8 * 2^-9 is the smallest normal, code 0x08
    sub = np.rint(a * np.float32(512.0)).astype(np.int32)
    code = np.where(a < np.float32(2.0 ** -6), sub, code)
    code = np.minimum(code, 0x7E).astype(np.uint8)
    return code | (np.signbit(x).astype(np.uint8) << np.uint8(7))


def normal_f8e4m3(rng, shape, std):
    return f32_to_f8e4m3_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(std))


def normal_f32(rng, shape, std):
    return rng.standard_normal(shape, dtype=np.float32) * np.float32(std)


def uniform_f32(rng, shape, lo, hi):
    return (rng.random(shape, dtype=np.float32) * np.float32(hi - lo) + np.float32(lo)).astype(np.float32)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def tiny_rmsnorm_gemm(seed=0, M=256, K=256, N=512):
    """Tiny fused RMSNorm-GEMM: X ~N(0,1), gamma ~U(0.5,1.5), W ~N(0,1/16), R ~N(0,1)."""
    g = _rng(seed)
    return {
        "X": normal_bf16(g, (M, K), 1.0),
        "gamma": uniform_f32(g, (K,), 0.5, 1.5),
        "W": normal_bf16(g, (K, N), 1.0 / 16.0),
        "R": normal_bf16(g, (M, N), 1.0),
        "eps": 1e-6,
    }


def up_projection(seed=0, M=8192, K=2048, N=16384, w_std=0.02):
    """MLP up-projection: X ~N(0,1) [M x K]; W [K x N] ~N(0,w_std), gate/up interleaved in pairs.

    The interleaved weight is drawn directly (an interleave of two i.i.d. draws is
    an i.i.d. draw).  rstd is not produced here: it is the method's own quantity.
    """
    g = _rng(seed)
    return {"X": normal_bf16(g, (M, K), 1.0), "W": normal_bf16(g, (K, N), w_std)}


def down_projection(seed=0, M=8192, K=8192, N=2048, w_std=0.02):
    """MLP down-projection: H ~N(0,1) [M x K]; W_down [K x N] ~N(0,w_std); residual R ~N(0,1)."""
    g = _rng(seed)
    return {
        "H": normal_bf16(g, (M, K), 1.0),
        "W": normal_bf16(g, (K, N), w_std),
        "R": normal_bf16(g, (M, N), 1.0),
    }


def mlp_backward(seed=0, M=8192, F=8192, d=2048, w_std=0.02):
    """MLP backward: dY ~N(0,1e-2) [M x d]; W_down [F x d]; saved pre-activation Z ~N(0,1)
    [M x 2F]; H ~N(0,1) [M x F]; existing fp32 gradient buffer ~N(0,1e-3) [F x d]."""
    g = _rng(seed)
    return {
        "dY": normal_bf16(g, (M, d), 1e-2),
        "W": normal_bf16(g, (F, d), w_std),
        "Z": normal_bf16(g, (M, 2 * F), 1.0),
        "H": normal_bf16(g, (M, F), 1.0),
        "G": normal_f32(g, (F, d), 1e-3),
    }


def block_8b(seed=0, M=16384, d=4096, F=14336, n_qkv=6144, w_std=0.02):
    """LLaMA-3-8B-style non-attention chain: X [M x d]; W_qkv [d x n_qkv] (gamma already folded);
    W_up [d x 2F] interleaved; H [M x F]; W_down [F x d]; R [M x d]."""
    g = _rng(seed)
    return {
        "X": normal_bf16(g, (M, d), 1.0),
        "Wqkv": normal_bf16(g, (d, n_qkv), w_std),
        "Wup": normal_bf16(g, (d, 2 * F), w_std),
        "H": normal_bf16(g, (M, F), 1.0),
        "Wdown": normal_bf16(g, (F, d), w_std),
        "R": normal_bf16(g, (M, d), 1.0),
    }


def rope_tables(T, head_dim, base=10000.0):
    """fp32 cos / sin tables [T x head_dim/2] for angles t * base^(-2f/head_dim) (input data for the RoPE
    epilogue; the method itself only consumes the tables)."""
    f = np.arange(head_dim // 2, dtype=np.float64)
    ang = np.arange(T, dtype=np.float64)[:, None] * (base ** (-2.0 * f / head_dim))[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def qkv_projection(seed=0, M=16384, K=4096, N=6144, w_std=0.02, seq_len=2048):
    """Fused QKV projection input: X ~N(0,1) [M x K], W [K x N] ~N(0,w_std) (gamma folded), and the token
    positions of M rows laid out as consecutive sequences of seq_len tokens."""
    g = _rng(seed)
    return {"X": normal_bf16(g, (M, K), 1.0), "W": normal_bf16(g, (K, N), w_std),
            "pos": (np.arange(M) % seq_len).astype(np.int32)}


def sample_rows(M, n, seed=0):
    """Deterministic row sample: tile-boundary rows plus a seeded draw, sorted and unique."""
    fixed = [r for r in (0, 1, 31, 32, 127, 128, 255, 256, M - 2, M - 1) if 0 <= r < M]
    g = _rng(seed)
    extra = g.choice(M, size=min(M, max(0, n - len(fixed))), replace=False).tolist()
    rows = sorted(set(fixed + extra))
    return np.asarray(rows, dtype=np.int64)


def sample_rows_per_tile(M, per_tile, seed=0, tile=256):
    """Deterministic row sample that reaches every row tile: the tile-boundary rows of sample_rows plus `per_tile`
    seeded rows inside each block of `tile` consecutive rows, sorted and unique."""
    fixed = [r for r in (0, 1, 31, 32, 127, 128, 255, 256, M - 2, M - 1) if 0 <= r < M]
    g = _rng(seed)
    extra = []
    for t0 in range(0, M, tile):
        n = min(tile, M - t0)
        extra += (t0 + g.choice(n, size=min(n, per_tile), replace=False)).tolist()
    return np.asarray(sorted(set(fixed + extra)), dtype=np.int64)
