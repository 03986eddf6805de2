"""Helpers for the GPU parity tests: host<->device marshalling of raw bf16 bits, guarded
output buffers, and the tolerance rules.

Tolerances (from the benchmark spec of this build):
  * bf16 outputs:  |delta| <= 1e-2 + 1e-2*|ref|.  Where outputs are much smaller than 1 the
    absolute term would make that vacuous, so the scale-aware form
    |delta| <= 1e-2*rms(ref) + 1e-2*|ref| is enforced as well.
  * fp32 row reductions of squares (strictly positive): |delta| <= 1e-3*|ref|.
  * fp32 signed reductions / gradients: |delta| <= 1e-3*max(|ref|, rms(ref)) elementwise and
    ||delta||_2 <= 1e-3*||ref||_2.
"""
import numpy as np
import torch

SENTINEL_BF16 = 0x7F7F  # a large finite bf16 (3.39e38) no computation here produces
SENTINEL_F32 = -1.2345e30


def dev_bf16(bits):
    """numpy uint16 bits -> CUDA bf16 tensor with the same bytes."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).copy())
    return t.view(torch.bfloat16).cuda()


def dev_f32(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32).copy()).cuda()


def host_bits(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(bits):
    return (np.ascontiguousarray(bits).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def host_f64(t):
    if t.dtype == torch.bfloat16:
        return bits_to_f64(host_bits(t))
    return t.detach().cpu().numpy().astype(np.float64)


class Guarded:
    """A [rows x cols] output inside a larger sentinel-filled buffer (extra rows above and below,
    pad columns on the right), so out-of-bounds and unwritten elements are caught."""

    def __init__(self, rows, cols, dtype, pad_cols=8, guard_rows=2):
        self.rows, self.cols, self.guard = rows, cols, guard_rows
        ld = (cols + pad_cols + 7) // 8 * 8   # pitches must be multiples of 8 elements
        self.full = torch.empty((rows + 2 * guard_rows, ld), dtype=dtype, device="cuda")
        if dtype == torch.bfloat16:
            self.full.view(torch.int16).fill_(int(np.int16(np.uint16(SENTINEL_BF16).view(np.int16))))
        else:
            self.full.fill_(SENTINEL_F32)
        self.t = self.full[guard_rows:guard_rows + rows, :cols]
        self.ref = self.full.clone()

    def check_guards(self):
        cur, ref = self.full.clone(), self.ref
        cur[self.guard:self.guard + self.rows, :self.cols] = 0
        ref = ref.clone()
        ref[self.guard:self.guard + self.rows, :self.cols] = 0
        same = torch.equal(cur.view(torch.int16) if cur.dtype == torch.bfloat16 else cur.view(torch.int32),
                           ref.view(torch.int16) if ref.dtype == torch.bfloat16 else ref.view(torch.int32))
        assert same, "kernel wrote outside its output region"

    def written(self):
        """Assert that no sentinel survives inside the region."""
        if self.t.dtype == torch.bfloat16:
            left = (self.t.contiguous().view(torch.int16) == int(np.uint16(SENTINEL_BF16).view(np.int16))).sum().item()
        else:
            left = (self.t == SENTINEL_F32).sum().item()
        assert left == 0, "%d output elements were never written" % left


def rms(x):
    x = np.asarray(x, dtype=np.float64)
    return float(np.sqrt(np.mean(x * x))) if x.size else 0.0


def assert_bf16_close(got, ref, what=""):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return
    d = np.abs(got - ref)
    bad1 = d > 1e-2 + 1e-2 * np.abs(ref)
    assert not bad1.any(), "%s: %d elements beyond 1e-2+1e-2|ref| (max delta %.3g)" % (what, bad1.sum(), d.max())
    bad2 = d > 1e-2 * rms(ref) + 1e-2 * np.abs(ref)
    assert not bad2.any(), "%s: %d elements beyond the scale-aware bound (max delta %.3g, rms %.3g)" % (
        what, bad2.sum(), d.max(), rms(ref))


def assert_chain_close(got, ref, what=""):
    """Bound for a result that passed through several bf16 roundings (folded weight, stored
    intermediate activation, final store) against the never-rounded fp64 chain.  Each rounding
    contributes a relative error of at most 2^-8 (rms about 2^-9) per element; through a GEMM
    these add in quadrature to roughly 0.3% of rms(ref) per element, so over 1e5 elements the
    largest deviation sits near 6 sigma = 2% of rms(ref).  Enforced: elementwise
    |delta| <= 3e-2*rms(ref) + 1e-2*|ref| and normwise ||delta|| <= 1e-2*||ref||."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape
    d = np.abs(got - ref)
    bound = 3e-2 * rms(ref) + 1e-2 * np.abs(ref)
    assert (d <= bound).all(), "%s: %d elements beyond the chain bound (max delta %.3g, rms %.3g)" % (
        what, (d > bound).sum(), d.max(), rms(ref))
    assert np.linalg.norm((got - ref).ravel()) <= 1e-2 * np.linalg.norm(ref.ravel()), what + ": normwise"


def assert_sumsq_close(got, ref, what=""):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape
    if ref.size == 0:
        return
    rel = np.abs(got - ref) / np.maximum(np.abs(ref), 1e-300)
    assert rel.max() <= 1e-3, "%s: max relative error %.3g" % (what, rel.max())


def assert_f32_signed_close(got, ref, what=""):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape
    if ref.size == 0:
        return
    d = np.abs(got - ref)
    bound = 1e-3 * np.maximum(np.abs(ref), rms(ref))
    assert (d <= bound).all(), "%s: %d elements beyond 1e-3*max(|ref|, rms) (max delta %.3g)" % (
        what, (d > bound).sum(), d.max())
    nrm = np.linalg.norm(ref.ravel())
    assert np.linalg.norm((got - ref).ravel()) <= 1e-3 * max(nrm, 1e-300), what + ": normwise"
