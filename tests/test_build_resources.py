"""Host check of what the compiler reported for every kernel of libcoda.so (written next to the library by the build):
register budget, LDS size, and register spills.  A spill in a mainloop costs far more than its size suggests, and a
harmless-looking edit of an epilogue can push a 256-register kernel over the edge, so the spill counts are pinned."""
import os
import re

import pytest

from paper_2605_19269_amd import build as B


@pytest.fixture(scope="module")
def kernels():
    if not os.path.exists(B.RESOURCES):
        B.build(force=True)
    rows = {}
    for line in open(B.RESOURCES):
        name, vgpr, agpr, scratch, spill, lds = line.split()
        rows[name] = dict(vgpr=int(vgpr), agpr=int(agpr), scratch=int(scratch), spill=int(spill), lds=int(lds))
    return rows


def _gemm(kernels):
    out = {}
    for name, r in kernels.items():
        m = re.search(r"gemm_kernel_dlINS_5DlCfg\w+?EEELb([01])ELb([01])ELi(\d)ELb([01])ELb([01])EEEv", name)
        if m:
            out[tuple(int(x) for x in m.groups())] = r   # (A K-contiguous, B K-contiguous, epilogue mode, ragged, shared tail)
    return out


def _gemm_f8(kernels):
    out = {}
    for name, r in kernels.items():
        m = re.search(r"gemm_kernel_dl_f8INS_5DlCfg\w+?EEELb([01])ELb([01])ELi(\d)ELb([01])ELb([01])EEEv", name)
        if m:
            out[tuple(int(x) for x in m.groups())] = r   # (A K-contiguous, B K-contiguous, epilogue mode, ragged, shared tail)
    return out


def test_every_instance_is_there_and_fits_the_compute_unit(kernels):
    g, f8 = _gemm(kernels), _gemm_f8(kernels)
    assert len(g) == 4 * 5 * 2 * 2, sorted(g)
    assert len(f8) == 4 * 5 * 2 * 2
    for r in list(g.values()) + list(f8.values()):
        assert r["vgpr"] <= 256 and r["agpr"] == 0          # two waves per SIMD
        assert r["lds"] <= 160 * 1024


def test_whole_tile_kernels_do_not_spill(kernels):
    """The kernels of every launch without shared tiles, on shapes that are whole multiples of the tile: all five epilogue
    modes, all four layouts and the 8-bit kernel run without a single spilled register."""
    for key, r in _gemm(kernels).items():
        if not key[3] and not key[4]:
            assert r["scratch"] == 0 and r["spill"] == 0, (key, r)
    for key, r in _gemm_f8(kernels).items():
        if not key[3] and not key[4]:
            assert r["scratch"] == 0 and r["spill"] == 0, (key, r)


def test_spills_of_the_other_instances_stay_small(kernels):
    """Ragged instances carry both the bounds-checked and the plain epilogue (interior tiles take the plain one); the
    instances for launches with shared tiles carry the exchange of partial tiles as well.  Only the ragged bf16 instances of
    the two pairwise SwiGLU programs (staging of two tile-shaped operands with bounds checks) spill more than a few
    registers; the 8-bit kernels spill nowhere."""
    for key, r in _gemm(kernels).items():
        limit = (40 if key[2] in (1, 2) else 10) if key[3] else 0
        assert r["spill"] <= limit, (key, r)
    for key, r in _gemm_f8(kernels).items():
        assert r["spill"] == 0 and r["scratch"] == 0, (key, r)
