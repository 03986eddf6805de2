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
        m = re.search(r"gemm_kernel_dlINS_5DlCfg\w+?EEELb([01])ELb([01])ELi(\d)ELb([01])EEEv", name)
        if m:
            out[tuple(int(x) for x in m.groups())] = r          # (A K-contiguous, B K-contiguous, epilogue mode, ragged)
    return out


def test_every_instance_is_there_and_fits_the_compute_unit(kernels):
    g = _gemm(kernels)
    assert len(g) == 4 * 5 * 2, sorted(g)
    f8 = [r for n, r in kernels.items() if "gemm_kernel_dl_f8" in n]
    assert len(f8) == 5 * 2
    for r in list(g.values()) + f8:
        assert r["vgpr"] <= 256 and r["agpr"] == 0          # two waves per SIMD
        assert r["lds"] <= 160 * 1024


def test_spills_stay_out_of_the_step_kernels(kernels):
    g = _gemm(kernels)
    assert g[(1, 0, 1, 0)]["scratch"] == 0                      # up-projection: row scale + SwiGLU
    assert g[(1, 0, 0, 0)]["scratch"] == 0                      # down-projection / QKV: linear programs
    assert g[(0, 0, 3, 0)]["scratch"] == 0                      # weight gradient: fp32 accumulate
    assert g[(1, 1, 2, 0)]["spill"] <= 4                        # SwiGLU backward: four epilogue-only spills
    for key, r in g.items():
        if key[2] == 4 and not key[3]:
            assert r["scratch"] == 0, (key, r)                  # RMSNorm backward, whole tiles: nothing spilled
        # the ragged instances carry both the bounds-checked and the plain epilogue (interior tiles take the plain one)
        limit = 40 if key[3] else 20
        assert r["spill"] <= limit, (key, r)


def test_spills_of_the_8bit_kernels(kernels):
    for name, r in kernels.items():
        m = re.search(r"gemm_kernel_dl_f8INS_5DlCfg\w+?EEELi(\d)ELb([01])EEEv", name)
        if not m:
            continue
        mode, ragged = int(m.group(1)), int(m.group(2))
        assert r["spill"] <= 24, (name, r)
