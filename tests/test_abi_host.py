"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
headers declare, and turns bad arguments into status codes before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def coda():
    from paper_2605_19269_amd import coda as c
    return c


def declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(coda_[a-z0-9_]+)\s*\(", text)))


def exported_symbols(path):
    """Names of the functions a shared object defines and exports (dynamic symbol table)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    return sorted(line.split()[2] for line in out.splitlines() if len(line.split()) == 3 and line.split()[1] in "TW")


def test_libraries_export_exactly_what_the_headers_declare(coda):
    # the product library is the boundary: every declared entry point and nothing else
    got = [n for n in exported_symbols(coda.LIB_PATH) if not n.startswith("__hip")]   # the HIP runtime's registration hooks
    assert got == declared_symbols("coda.h"), "libcoda.so exports differ from include/coda.h"
    assert "coda_gemm" in got and "coda_gemm_static_ws" in got
    # measurement-only entry points live in their own library
    gotb = [n for n in exported_symbols(coda.LIB_BENCH_PATH) if not n.startswith("__hip")]
    assert gotb == sorted(declared_symbols("coda_unfused.h") + declared_symbols("coda_calib.h"))
    lib, blib = ctypes.CDLL(coda.LIB_PATH), ctypes.CDLL(coda.LIB_BENCH_PATH)
    assert all(hasattr(lib, n) for n in got) and all(hasattr(blib, n) for n in gotb)
    assert set(coda.EXPORTS) == set(declared_symbols("coda.h"))
    assert set(coda.EXPORTS_UNFUSED) == set(declared_symbols("coda_unfused.h"))
    assert set(coda.EXPORTS_CALIB) == set(declared_symbols("coda_calib.h"))


def test_binding_mirrors_header_enums(coda):
    text = open(os.path.join(ROOT, "include", "coda.h")).read()
    for name in ["CODA_OK", "CODA_ERR_NULL", "CODA_ERR_SHAPE", "CODA_ERR_ALIGN", "CODA_ERR_DTYPE", "CODA_ERR_PROGRAM",
                 "CODA_ERR_WORKSPACE", "CODA_ERR_LAUNCH", "CODA_EPI_ROW_SCALE", "CODA_EPI_COL_SCALE_SIDE",
                 "CODA_EPI_ADD_TILE", "CODA_EPI_SWIGLU_FWD", "CODA_EPI_SWIGLU_BWD", "CODA_EPI_ROW_SUMSQ",
                 "CODA_EPI_STORE", "CODA_EPI_ACCUM_F32", "CODA_EPI_ROPE", "CODA_EPI_RMSNORM_BWD", "CODA_EPI_LSE_PARTIAL"]:
        m = re.search(r"\b%s\s*=\s*(\d+)" % name, text)
        assert m and int(m.group(1)) == getattr(coda, name), name
    assert ctypes.sizeof(coda.coda_mat) == 40 and ctypes.sizeof(coda.coda_epi_op) == 96


def _mat(coda, ptr, rows, cols, ld=None, trans=0, dtype=0):
    return coda.coda_mat(ptr, rows, cols, ld if ld is not None else cols, trans, dtype)


def _op(coda, kind, flags=0, in_=None, out=None, out2=None, ld_in=0, ld_out=0, in2=None, in3=None, in4=None, out3=None, i0=0, i1=0):
    return coda.coda_epi_op(kind, flags, in_, out, out2, ld_in, ld_out, in2, in3, in4, out3, i0, i1)


P = 0x1000  # a fake, 16-byte aligned "device pointer"; no call below ever reaches a launch


def test_argument_errors_are_status_codes(coda):
    A, B = _mat(coda, P, 64, 32), _mat(coda, P, 32, 64)
    store = _op(coda, coda.CODA_EPI_STORE, out=P, ld_out=64)
    g = lambda M, N, K, a, b, ops: coda.coda_gemm_raw(None, M, N, K, a, b, ops)
    assert g(64, 64, 32, None, B, [store]) == coda.CODA_ERR_NULL
    assert g(64, 64, 32, A, B, []) == coda.CODA_ERR_PROGRAM                       # no final op
    assert g(64, 64, 40, A, B, [store]) == coda.CODA_ERR_SHAPE                    # K mismatch
    assert g(-1, 64, 32, A, B, [store]) == coda.CODA_ERR_SHAPE
    assert g(64, 64, 32, _mat(coda, P + 2, 64, 32), B, [store]) == coda.CODA_ERR_ALIGN
    assert g(64, 64, 32, _mat(coda, P, 64, 32, ld=36), B, [store]) == coda.CODA_ERR_ALIGN
    assert g(64, 64, 32, _mat(coda, P, 64, 32, ld=24), B, [store]) == coda.CODA_ERR_SHAPE
    assert g(64, 64, 32, _mat(coda, P, 64, 32, dtype=1), B, [store]) == coda.CODA_ERR_DTYPE
    assert g(64, 60, 32, A, _mat(coda, P, 32, 60, ld=64), [store]) == coda.CODA_ERR_SHAPE   # N % 8
    assert g(64, 64, 32, A, B, [_op(coda, coda.CODA_EPI_STORE, out=None, ld_out=64)]) == coda.CODA_ERR_NULL
    assert g(64, 64, 32, A, B, [_op(coda, coda.CODA_EPI_STORE, out=P, ld_out=32)]) == coda.CODA_ERR_SHAPE
    # 8-bit operands (dtype 2): any layout; 16-byte chunks along K and along whichever output index is contiguous
    A8, B8 = _mat(coda, P, 64, 32, dtype=2), _mat(coda, P, 64, 32, trans=1, dtype=2)
    assert g(64, 64, 32, A8, _mat(coda, P, 64, 32, trans=1), [store]) == coda.CODA_ERR_DTYPE          # mixed
    assert g(0, 64, 32, _mat(coda, P, 0, 32, dtype=2), _mat(coda, P, 32, 64, dtype=2), [store]) == coda.CODA_OK   # N-contiguous B
    assert g(64, 72, 32, A8, _mat(coda, P, 32, 72, ld=80, dtype=2), [_op(coda, coda.CODA_EPI_STORE, out=P, ld_out=72)]) == coda.CODA_ERR_SHAPE   # N % 16
    assert g(72, 64, 32, _mat(coda, P, 32, 72, ld=80, trans=1, dtype=2), B8, [store]) == coda.CODA_ERR_SHAPE      # A^T: M % 16
    assert g(64, 64, 24, _mat(coda, P, 64, 24, ld=32, dtype=2), _mat(coda, P, 64, 24, ld=32, trans=1, dtype=2), [store]) == coda.CODA_ERR_SHAPE
    assert g(0, 64, 32, _mat(coda, P, 0, 32, dtype=2), B8, [store]) == coda.CODA_OK
    # row pitches beyond 2^22 elements are refused (32-bit lane offsets in the kernels)
    assert g(64, 64, 32, _mat(coda, P, 64, 32, ld=(1 << 22) + 8), B, [store]) == coda.CODA_ERR_SHAPE
    assert g(64, 64, 32, A, B, [_op(coda, coda.CODA_EPI_STORE, out=P, ld_out=(1 << 22) + 8)]) == coda.CODA_ERR_SHAPE
    # transposed operands are described as stored ([K x M]); M == 0 so nothing is launched
    assert g(0, 64, 32, _mat(coda, P, 32, 0, ld=8, trans=1), B, [store]) == coda.CODA_OK
    assert g(0, 64, 32, _mat(coda, P, 0, 32, ld=32, trans=1), B, [store]) == coda.CODA_ERR_SHAPE


def test_program_grammar(coda):
    A, B = _mat(coda, P, 0, 32), _mat(coda, P, 32, 64)      # M == 0: validates, launches nothing
    g = lambda ops: coda.coda_gemm_raw(None, 0, 64, 32, A, B, ops)
    rs = _op(coda, coda.CODA_EPI_ROW_SCALE, in_=P)
    add = _op(coda, coda.CODA_EPI_ADD_TILE, in_=P, ld_in=64)
    ssq = _op(coda, coda.CODA_EPI_ROW_SUMSQ, out=P)
    side = _op(coda, coda.CODA_EPI_COL_SCALE_SIDE, in_=P, out=P, ld_out=64)
    st = _op(coda, coda.CODA_EPI_STORE, out=P, ld_out=64)
    st_half = _op(coda, coda.CODA_EPI_STORE, out=P, ld_out=32)
    st_dbl = _op(coda, coda.CODA_EPI_STORE, out=P, ld_out=128)
    fwd = _op(coda, coda.CODA_EPI_SWIGLU_FWD)
    bwd = _op(coda, coda.CODA_EPI_SWIGLU_BWD, in_=P, ld_in=128)
    acc = _op(coda, coda.CODA_EPI_ACCUM_F32, out=P, ld_out=64)
    OK, BAD = coda.CODA_OK, coda.CODA_ERR_PROGRAM
    assert g([st]) == OK
    assert g([rs, st]) == OK
    assert g([rs, add, ssq, side, st]) == OK
    assert g([add, ssq, st]) == OK
    assert g([rs, fwd, st_half]) == OK
    assert g([fwd, st_half]) == OK
    assert g([bwd, st_dbl]) == OK
    assert g([acc]) == OK
    assert g([add, rs, st]) == BAD            # row scale after the residual add: not the supported order
    assert g([ssq, add, st]) == BAD
    assert g([st, rs]) == BAD                 # nothing may follow the final op
    assert g([rs, rs, st]) == BAD
    assert g([add, fwd, st_half]) == BAD
    assert g([rs, bwd, st_dbl]) == BAD
    assert g([rs, acc]) == BAD
    assert g([fwd]) == BAD                    # pairwise op without a store
    assert g([_op(coda, 99), st]) == BAD
    assert g([fwd, _op(coda, coda.CODA_EPI_STORE, flags=coda.CODA_STORE_F32, out=P, ld_out=32)]) == BAD
    assert g([bwd, st]) == coda.CODA_ERR_SHAPE     # store narrower than the widened output
    assert g([_op(coda, coda.CODA_EPI_ROW_SUMSQ, flags=7, out=P), st]) == BAD
    rope = _op(coda, coda.CODA_EPI_ROPE, in_=P, in2=P, in3=P, ld_in=128, i0=16, i1=32)
    assert g([rope, st]) == OK and g([rs, rope, st]) == OK
    assert g([rope, add, st]) == BAD and g([add, rope, st]) == BAD and g([rope, fwd, st_half]) == BAD
    assert g([rope, side, st]) == BAD and g([rope, rs, st]) == BAD
    lse = _op(coda, coda.CODA_EPI_LSE_PARTIAL, in3=P, out=P, out2=P, out3=P)
    assert g([lse, st]) == OK and g([rs, lse, st]) == OK
    assert g([lse, add, st]) == BAD and g([lse, fwd, st_half]) == BAD and g([lse]) == BAD
    assert g([_op(coda, coda.CODA_EPI_LSE_PARTIAL, in3=P, out=P, out2=None, out3=P), st]) == coda.CODA_ERR_NULL
    rnb = _op(coda, coda.CODA_EPI_RMSNORM_BWD, in_=P, ld_in=64, in2=P, in3=P, in4=P, out=P, ld_out=64, out2=P)
    assert g([rnb, st]) == OK and g([rnb, add, st]) == OK
    assert g([rs, rnb, st]) == BAD and g([rnb, ssq, st]) == BAD and g([rnb, rope, st]) == BAD and g([rnb, fwd, st_half]) == BAD
    assert g([rnb, _op(coda, coda.CODA_EPI_STORE, flags=coda.CODA_STORE_F32, out=P, ld_out=64)]) == BAD
    assert g([_op(coda, coda.CODA_EPI_RMSNORM_BWD, in_=P, ld_in=64, in2=P, in3=None, in4=P), st]) == coda.CODA_ERR_NULL
    assert g([_op(coda, coda.CODA_EPI_ROPE, in_=P, in2=P, in3=P, ld_in=128, i0=12, i1=32), st]) == coda.CODA_ERR_SHAPE
    assert g([_op(coda, coda.CODA_EPI_ROPE, in_=P, in2=P, in3=P, ld_in=128, i0=16, i1=72), st]) == coda.CODA_ERR_SHAPE
    assert g([_op(coda, coda.CODA_EPI_ROPE, in_=P, in2=None, in3=P, ld_in=128, i0=16, i1=32), st]) == coda.CODA_ERR_NULL


def test_aux_argument_errors(coda):
    import ctypes as C
    lib = C.CDLL(coda.LIB_PATH)
    lib.coda_row_finalize.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_float]
    assert lib.coda_row_finalize(None, P, 8, 2, None, None, 8, 0.0) == coda.CODA_ERR_NULL
    assert lib.coda_row_finalize(None, P, 8, 2, P, None, 0, 0.0) == coda.CODA_ERR_SHAPE
    assert lib.coda_row_finalize(None, P, 0, 2, P, None, 8, 0.0) == coda.CODA_OK
    assert coda.coda_row_partial_blocks(0) == 0 and coda.coda_row_partial_blocks(1) == 1
    assert coda.coda_row_partial_blocks(2048) * 256 >= 2048
    assert coda.coda_gemm_workspace_bytes(8, 8, 8, []) == 0
    assert coda.coda_status_string(coda.CODA_ERR_PROGRAM) == "unsupported epilogue program"


def test_splitk_workspace_planning_and_errors(coda):
    """Host logic only: which shapes are planned for split-K, how much workspace they ask for, and the status codes
    of a workspace that is too small or misaligned (returned before anything is launched)."""
    wb = lambda M, N, K: coda.coda_gemm_workspace_bytes(M, N, K, [])
    tile = 256 * 256 * 4
    assert wb(512, 512, 4096) == 1024 + 4 * 4 * tile        # 4 tiles, K / 1024 = 4 parts
    assert wb(256, 256, 8192) == 1024 + 1 * 8 * tile        # 1 tile, capped at 8 parts
    assert wb(2048, 2048, 8192) == 1024 + 64 * 4 * tile     # 64 tiles: 4 parts fill the 256 compute units
    assert wb(2048, 2048 + 256, 8192) == 1024 + 72 * 5 * tile   # 72 tiles: 256 ranges of 9/32 of a tile, up to 5 reach into one tile
    assert wb(512, 512, 1024) == 0                          # contraction too short to split
    assert wb(512, 512, 4096 + 32) == 1024 + 4 * 4 * tile   # 130 K-steps (ragged K rounds up to pairs): parts of 32 or 34
    assert wb(504, 264, 4096) == 1024 + 4 * 4 * tile        # ragged M and N: 2 x 2 tiles, shared like whole ones
    assert wb(256, 256, 6 * 1024 + 128) == 1024 + 1 * 6 * tile  # 196 K-steps: six parts of 32 or 34
    # more than 256 tiles: only a partly filled last round is shared, and only when it pays
    assert wb(5120, 4096, 4096) == 1024 + 64 * 4 * tile     # 320 tiles: the last 64 shared by 4 workgroups each
    assert wb(6144, 4096, 8192) == 1024 + 128 * 2 * tile    # 384 tiles: the last 128 shared by 2
    assert wb(6144, 4096, 4096) == 1024 + 128 * 2 * tile    # the same with K = 4096: each workgroup is spared 64 K-steps
    assert wb(6144, 4096, 2048) == 0                        # ... with K = 2048 only 32: not worth the exchange
    assert wb(5120, 4096, 2048) == 0                        # contraction too short
    assert wb(2560, 1024, 8192) == 1024 + 40 * 8 * tile     # 40 tiles x 8 parts exceed the chip: 256 ranges that straddle tiles, up to 8 per tile
    assert wb(2304, 4096, 8192) == 0                        # one round of 144 tiles: more than half full, measured to lose
    assert wb(7168, 4096, 8192) == 0                        # 448 tiles: the last round is three quarters full (measured: a loss)
    assert wb(8192, 4096, 4096) == 0                        # 512 tiles: whole rounds
    assert wb(0, 512, 4096) == 0 and wb(-1, 512, 4096) == 0
    A, B = _mat(coda, P, 512, 4096), _mat(coda, P, 4096, 512)
    store = _op(coda, coda.CODA_EPI_STORE, out=P, ld_out=512)
    need = wb(512, 512, 4096)
    assert coda.coda_gemm_raw(None, 512, 512, 4096, A, B, [store], P, need - 1) == coda.CODA_ERR_WORKSPACE
    assert coda.coda_gemm_raw(None, 512, 512, 4096, A, B, [store], P + 4, need) == coda.CODA_ERR_ALIGN


def test_epilogue_op_keeps_its_tensors_alive():
    """An op built from a temporary tensor must keep that tensor's memory from being recycled before the launch."""
    import weakref
    import torch
    from paper_2605_19269_amd import coda
    t = torch.zeros(8)
    ref = weakref.ref(t)
    op = coda.row_scale(t)
    del t
    assert ref() is not None and op.in_ == ref().data_ptr()
    del op
    assert ref() is None


def test_static_scratch_entry_refuses_oversized_plans_before_touching_the_gpu(coda):
    # 2048 x 2048 x 8192: 64 tiles in 4 parts = 64 MiB of partials, beyond the 32 MiB static array; the size check needs no GPU
    M = N = 2048
    K = 8192
    assert coda.coda_gemm_workspace_bytes(M, N, K, []) > coda.CODA_STATIC_WS_BYTES
    A, B = _mat(coda, P, M, K), _mat(coda, P, K, N)
    store = _op(coda, coda.CODA_EPI_STORE, out=P, ld_out=N)
    assert coda.coda_gemm_static_ws_raw(None, M, N, K, A, B, [store]) == coda.CODA_ERR_WORKSPACE
    assert coda.coda_gemm_static_ws_raw(None, M, N, K, None, B, [store]) == coda.CODA_ERR_NULL
    text = open(os.path.join(ROOT, "include", "coda.h")).read()
    m = re.search(r"#define CODA_STATIC_WS_BYTES \(\(size_t\)(\d+) \* 1024 \* 1024 \+ (\d+)\)", text)
    assert m and int(m.group(1)) * 1024 * 1024 + int(m.group(2)) == coda.CODA_STATIC_WS_BYTES
