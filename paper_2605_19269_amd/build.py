"""Build libcoda.so and libcoda_bench.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2605_19269_amd.build [--force]

Each translation unit is compiled to an object under paper_2605_19269_amd/_build/
(in parallel).  libcoda.so is the product: it exports exactly what include/coda.h declares.
libcoda_bench.so holds what only the measurement needs (the unfused baseline kernels of
include/coda_unfused.h and the MFMA-only calibration loops of include/coda_calib.h) and links
nothing of the product.  The ctypes binding loads both.  hipcc cross-compiles for gfx950
without a GPU present.
"""
import concurrent.futures
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcoda.so")
LIB_BENCH = os.path.join(HERE, "libcoda_bench.so")
RESOURCES = os.path.join(HERE, "libcoda.resources.txt")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops is switched off: the compiler must not form packed fp32 VALU ops.
# -fvisibility=hidden: only the entry points marked CODA_API in the headers are exported.
# -Wno-inline-asm: the direct-to-LDS load statement names M0 in its clobber list on purpose (it writes M0); the compiler
# honours the clobber and warns, once per use, that M0 is a reserved register.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         "-fvisibility=hidden", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

SOURCES = ["coda_api.hip", "aux_kernels.hip",
           "gemm_inst_nn.hip", "gemm_inst_nt.hip", "gemm_inst_tn.hip", "gemm_inst_tt.hip",
           "gemm_inst_f8_nn.hip", "gemm_inst_f8_nt.hip", "gemm_inst_f8_tn.hip", "gemm_inst_f8_tt.hip"]
SOURCES_BENCH = ["baseline_kernels.hip", "calib_kernels.hip"]


def _headers():
    return [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))] + \
           [os.path.join(os.path.dirname(HERE), "include", h) for h in ("coda.h", "coda_unfused.h", "coda_calib.h")]


def _compile(src, force):
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(p) for p in [path] + _headers())
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
        return obj, ""
    r = subprocess.run([HIPCC] + FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-c", path, "-o", obj],
                       capture_output=True, text=True)
    text = r.stdout + r.stderr
    with open(obj + ".resources", "w") as f:
        f.write(_resource_table(text))
    log = "\n".join(_strip_remarks(text))
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, log))
    return obj, log


_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|VGPRs Spill|SGPRs Spill|LDS Size \[bytes/block\]): (\S+)")


def _resource_table(text):
    """One line per kernel from the compiler's resource-usage remarks: name vgprs agprs scratch_bytes vgpr_spills lds_bytes."""
    rows, cur = [], None
    for line in text.splitlines():
        m = _REMARK.search(line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            cur = {"name": val}
            rows.append(cur)
        elif cur is not None:
            cur[key] = val
    return "".join("%s %s %s %s %s %s\n" % (k["name"], k.get("VGPRs", "?"), k.get("AGPRs", "?"), k.get("ScratchSize [bytes/lane]", "?"),
                                            k.get("VGPRs Spill", "?"), k.get("LDS Size [bytes/block]", "?")) for k in rows)


def _strip_remarks(text):
    """Compiler output without the resource-usage remarks (each is followed by a source line and a caret line)."""
    out, skip = [], 0
    for line in text.splitlines():
        if skip:
            skip -= 1
            continue
        if "-Rpass-analysis=kernel-resource-usage" in line:
            skip = 2 if "Function Name" in line else 0
            continue
        if "packed-fp32-ops" not in line and "remark generated" not in line and "remarks generated" not in line:
            out.append(line)
    if not any("warning:" in l or "error:" in l for l in out):
        out = [l for l in out if not l.startswith("In file included from")]   # include trails of the dropped remarks
    return out


def _link(lib, objs, force):
    if force or not os.path.exists(lib) or any(os.path.getmtime(o) > os.path.getmtime(lib) for o in objs):
        r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs,
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stdout + r.stderr)


def build(force=False, jobs=None):
    os.makedirs(BUILD, exist_ok=True)
    srcs = SOURCES + SOURCES_BENCH
    jobs = jobs or min(8, len(srcs))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(lambda s: _compile(s, force), srcs))
    objs = [o for o, _ in results]
    for _, log in results:
        if log.strip():
            print(log)
    _link(LIB, objs[:len(SOURCES)], force)
    _link(LIB_BENCH, objs[len(SOURCES):], force)
    # registers, scratch and LDS of every kernel of the two libraries, as the compiler reported them (read by the host tests)
    with open(RESOURCES, "w") as f:
        for o in objs:
            if os.path.exists(o + ".resources"):
                f.write(open(o + ".resources").read())
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
