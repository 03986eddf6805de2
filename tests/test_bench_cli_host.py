"""Host checks of bench.py's command line (no GPU): the single-GPU rule of the measurement contract and the named kernels
that the profiler summaries under profiles/ are made with."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + list(args), capture_output=True, text=True, cwd=ROOT, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_named_kernels_of_the_profiles_exist():
    """Every kernel name that a summary under profiles/ gives in its first column is a name that `bench.py --kernel` knows."""
    src = open(os.path.join(ROOT, "bench.py")).read()
    names = set(re.findall(r'"([a-z0-9_]+)"', src[src.index("SINGLE_KERNELS = ["):src.index("]", src.index("SINGLE_KERNELS = ["))]))
    assert {"llama1b_up", "llama1b_down", "llama1b_bwd_act", "llama1b_bwd_wgt", "copy256"} <= names
    prof = open(os.path.join(ROOT, "profiles", "gemm_epilogue_kernels_per_kernel_counters.md")).read()
    used = set(re.findall(r"^\| ([a-z0-9_]+) \|", prof, flags=re.M)) - {"name"}
    assert used and used <= names, sorted(used - names)
    help_text = _run("--help").stdout
    for n in names:
        assert n in help_text
