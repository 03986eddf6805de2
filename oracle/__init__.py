"""CPU oracle for the GEMM-plus-epilogue hot path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It holds a plain fp64 C implementation (coda_oracle.c) and a ctypes
wrapper that does argument marshalling only.  Nothing here touches the GPU or
the HIP library.
"""
from .binding import *  # noqa: F401,F403
from .binding import build, lib_path  # noqa: F401
