"""Build libcks.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcks.so")
PROBE_DIR = os.path.join(os.path.dirname(HERE), "bench_probe")
PROBE_LIB = os.path.join(PROBE_DIR, "libcks_probe.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _compile(src: str, lib: str, verbose: bool, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + ["-o", tmp, src]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


def build_lib(verbose: bool = False, tuning: bool = False) -> str:
    """Compile csrc/cks_api.hip (which includes every kernel header) into libcks.so, and the
    benchmark's measurement probes (bench_probe/cks_probe.hip) into bench_probe/libcks_probe.so.
    tuning=True builds the library with -DCKS_TUNING (CKS_TUNE_* environment hooks and the kernel
    variants only they select); the product build has neither."""
    _compile(os.path.join(PROBE_DIR, "cks_probe.hip"), PROBE_LIB, verbose)
    return _compile(os.path.join(CSRC, "cks_api.hip"), LIB, verbose, ["-DCKS_TUNING"] if tuning else [])


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv, tuning="--tuning" in sys.argv))
