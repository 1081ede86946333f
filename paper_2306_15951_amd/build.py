"""Build libcks.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcks.so")
PROBE_LIB = os.path.join(HERE, "libcks_probe.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _compile(src: str, lib: str, verbose: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", tmp, os.path.join(CSRC, src)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


def build_lib(verbose: bool = False) -> str:
    """Compile csrc/cks_api.hip (which includes every kernel header) into libcks.so, and the
    benchmark's measurement probes (csrc/cks_probe.hip) into libcks_probe.so."""
    _compile("cks_probe.hip", PROBE_LIB, verbose)
    return _compile("cks_api.hip", LIB, verbose)


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
