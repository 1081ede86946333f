"""Host-side sanitizer runs (CPU only): the oracle's C code, and the library's host layer (argument checks,
planning, work-list arithmetic), each built as an executable with -fsanitize=address,undefined and run over
a grid of geometries.  A heap overrun or undefined arithmetic aborts the executable."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_check")
    build = run(["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=undefined", "-fopenmp", "-Wall", "-Wextra", "-o", exe,
                 os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm"])
    assert build.returncode == 0, build.stdout
    out = run([exe], env=dict(os.environ, OMP_NUM_THREADS="4"))
    assert out.returncode == 0, out.stdout
    assert out.stdout.strip().endswith("geometries ok"), out.stdout


def test_host_layer_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "host_sanitize_check")
    # sanitizers on the host pass only (the device pass is compiled as always)
    build = run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
                 "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=undefined",
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", exe,
                 os.path.join(ROOT, "tests", "host_sanitize_check.cpp"),
                 os.path.join(ROOT, "paper_2306_15951_amd", "csrc", "cks_api.hip")])
    assert build.returncode == 0, build.stdout[-3000:]
    out = run([exe])
    assert out.returncode == 0, out.stdout[-3000:]
    assert out.stdout.strip().endswith("plans ok"), out.stdout[-3000:]
