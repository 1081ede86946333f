"""No kernel without a parity case (CPU only).

Which kernel serves a call is decided on the host from the geometry and the alignment of the pointers.
cks_plan_hw answers that question without a GPU, through the very code path of the entry points.  This test
asks it for every call the GPU parity tests make and compares the answers with the kernels the shipped
library actually contains (the host-side launch stubs in libcks.so name every instantiation): a kernel that
a caller can be given but that no parity case reaches fails the test."""
import os
import re
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
if HERE not in sys.path:
    sys.path.insert(0, HERE)


@pytest.fixture(scope="module")
def cks():
    from paper_2306_15951_amd import binding, build

    if not os.path.exists(binding.LIB_PATH):
        build.build_lib()
    binding.lib()
    return binding


def kernels_in_library(path):
    nm = shutil.which("nm") or "/opt/rocm/llvm/bin/llvm-nm"
    text = subprocess.check_output([nm, "-C", path]).decode()
    names = set(re.findall(r"cks::__device_stub__([^(]+)\(", text))
    return {n.replace(" ", "") for n in names}


def selected_by_parity_cases(cks):
    from paper_2306_15951_amd import synth
    import test_gpu_parity as T

    hit = {}
    for op, geo, mask in T.planned_calls():
        name, N, C, H, W, OC, FH, FW, s, p = geo
        for kernel, _shape in cks.cks_plan_hw(op, N, C, H, W, OC, FH, FW, synth.pair(s), synth.pair(p), mask):
            hit.setdefault(kernel.replace(" ", ""), (op, name, mask))
    return hit


def test_every_kernel_in_the_library_is_reached_by_a_parity_case(cks):
    built = kernels_in_library(cks.LIB_PATH)
    assert len(built) >= 40, built
    hit = selected_by_parity_cases(cks)
    unknown = sorted(set(hit) - built)
    assert not unknown, "the plan names kernels the library does not contain: %s" % unknown
    missing = sorted(built - set(hit))
    assert not missing, "kernels no GPU parity case selects: %s" % missing


def test_plan_of_the_benchmark_layers(cks):
    """The plan is the dispatch itself: spot values for the layers the benchmark times."""
    from paper_2306_15951_amd import synth

    def plan(op, L, mask=0):
        return [k for k, _ in cks.cks_plan_hw(op, L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW,
                                              synth.pair(L.stride), synth.pair(L.padding), mask)]

    L1, L4b = synth.LAYERS["cfg1"], synth.LAYERS["cfg4b"]
    assert plan(cks.CKS_OP_CONV2D_FWD, L1) == ["rowrun_gemm_dma<0, 64, 64, 2, 2, true>"]
    assert plan(cks.CKS_OP_DECONV2D, L1) == ["rowrun_gemm_dma<2, 64, 64, 2, 2, true>"]                 # filter read in place: one launch
    assert plan(cks.CKS_OP_DECONV2D, L1, 2) == ["pack_filter<0>", "rowrun_gemm_dma<1, 64, 64, 2, 2, true>"]  # Wt off by a float: Stage 1 first
    assert plan(cks.CKS_OP_DECONV2D, L1, 1) == ["pack_filter<0>", "rowrun_gemm<1, 64, 64, 2, 2, 0>"]   # dY off by a float: scalar loads
    assert plan(cks.CKS_OP_DILATED_CONV2D_WGRAD, L1) == ["pixel_gemm_dma<true>", "reduce_slices<16, 4>"]
    assert plan(cks.CKS_OP_CONV2D_FWD, L4b) == ["strip_fwd<7, 7, 3, 2>"]
    assert plan(cks.CKS_OP_DECONV2D, L4b) == ["sweep_deconv<7, 7, 2, 3, 3, 4>"]                         # one launch, no workspace
    assert plan(cks.CKS_OP_DECONV2D, L4b._replace(padding=2)) == ["scatter_deconv<10, true>", "add_heads"]   # another padding: the older stem kernel
    assert plan(cks.CKS_OP_DILATED_CONV2D_WGRAD, L4b) == ["strip_wgrad<7, 7, 3, 2, true>", "reduce_slices<16, 4>"]
    # bad geometry and a buffer that is too small are reported, not planned
    L = cks.lib()
    import ctypes
    buf = ctypes.create_string_buffer(8)
    assert L.cks_plan_hw(0, 128, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1, 0, buf, 8) == cks.CKS_ERR_WORKSPACE
    assert L.cks_plan_hw(0, 128, 64, 2, 2, 64, 5, 5, 1, 1, 1, 1, 0, buf, 8) == cks.CKS_ERR_SHAPE
    assert L.cks_plan_hw(99, 128, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1, 0, ctypes.create_string_buffer(256), 256) == cks.CKS_ERR_UNSUPPORTED
    assert L.cks_plan_hw(0, 128, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1, 0, None, 0) == cks.CKS_ERR_NULL
