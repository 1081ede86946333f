"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, validates arguments before touching the
device, and its geometry helpers agree with the oracle's enumeration."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def cks():
    from paper_2306_15951_amd import binding, build

    if not os.path.exists(binding.LIB_PATH):
        build.build_lib()
    binding.lib()
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cks.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cks_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(cks):
    names = declared_symbols()
    assert len(names) >= 22
    L = ctypes.CDLL(cks.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(cks.EXPORTS) == names          # the binding covers the same set
    for n in names:
        assert hasattr(cks, n) or n in ("cks_strerror", "cks_last_hip_error")


def test_probe_library_exports_its_header(cks):
    """The benchmark's measurement probes (bench_probe/cks_probe.h -> bench_probe/libcks_probe.so)."""
    from paper_2306_15951_amd import build

    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "bench_probe", "cks_probe.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(cks_probe_[a-z0-9_]+)\s*\(", text)))
    assert len(names) == 3
    if not os.path.exists(build.PROBE_LIB):
        build.build_lib()
    L = ctypes.CDLL(build.PROBE_LIB)
    for n in names:
        assert hasattr(L, n), n
    # arguments are checked before anything is launched
    L.cks_probe_mfma_registers.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    assert L.cks_probe_mfma_registers(None, 1, 1, 0, None) == -2
    L.cks_probe_mfma_lds.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 4 + [ctypes.c_void_p]
    assert L.cks_probe_mfma_lds(ctypes.c_void_p(0x1000), 1, 3, 1, 0, None) == -2    # odd chunk count


def test_out_dims_and_shape_errors(cks):
    assert cks.cks_out_dims(224, 224, 7, 7, 2, 3) == (112, 112)
    assert cks.cks_out_dims(7, 4, 3, 3, 1, 1) == (7, 4)
    assert cks.cks_out_dims(8, 8, 3, 3, 2, 0) == (3, 3)
    L = cks.lib()
    assert L.cks_out_dims(2, 2, 5, 5, 1, 1, None, None) == cks.CKS_ERR_SHAPE
    assert L.cks_out_dims(4, 4, 3, 3, 0, 1, None, None) == cks.CKS_ERR_SHAPE
    assert L.cks_out_dims(4, 4, 3, 3, 1, -1, None, None) == cks.CKS_ERR_SHAPE
    with pytest.raises(cks.CksError):
        cks.cks_out_dims(2, 2, 5, 5, 1, 1)


def test_entry_points_reject_bad_arguments_before_any_launch(cks):
    L = cks.lib()
    good = (2, 4, 8, 8, 4, 3, 3, 1, 1)
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every call below must fail in validation
    for fn in (L.cks_conv2d_fwd, L.cks_deconv2d, L.cks_dilated_conv2d_wgrad):
        assert fn(None, fake, fake, *good, None, 0, None) == cks.CKS_ERR_NULL
        assert fn(fake, None, fake, *good, None, 0, None) == cks.CKS_ERR_NULL
        assert fn(fake, fake, None, *good, None, 0, None) == cks.CKS_ERR_NULL
        for bad in ((0, 4, 8, 8, 4, 3, 3, 1, 1), (2, 4, 8, 8, 4, 3, 3, 0, 1), (2, 4, 8, 8, 4, 3, 3, 1, -1),
                    (2, 4, 2, 8, 4, 5, 3, 1, 1), (2, 4, 8, 8, 0, 3, 3, 1, 1),
                    (1 << 16, 1 << 10, 1 << 6, 1 << 6, 4, 3, 3, 1, 1)):      # 2^38 elements
            assert fn(fake, fake, fake, *bad, None, 0, None) == cks.CKS_ERR_SHAPE
    # KS-deconv always needs the split-kernel workspace
    need = L.cks_deconv2d_workspace(*good)
    assert need == cks.cks_kernel_split_bytes(4, 4, 3, 3, 1) == 4 * 4 * 3 * 3 * 4
    assert L.cks_deconv2d(fake, fake, fake, *good, None, 0, None) == cks.CKS_ERR_WORKSPACE
    assert L.cks_deconv2d(fake, fake, fake, *good, fake, need - 1, None) == cks.CKS_ERR_WORKSPACE
    # Sk-dilated needs one slice of dW per segment when the contraction axis is split
    big = (128, 64, 32, 32, 64, 3, 3, 1, 1)
    gz = L.cks_dilated_conv2d_wgrad_segments(*big)
    assert gz > 1
    assert L.cks_dilated_conv2d_wgrad_workspace(*big) == 4 * gz * 64 * 9 * 64
    assert L.cks_dilated_conv2d_wgrad(fake, fake, fake, *big, None, 0, None) == cks.CKS_ERR_WORKSPACE
    assert L.cks_kernel_split(None, fake, 4, 4, 3, 3, 2, None) == cks.CKS_ERR_NULL
    assert L.cks_kernel_split(fake, fake, 4, 4, 3, 3, 0, None) == cks.CKS_ERR_SHAPE
    assert L.cks_filter_transpose(fake, None, 4, 4, 3, 3, None) == cks.CKS_ERR_NULL
    assert L.cks_deconv2d_presplit(fake, fake, None, *good, None) == cks.CKS_ERR_NULL
    assert L.cks_strerror(cks.CKS_ERR_WORKSPACE).decode().startswith("workspace")
    assert L.cks_deconv2d_workspace(2, 4, 2, 8, 4, 5, 3, 1, 1) == 0


def test_split_tensor_size_matches_the_paper_layout(cks):
    # Algorithm 2 Stage 1: s * s * OC * ceil(FH/s) * ceil(FW/s) * IC elements
    assert cks.cks_kernel_split_bytes(3, 5, 7, 7, 2) == 4 * 2 * 2 * 5 * 4 * 4 * 3
    assert cks.cks_kernel_split_bytes(1, 1, 3, 3, 2) == 4 * 16      # Fig. 5: C is 2x2x2x2
    assert cks.cks_kernel_split_bytes(2, 2, 1, 1, 3) == 4 * 9 * 4


def test_useful_macs_agree_with_enumeration(cks, oracle):
    from paper_2306_15951_amd import synth

    for L in synth.LAYERS.values():
        g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding)
        assert cks.cks_useful_macs(*g) == oracle.mac_counts(*g)["useful"], L.name
    for g in [(1, 1, 4, 4, 1, 3, 3, 2, 1), (2, 3, 5, 8, 2, 4, 2, 3, 3), (1, 2, 3, 5, 2, 1, 1, 2, 0), (1, 1, 7, 4, 1, 5, 5, 1, 4)]:
        assert cks.cks_useful_macs(*g) == oracle.mac_counts(*g)["useful"], g
    assert 2 * cks.cks_useful_macs(1, 1, 4, 4, 1, 3, 3, 2, 1) == 50   # the paper's worked example
    assert cks.cks_useful_macs(1, 1, 2, 2, 1, 5, 5, 1, 1) == -1


def test_per_axis_entry_points_on_the_host(cks, oracle):
    """<sh sw>, <ph pw> of Table I: output size, validation and the useful multiply-add count."""
    assert cks.cks_out_dims_hw(9, 12, 3, 5, (2, 3), (1, 2)) == (5, 4)
    assert cks.cks_out_dims_hw(224, 224, 7, 7, (2, 2), (3, 3)) == cks.cks_out_dims(224, 224, 7, 7, 2, 3)
    L = cks.lib()
    assert L.cks_out_dims_hw(4, 4, 3, 3, 1, 0, 1, 1, None, None) == cks.CKS_ERR_SHAPE
    assert L.cks_out_dims_hw(4, 4, 3, 3, 1, 1, 1, -1, None, None) == cks.CKS_ERR_SHAPE
    assert L.cks_out_dims_hw(2, 8, 5, 3, 1, 1, 1, 4, None, None) == cks.CKS_ERR_SHAPE   # rows: 2 + 2 < 5
    assert L.cks_out_dims_hw(8, 2, 3, 5, 1, 1, 4, 1, None, None) == cks.CKS_ERR_SHAPE   # columns
    fake = ctypes.c_void_p(0x1000)
    good = (2, 4, 8, 8, 4, 3, 3, 2, 1, 0, 1)
    for fn in (L.cks_conv2d_fwd_hw, L.cks_deconv2d_hw, L.cks_dilated_conv2d_wgrad_hw):
        assert fn(None, fake, fake, *good, None, 0, None) == cks.CKS_ERR_NULL
        assert fn(fake, fake, fake, 2, 4, 8, 8, 4, 3, 3, 2, 0, 0, 1, None, 0, None) == cks.CKS_ERR_SHAPE
    # the split tensor has sh*sw sub-kernels of ceil(FH/sh) x ceil(FW/sw) taps
    assert L.cks_deconv2d_workspace_hw(*good) == 4 * 2 * 1 * 4 * 2 * 3 * 4
    assert L.cks_deconv2d_hw(fake, fake, fake, *good, None, 0, None) == cks.CKS_ERR_WORKSPACE
    for g in [(1, 1, 4, 4, 1, 3, 3, (2, 1), (1, 0)), (2, 3, 5, 8, 2, 4, 2, (3, 2), (3, 0)), (1, 2, 7, 5, 2, 1, 3, (2, 4), (0, 2)),
              (1, 1, 7, 4, 1, 5, 2, (1, 3), (4, 1))]:
        assert cks.cks_useful_macs_hw(*g) == oracle.mac_counts(*g)["useful"], g
    g = (3, 2, 6, 9, 5, 3, 4, 2, 1)
    assert cks.cks_useful_macs_hw(*g[:7], (2, 2), (1, 1)) == cks.cks_useful_macs(*g)


def test_no_alloc_entry_point_checks_its_limit_on_the_host(cks):
    """cks_dilated_conv2d_wgrad_noalloc_hw refuses, before any device call, a geometry whose partial sums
    exceed the static scratch array."""
    L = cks.lib()
    fake = ctypes.c_void_p(0x1000)
    big = (256, 512, 7, 7, 512, 3, 3, 1, 1, 1, 1)
    assert L.cks_dilated_conv2d_wgrad_workspace_hw(*big) > cks.CKS_STATIC_SCRATCH_BYTES
    assert L.cks_dilated_conv2d_wgrad_noalloc_hw(fake, fake, fake, *big, None) == cks.CKS_ERR_SCRATCH
    assert L.cks_dilated_conv2d_wgrad_noalloc_hw(fake, None, fake, *big, None) == cks.CKS_ERR_NULL
    assert L.cks_dilated_conv2d_wgrad_noalloc_hw(fake, fake, fake, 256, 512, 7, 7, 512, 3, 3, 1, 0, 1, 1, None) == cks.CKS_ERR_SHAPE
    assert b"static" in L.cks_strerror(cks.CKS_ERR_SCRATCH)
    text = open(os.path.join(ROOT, "include", "cks.h")).read()
    assert "#define CKS_STATIC_SCRATCH_BYTES (32u << 20)" in text and cks.CKS_STATIC_SCRATCH_BYTES == 32 << 20


def test_forward_on_the_transposed_filter_refuses_on_the_host(cks):
    """cks_conv2d_fwd_transposed has a kernel for whole 32-channel chunks of C, OC a multiple of 4 and 16-byte
    aligned pointers only; everything else is refused before any device call."""
    L = cks.lib()
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    assert L.cks_conv2d_fwd_transposed(fake, fake, fake, 4, 36, 6, 6, 8, 3, 3, 1, 1, None) == cks.CKS_ERR_UNSUPPORTED   # C = 36
    assert L.cks_conv2d_fwd_transposed(fake, fake, fake, 4, 32, 6, 6, 6, 3, 3, 1, 1, None) == cks.CKS_ERR_UNSUPPORTED   # OC = 6
    assert L.cks_conv2d_fwd_transposed(odd, fake, fake, 4, 32, 6, 6, 8, 3, 3, 1, 1, None) == cks.CKS_ERR_UNSUPPORTED    # X off by a float
    assert L.cks_conv2d_fwd_transposed(None, fake, fake, 4, 32, 6, 6, 8, 3, 3, 1, 1, None) == cks.CKS_ERR_NULL
    assert L.cks_conv2d_fwd_transposed_hw(fake, fake, fake, 4, 32, 6, 6, 8, 3, 3, 0, 1, 1, 1, None) == cks.CKS_ERR_SHAPE
    names = [k for k, _ in cks.cks_plan_hw(cks.CKS_OP_CONV2D_FWD_TRANSPOSED, 128, 64, 32, 32, 64, 3, 3, (1, 1), (1, 1))]
    assert names == ["rowrun_gemm_dma<3, 64, 64, 2, 2, true>"]
