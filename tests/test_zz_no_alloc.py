"""The entry point that allocates nothing (cks_dilated_conv2d_wgrad_noalloc_hw): same bits as the entry point
that takes a workspace, on two calls in a row that share the library's static scratch array, the second
with a smaller input; and the oracle's result on both."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cks():
    import torch
    from paper_2306_15951_amd import binding

    assert torch.cuda.is_available(), "this test needs the MI355X"
    binding.lib()
    return binding


def dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


# first a layer whose partial sums fill half of the static array, then smaller ones (whose segments are
# then a prefix of the array still holding the first call's sums), one of them with stride / padding per axis
CALLS = [
    ("cfg1", 128, 64, 32, 32, 64, 3, 3, (1, 1), (1, 1)),
    ("smaller_s2", 96, 64, 11, 9, 96, 3, 3, (2, 2), (1, 1)),
    ("smaller_per_axis", 33, 20, 11, 9, 20, 3, 5, (3, 1), (0, 2)),
    ("stem_like", 6, 3, 40, 37, 64, 7, 7, (2, 2), (3, 3)),
]


def test_no_alloc_entry_point_equals_the_workspace_one(cks, oracle):
    import torch
    from paper_2306_15951_amd import synth

    for kind in ("int", "normal"):
        for geo in CALLS:
            L = synth.Layer(*geo)
            print("geometry", geo, kind, flush=True)
            g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding)
            need = cks.cks_dilated_conv2d_wgrad_workspace_hw(*g)
            assert 0 < need <= cks.CKS_STATIC_SCRATCH_BYTES
            X, W, dY = synth.make_inputs(L, kind, 60)
            Xd, dYd = dev(X), dev(dY)
            ws = torch.full((need // 4,), float("nan"), device="cuda")
            want = torch.full(W.shape, float("nan"), device="cuda")
            got = torch.full(W.shape, float("nan"), device="cuda")
            cks.cks_dilated_conv2d_wgrad_hw(Xd, dYd, want, L.stride, L.padding, ws)
            cks.cks_dilated_conv2d_wgrad_noalloc_hw(Xd, dYd, got, L.stride, L.padding)
            torch.cuda.synchronize()
            g_h, w_h = got.cpu().numpy(), want.cpu().numpy()
            assert np.array_equal(g_h.view(np.uint32), w_h.view(np.uint32)), "%s %s: differs from cks_dilated_conv2d_wgrad_hw" % (L.name, kind)
            ref = oracle.wgrad(X, dY, L.FH, L.FW, L.stride, L.padding)
            if kind == "int":
                assert np.array_equal(g_h.astype(np.float64), ref), "%s: differs from the oracle" % L.name
            else:
                bound = oracle.wgrad(np.abs(X), np.abs(dY), L.FH, L.FW, L.stride, L.padding)
                assert (np.abs(g_h - ref) <= 1e-5 * bound + 1e-30).all(), "%s: out of tolerance" % L.name


def test_no_alloc_entry_point_rejects_what_does_not_fit(cks):
    import torch

    # 512 -> 512 channels, 3x3: 8 segments of 9.4 MB each
    g = (256, 512, 7, 7, 512, 3, 3, (1, 1), (1, 1))
    assert cks.cks_dilated_conv2d_wgrad_workspace_hw(*g) > cks.CKS_STATIC_SCRATCH_BYTES
    X = torch.zeros((256, 7, 7, 512), device="cuda")
    dW = torch.full((512, 3, 3, 512), 7.0, device="cuda")
    with pytest.raises(cks.CksError) as e:
        cks.cks_dilated_conv2d_wgrad_noalloc_hw(X, X, dW, (1, 1), (1, 1))
    assert e.value.status == cks.CKS_ERR_SCRATCH
    torch.cuda.synchronize()
    assert bool((dW == 7.0).all()), "a rejected call must not enqueue anything"
    L = cks.lib()
    fake = ctypes.c_void_p(0x1000)
    assert L.cks_dilated_conv2d_wgrad_noalloc_hw(None, fake, fake, 2, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, None) == cks.CKS_ERR_NULL
    assert L.cks_dilated_conv2d_wgrad_noalloc_hw(fake, fake, fake, 2, 4, 8, 8, 4, 3, 3, 0, 1, 1, 1, None) == cks.CKS_ERR_SHAPE
