"""GPU parity: every operator, through the C ABI, element by element against
the CPU oracle on the same seeded inputs.

Bars: bit-exact on small-integer inputs (all partial sums are exact in fp32);
otherwise |gpu - oracle| <= 1e-5 * sum(|x||w|) per output element, the sum
being the oracle applied to the absolute values of the same inputs.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def cks():
    import torch
    from paper_2306_15951_amd import binding

    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    return binding


def dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def nan_like(shape):
    import torch

    return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")


def run_three(cks, L, X, W, dY):
    """All three operators of layer L through the ABI.  Outputs start as NaN so
    an element the kernels forget to write cannot pass.  A layer whose stride or
    padding is a pair goes through the per-axis entry points."""
    import torch
    from paper_2306_15951_amd import synth

    hw = isinstance(L.stride, tuple) or isinstance(L.padding, tuple)
    st, pd = (synth.pair(L.stride), synth.pair(L.padding)) if hw else (L.stride, L.padding)
    f = (lambda name: getattr(cks, name + "_hw")) if hw else (lambda name: getattr(cks, name))
    g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, st, pd)
    OH, OW = f("cks_out_dims")(L.IH, L.IW, L.FH, L.FW, st, pd)
    Xd, Wd, dYd = dev(X), dev(W), dev(dY)
    Y = nan_like((L.N, OH, OW, L.OC))
    dX = nan_like((L.N, L.IH, L.IW, L.IC))
    dW = nan_like((L.OC, L.FH, L.FW, L.IC))
    ws1 = torch.full((max(f("cks_deconv2d_workspace")(*g) // 4, 1),), float("nan"), device="cuda")
    ws2 = torch.full((max(f("cks_dilated_conv2d_wgrad_workspace")(*g) // 4, 1),), float("nan"), device="cuda")
    f("cks_conv2d_fwd")(Xd, Wd, Y, st, pd)
    f("cks_deconv2d")(dYd, Wd, dX, st, pd, ws1)
    f("cks_dilated_conv2d_wgrad")(Xd, dYd, dW, st, pd, ws2)
    torch.cuda.synchronize()
    return Y.cpu().numpy(), dX.cpu().numpy(), dW.cpu().numpy()


def oracle_three(oracle, L, X, W, dY, samples=None):
    s = samples or (None, None, None)
    return (oracle.conv_fwd(X, W, L.stride, L.padding, sample=s[0]),
            oracle.deconv(dY, W, L.IH, L.IW, L.stride, L.padding, sample=s[1]),
            oracle.wgrad(X, dY, L.FH, L.FW, L.stride, L.padding, sample=s[2]))


def assert_exact(got, want, what):
    """Bitwise: same value and no negative zero."""
    want32 = want.astype(np.float32)
    assert np.array_equal(want32.astype(np.float64), want), "oracle value not representable: " + what
    bad = got.view(np.uint32) != (want32 + np.float32(0)).view(np.uint32)
    assert not bad.any(), "%s: %d of %d elements differ, first at %s" % (
        what, bad.sum(), bad.size, np.argwhere(bad)[:3].tolist())


def assert_close(got, want, bound, what):
    err = np.abs(got.astype(np.float64) - want)
    lim = TOL * bound + 1e-30
    bad = ~(err <= lim)      # also catches NaN
    assert not bad.any(), "%s: %d of %d elements out of tolerance, worst err/bound %.3g" % (
        what, bad.sum(), bad.size, np.nanmax(err / np.maximum(bound, 1e-30)))


def check_layer(cks, oracle, L, seed=0, kinds=("int", "normal"), samples=None):
    from paper_2306_15951_amd import synth

    for kind in kinds:
        X, W, dY = synth.make_inputs(L, kind, seed)
        got = run_three(cks, L, X, W, dY)
        if samples is not None:
            got = tuple(g.ravel()[s] for g, s in zip(got, samples))
        want = oracle_three(oracle, L, X, W, dY, samples)
        names = ["%s %s %s" % (L.name, kind, op) for op in ("conv2d_fwd", "deconv2d", "dilated_conv2d_wgrad")]
        if kind == "int":
            for g, w, nm in zip(got, want, names):
                assert_exact(g, w, nm)
        else:
            bound = oracle_three(oracle, L, np.abs(X), np.abs(W), np.abs(dY), samples)
            for g, w, b, nm in zip(got, want, bound, names):
                assert_close(g, w, b, nm)


def test_config0_uniform_and_integer(cks, oracle):
    from paper_2306_15951_amd import synth

    check_layer(cks, oracle, synth.LAYERS["cfg0"], kinds=("int", "uniform", "normal"))


# (name, N, IC, IH, IW, OC, FH, FW, stride, padding): several tiles and ragged
# tails in every GEMM dimension, both load paths (channel counts that are and
# are not multiples of 4), non-square maps and filters, strides 1-3, padding
# from 0 to beyond the filter, stride larger than the filter, remainder rows.
MID = [
    ("tiles_ragged", 150, 36, 9, 10, 72, 3, 3, 1, 1),
    ("wide_channels", 70, 136, 6, 5, 200, 3, 3, 1, 1),
    ("stride2_3x3", 130, 40, 11, 12, 68, 3, 3, 2, 1),
    ("stride2_4x4", 66, 24, 10, 10, 36, 4, 4, 2, 1),
    ("stride3_5x4", 40, 8, 13, 11, 12, 5, 4, 3, 2),
    ("odd_channels", 33, 5, 9, 7, 7, 3, 3, 1, 1),
    ("stem_like", 20, 3, 30, 28, 16, 7, 7, 2, 3),
    ("odd_channels_s2", 9, 6, 8, 9, 10, 2, 3, 2, 0),
    ("pad_ge_filter", 12, 4, 5, 6, 8, 2, 2, 1, 3),
    ("stride_gt_filter", 10, 8, 9, 9, 4, 1, 1, 2, 0),
    ("stride_gt_filter_p", 10, 4, 7, 8, 4, 2, 2, 3, 1),
    ("one_by_one", 200, 48, 5, 5, 96, 1, 1, 1, 0),
    ("remainder_rows", 16, 12, 8, 9, 20, 3, 3, 2, 0),
    ("single_image", 1, 16, 12, 12, 16, 3, 3, 1, 1),
    ("filter_covers_map", 8, 4, 3, 3, 4, 5, 5, 1, 2),
    ("small_map_big_batch", 300, 20, 4, 4, 24, 3, 3, 1, 1),
    # few input channels: the filter gradient puts the whole filter patch in one tile
    ("patch_ic16", 40, 16, 9, 10, 70, 3, 3, 1, 1),
    ("patch_ic32_s2", 24, 32, 11, 9, 40, 3, 3, 2, 1),
    ("patch_ic5_5x5", 12, 5, 12, 13, 33, 5, 5, 2, 2),
    ("patch_ic60", 16, 60, 8, 8, 64, 3, 3, 1, 1),
    ("patch_ic3_pad_ge_filter", 6, 3, 6, 7, 8, 7, 7, 3, 7),
    ("gray_1ch", 5, 1, 10, 11, 70, 3, 3, 1, 1),
    ("ic7_5x5", 3, 7, 9, 9, 65, 5, 5, 1, 2),
    # image stems: 7x7/s2 on 3 channels has kernels of its own (input strip in LDS; input gradient with 64 output
    # channels: on the 4x4x1 matrix instruction with padding 3, tap-stationary GEMM + LDS composing otherwise),
    # other few-channel layers take the generic variants of those
    ("stem_oc64_ragged", 3, 3, 40, 37, 64, 7, 7, 2, 3),
    ("stem_oc70", 2, 3, 23, 50, 70, 7, 7, 2, 3),
    ("stem_pad0", 2, 3, 21, 33, 8, 7, 7, 2, 0),
    ("stem_pad5_tiny", 3, 3, 7, 9, 12, 7, 7, 2, 5),
    ("stem_remainder_rows", 2, 3, 32, 31, 64, 7, 7, 2, 3),
    ("stem_single_pixel_rows", 1, 3, 9, 130, 64, 7, 7, 2, 3),
    # sweep_deconv: waves with runs of two or three rows that start and end inside images and run on into the next
    # window (2176 rows of 34 windows on 1024 waves); a line of columns that ends inside a window; one column per image
    ("stem_runs_across_windows", 32, 3, 128, 128, 64, 7, 7, 2, 3),
    ("stem_one_column_images", 70, 3, 16, 2, 64, 7, 7, 2, 3),
    ("stem_tiny_image", 1, 3, 1, 1, 64, 7, 7, 2, 3),
    # the stem input gradient's check-free output steps start and end by padding and image height; with
    # padding 0 and width 38 the last band's row has three floats that no pixel reaches
    ("stem_oc64_pad0_unreached_columns", 2, 3, 75, 38, 64, 7, 7, 2, 0),
    ("stem_oc64_pad6", 2, 3, 44, 45, 64, 7, 7, 2, 6),
    ("stem_oc64_pad9_tall", 1, 3, 61, 26, 64, 7, 7, 2, 9),
    ("stem_oc64_pad20", 1, 3, 40, 20, 64, 7, 7, 2, 20),
    ("rgb_3x3", 6, 3, 20, 21, 16, 3, 3, 1, 1),
    ("rgb_5x5_s2", 4, 3, 19, 40, 32, 5, 5, 2, 2),
    ("rgb_4x4_s3", 3, 3, 17, 35, 8, 4, 4, 3, 1),
    ("rgb_wide", 2, 3, 9, 70, 4, 3, 3, 1, 1),
    ("two_ch_6x6_s2", 3, 2, 15, 18, 60, 6, 6, 2, 2),
    # OC a multiple of 32: the input gradient reads its sub-kernels from the filter in place
    ("inplace_s2", 70, 36, 11, 12, 96, 3, 3, 2, 1),
    ("inplace_s3_5x4", 33, 20, 13, 11, 32, 5, 4, 3, 2),
    ("inplace_c_ragged", 40, 100, 7, 7, 160, 3, 3, 1, 1),
    ("inplace_stride_gt_filter", 10, 8, 9, 9, 32, 1, 1, 2, 0),
    ("inplace_4x4_s2_remainder", 9, 12, 10, 9, 64, 4, 4, 2, 1),
    # the kernels that load their chunks straight into LDS (64x64 tiles, whole 32-float chunks, 16-byte aligned;
    # filter gradient: batch a multiple of 32): one, two and odd numbers of chunks, ragged batch and channel
    # tiles, strided classes reading the filter in place
    ("lds_direct_1x1_one_chunk", 70, 32, 5, 6, 64, 1, 1, 1, 0),
    ("lds_direct_1x1_two_chunks_oc96", 64, 64, 5, 6, 96, 1, 1, 1, 0),
    ("lds_direct_s2_classes", 96, 64, 11, 9, 96, 3, 3, 2, 1),
    ("lds_direct_ragged_columns", 33, 68, 7, 7, 64, 3, 3, 1, 1),
    ("lds_direct_s3_5x4", 32, 32, 13, 11, 128, 5, 4, 3, 2),
    ("lds_direct_narrow_output", 130, 32, 9, 9, 40, 3, 3, 1, 1),
    # many positions and a last, partial round of bands that is dealt to the dies in pieces (row-major
    # list with bands of a row; class-major list of the stride-2 input gradient)
    ("lds_direct_partial_round", 64, 64, 12, 13, 64, 3, 3, 1, 1),
    ("lds_direct_partial_round_s2", 64, 64, 25, 23, 64, 3, 3, 2, 1),
    # more bands than compute units: the input gradient's workgroups take runs of sweep steps that
    # start and end inside bands, and the rows two runs share are added afterwards
    ("stem_row_heads", 37, 3, 24, 224, 64, 7, 7, 2, 3),
    ("rgb7_row_heads_oc16", 37, 3, 27, 230, 16, 7, 7, 2, 3),
    ("rgb3_row_heads", 40, 3, 12, 112, 8, 3, 3, 1, 1),
    # the filter gradient's whole-patch tiles with 5, 10 and 18 column blocks in batch-innermost order
    # (batch a multiple of the chunk, channel counts multiples of 4, 16-byte aligned tensors)
    ("patch_fast_5_blocks", 64, 16, 9, 10, 64, 3, 3, 1, 1),
    ("patch_fast_10_blocks_s2", 32, 32, 11, 9, 40, 3, 3, 2, 1),
    ("patch_fast_18_blocks_4x4", 32, 32, 16, 15, 64, 4, 4, 1, 2),
    # ... and in pixel order with channel counts that rule out 16-byte loads on either operand
    ("patch_10_blocks_scalar_both", 10, 25, 9, 10, 7, 3, 3, 1, 1),
    ("patch_10_blocks_scalar_dY", 10, 28, 9, 10, 7, 3, 3, 1, 1),
    ("patch_10_blocks_scalar_X", 10, 25, 9, 10, 8, 3, 3, 1, 1),
    ("patch_18_blocks_scalar_both", 9, 27, 8, 9, 7, 4, 4, 1, 2),
    ("patch_18_blocks_scalar_dY", 9, 28, 8, 9, 7, 4, 4, 1, 2),
    ("patch_18_blocks_scalar_X", 9, 27, 8, 9, 8, 4, 4, 2, 1),
    # forward with 64 output columns per tile and an input channel count that rules out 16-byte loads
    ("fwd_scalar_loads_wide", 20, 9, 7, 8, 50, 3, 3, 1, 1),
    # input gradient through Stage 1 + Stage 2&3 on the split filter with whole 32-channel chunks of OC,
    # loaded straight into LDS (C not a multiple of 4 rules out reading the filter in place)
    ("split_lds_direct_c50", 70, 50, 9, 8, 64, 3, 3, 2, 1),
    ("split_lds_direct_c50_s1", 33, 50, 6, 7, 96, 3, 3, 1, 1),
    # 3x3 / stride 2 on three channels: strip kernels of their own
    ("rgb_3x3_s2", 5, 3, 21, 22, 16, 3, 3, 2, 1),
    ("rgb_3x3_s2_oc6", 4, 3, 19, 40, 6, 3, 3, 2, 1),
]


@pytest.mark.parametrize("geo", MID, ids=[g[0] for g in MID])
def test_midsize_geometries(cks, oracle, geo):
    from paper_2306_15951_amd import synth

    print("geometry", geo, flush=True)
    check_layer(cks, oracle, synth.Layer(*geo), seed=100 + [g[0] for g in MID].index(geo[0]))


def random_geometries(count, seed):
    """Valid layer geometries drawn at random (fixed seed): small enough for the full oracle, biased
    towards the channel counts and filters that select the specialised kernels."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        C = int(rng.choice([1, 2, 3, 3, 3, 4, 5, 8, 12, 16, 20, 32, 36, 64, 96]))
        OC = int(rng.choice([1, 3, 4, 8, 16, 20, 32, 32, 64, 64, 70, 96, 128]))
        FH, FW = (int(rng.choice([1, 2, 3, 3, 3, 4, 5, 7, 7])) for _ in range(2))
        if rng.random() < 0.6:
            FW = FH
        s = int(rng.choice([1, 1, 2, 2, 3]))
        p = int(rng.integers(0, max(FH, FW) + 1))
        H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        if C <= 3 and rng.random() < 0.5:
            W = int(rng.integers(40, 260))        # several bands of the few-channel kernels
        N = int(rng.choice([1, 2, 3, 5, 16, 33, 64, 70]))
        if H + 2 * p < FH or W + 2 * p < FW:
            continue
        OH, OW = (H + 2 * p - FH) // s + 1, (W + 2 * p - FW) // s + 1
        macs = N * OH * OW * OC * FH * FW * C
        if macs > 3e8 or N * H * W * C > 4e6 or N * OH * OW * OC > 4e6:
            continue
        out.append(("rand%02d" % len(out), N, C, H, W, OC, FH, FW, s, p))
    return out


RANDOM = random_geometries(48, 20230615)


@pytest.mark.parametrize("geo", RANDOM, ids=[g[0] for g in RANDOM])
def test_random_geometries(cks, oracle, geo):
    from paper_2306_15951_amd import synth

    print("geometry", geo, flush=True)
    check_layer(cks, oracle, synth.Layer(*geo), seed=500 + int(geo[0][4:]), kinds=("int",))


# Stride and padding that differ between the axes (Table I: <sh sw>, <ph pw>), through the *_hw entry
# points: every general kernel and load path, and few-channel layers (which must not take the kernels
# built for equal strides).
ASYM = [
    ("asym_fast_loads", 70, 32, 9, 12, 64, 3, 3, (1, 2), (1, 0)),
    ("asym_in_place_s23", 64, 36, 13, 11, 96, 4, 5, (2, 3), (1, 2)),
    ("asym_split_s31", 33, 20, 11, 9, 20, 3, 5, (3, 1), (0, 2)),
    ("asym_scalar_loads", 17, 5, 9, 10, 7, 3, 2, (2, 1), (2, 0)),
    ("asym_wide_pixel_fast", 32, 64, 8, 10, 72, 3, 3, (2, 1), (0, 1)),
    ("asym_stride_gt_filter", 10, 8, 9, 9, 32, 1, 2, (2, 3), (0, 1)),
    ("asym_pad_ge_filter", 12, 4, 5, 6, 8, 2, 3, (1, 2), (3, 1)),
    ("asym_patch_ic16", 32, 16, 9, 10, 70, 3, 3, (1, 2), (0, 1)),
    ("asym_patch_ic12_pixel_order", 9, 12, 11, 9, 40, 3, 3, (2, 1), (1, 1)),
    ("asym_rgb_7x7_pad", 3, 3, 30, 41, 64, 7, 7, (2, 2), (3, 2)),
    ("asym_rgb_3x3", 5, 3, 20, 70, 16, 3, 3, (1, 2), (1, 1)),
    # the 7x7/s2 stem input gradient on the 4x4x1 matrix instruction takes any padding above and below (3 left and right)
    ("asym_stem_sweep_ph1", 5, 3, 30, 41, 64, 7, 7, (2, 2), (1, 3)),
    ("asym_stem_sweep_ph5_tall", 2, 3, 67, 26, 64, 7, 7, (2, 2), (5, 3)),
    ("asym_stem_sweep_ph0_remainder", 3, 3, 38, 39, 64, 7, 7, (2, 2), (0, 3)),
    ("asym_gray", 4, 1, 12, 13, 70, 5, 3, (3, 2), (2, 0)),
    ("asym_remainder_rows", 16, 12, 8, 9, 32, 3, 3, (2, 3), (0, 0)),
    ("asym_one_by_one", 40, 48, 5, 6, 96, 1, 1, (2, 1), (0, 0)),
    ("asym_tall_filter", 6, 8, 14, 5, 16, 7, 1, (3, 1), (3, 0)),
]


@pytest.mark.parametrize("geo", ASYM, ids=[g[0] for g in ASYM])
def test_per_axis_stride_and_padding(cks, oracle, geo):
    from paper_2306_15951_amd import synth

    print("geometry", geo, flush=True)
    check_layer(cks, oracle, synth.Layer(*geo), seed=700 + [g[0] for g in ASYM].index(geo[0]))


def random_asymmetric_geometries(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        C = int(rng.choice([1, 3, 4, 5, 8, 16, 20, 32, 36, 64]))
        OC = int(rng.choice([1, 4, 8, 20, 32, 64, 70, 96]))
        FH, FW = (int(rng.choice([1, 2, 3, 3, 4, 5, 7])) for _ in range(2))
        st = (int(rng.choice([1, 2, 3, 4])), int(rng.choice([1, 2, 3, 4])))
        pd = (int(rng.integers(0, FH + 1)), int(rng.integers(0, FW + 1)))
        if st[0] == st[1] and pd[0] == pd[1]:
            continue
        H, W = int(rng.integers(1, 33)), int(rng.integers(1, 33))
        N = int(rng.choice([1, 2, 5, 16, 32, 33, 64, 70]))
        if H + 2 * pd[0] < FH or W + 2 * pd[1] < FW:
            continue
        OH, OW = (H + 2 * pd[0] - FH) // st[0] + 1, (W + 2 * pd[1] - FW) // st[1] + 1
        if N * OH * OW * OC * FH * FW * C > 3e8:
            continue
        out.append(("arand%02d" % len(out), N, C, H, W, OC, FH, FW, st, pd))
    return out


RANDOM_ASYM = random_asymmetric_geometries(32, 20230616)


@pytest.mark.parametrize("geo", RANDOM_ASYM, ids=[g[0] for g in RANDOM_ASYM])
def test_random_per_axis_geometries(cks, oracle, geo):
    from paper_2306_15951_amd import synth

    print("geometry", geo, flush=True)
    check_layer(cks, oracle, synth.Layer(*geo), seed=900 + int(geo[0][5:]), kinds=("int",))


def random_stem_geometries(count, seed):
    """7x7 / stride 2 / 3 -> 64 channels with padding 3 left and right: the layers sweep_deconv serves, any height,
    width, batch and vertical padding."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        N, H, W, ph = int(rng.integers(1, 9)), int(rng.integers(1, 90)), int(rng.integers(1, 150)), int(rng.integers(0, 7))
        if H + 2 * ph < 7:
            continue
        out.append(("srand%02d" % len(out), N, 3, H, W, 64, 7, 7, (2, 2), (ph, 3)))
    return out


RANDOM_STEM = random_stem_geometries(16, 20230617)


@pytest.mark.parametrize("geo", RANDOM_STEM, ids=[g[0] for g in RANDOM_STEM])
def test_random_stem_geometries(cks, oracle, geo):
    from paper_2306_15951_amd import synth

    print("geometry", geo, flush=True)
    assert [k for k, _ in cks.cks_plan_hw(cks.CKS_OP_DECONV2D, *geo[1:])] == ["sweep_deconv<7, 7, 2, 3, 3, 4>"]
    check_layer(cks, oracle, synth.Layer(*geo), seed=1300 + int(geo[0][5:]), kinds=("int",))


def structured_samples(shape, rng, n_random):
    """Random flat indices plus the corners / borders of every axis."""
    idx = [rng.integers(0, int(np.prod(shape)), size=n_random)]
    edges = [sorted({0, 1, d // 2, d - 2, d - 1} & set(range(d))) for d in shape]
    grid = np.stack(np.meshgrid(*edges, indexing="ij"), -1).reshape(-1, len(shape))
    idx.append(np.ravel_multi_index(grid.T, shape))
    return np.unique(np.concatenate(idx))


# The filter gradient's 128x64 tile: at least 96 output channels, between 128 and 1024 tiles of 64x64 and
# 8192 pixels to contract, where 64x64 tiles would come to between 4 and 8 workgroups per compute unit (or
# cannot load straight into LDS).  Batch-innermost order (batch a multiple of 16) and pixel order with every
# combination of 16-byte / 4-byte loads.  Too large for the full oracle: sampled outputs.
WIDE_TILE = [
    ("wide_tile_sweep_shape", 64, 256, 16, 16, 256, 3, 3, 1, 1),
    ("wide_tile_batch48_5x5", 48, 132, 14, 14, 96, 5, 5, 1, 2),
    ("wide_tile_pixel_order", 33, 132, 16, 16, 96, 5, 5, 1, 2),
    ("wide_tile_scalar_dY", 33, 132, 16, 16, 98, 5, 5, 1, 2),
    ("wide_tile_scalar_X", 33, 130, 16, 16, 96, 5, 5, 1, 2),
    ("wide_tile_scalar_both", 33, 130, 16, 16, 98, 5, 5, 1, 2),
]


@pytest.mark.parametrize("geo", WIDE_TILE, ids=[g[0] for g in WIDE_TILE])
def test_wide_filter_gradient_tile_sampled(cks, oracle, geo):
    from paper_2306_15951_amd import synth

    L = synth.Layer(*geo)
    print("geometry", geo, flush=True)
    g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, (L.stride,) * 2, (L.padding,) * 2)
    names = [k for k, _ in cks.cks_plan_hw(cks.CKS_OP_DILATED_CONV2D_WGRAD, *g)]
    assert names[0].startswith(("pixel_gemm<128, 64,", "pixel_gemm_fast<128, 64,")), names   # the case must not fall to another tile
    xs, ws, ys = synth.shapes(L)
    rng = np.random.default_rng(23)
    samples = (structured_samples(ys, rng, 3000), structured_samples(xs, rng, 3000), structured_samples(ws, rng, 3000))
    check_layer(cks, oracle, L, seed=300 + [g[0] for g in WIDE_TILE].index(geo[0]), samples=samples)


FULL = ["cfg1", "cfg2", "cfg3a", "cfg3b", "cfg4a", "cfg4b"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_configs_sampled(cks, oracle, name):
    """The benchmark layers at full size, in the launch configuration the
    benchmark times.  The oracle evaluates a sample of output elements (random
    ones plus the borders of every axis) one by one."""
    from paper_2306_15951_amd import synth

    L = synth.LAYERS[name]
    print("layer", L, flush=True)
    xs, ws, ys = synth.shapes(L)
    rng = np.random.default_rng(17)
    samples = (structured_samples(ys, rng, 20000), structured_samples(xs, rng, 20000),
               structured_samples(ws, rng, 600))
    check_layer(cks, oracle, L, samples=samples)


def test_tensors_beyond_2GiB_sampled(cks, oracle):
    """X and dX of 2.4 GB: element offsets no longer fit 31 bits of bytes, so the kernels take
    their 64-bit addressing paths (no scalar-offset buffer loads); sampled outputs against the oracle."""
    from paper_2306_15951_amd import synth

    L = synth.Layer("beyond_2GiB", 9, 64, 1024, 1024, 16, 3, 3, 1, 1)
    assert L.N * L.IH * L.IW * L.IC * 4 > 2 ** 31
    print("layer", L, flush=True)
    rng = np.random.default_rng(77)
    shapes = ((L.N, L.IH, L.IW, L.OC), (L.N, L.IH, L.IW, L.IC), (L.OC, L.FH, L.FW, L.IC))
    samples = tuple(structured_samples(sh, rng, 1500) for sh in shapes)
    check_layer(cks, oracle, L, seed=9, kinds=("normal",), samples=samples)


@pytest.mark.parametrize("name", ["cfg2", "cfg3a", "cfg3b", "cfg4a", "cfg4b"])
def test_full_size_layers_every_element(cks, oracle, name):
    """The other benchmark layers compared in full (every output element of all three operators, integer
    inputs, bit for bit): the stride-2 layer with its four sub-kernel classes, the two 512-channel layers (the
    4x4 maps' trimmed taps are 31 % of the filter), the 4x4-filter upsampler and the 224x224 stem."""
    from paper_2306_15951_amd import synth

    L = synth.LAYERS[name]
    print("layer", L, flush=True)
    X, W, dY = synth.make_inputs(L, "int", 6)
    Y, dX, dW = run_three(cks, L, X, W, dY)
    assert_exact(Y, oracle.conv_fwd(X, W, L.stride, L.padding), name + " fwd full")
    assert_exact(dX, oracle.deconv(dY, W, L.IH, L.IW, L.stride, L.padding), name + " deconv full")
    assert_exact(dW, oracle.wgrad(X, dY, L.FH, L.FW, L.stride, L.padding), name + " wgrad full")


def test_full_size_cfg1_every_element(cks, oracle):
    """One benchmark layer compared in full, not sampled: all three operators, and the input gradient
    once more in the mode with the filter operations done before the loop (Stage 1, then Stage 2&3 on
    the split filter), and the forward pass once more on the transposed filter."""
    import torch
    from paper_2306_15951_amd import synth

    L = synth.LAYERS["cfg1"]
    X, W, dY = synth.make_inputs(L, "int", 3)
    Y, dX, dW = run_three(cks, L, X, W, dY)
    want_dX = oracle.deconv(dY, W, L.IH, L.IW, L.stride, L.padding)
    assert_exact(Y, oracle.conv_fwd(X, W, L.stride, L.padding), "cfg1 fwd full")
    assert_exact(dX, want_dX, "cfg1 deconv full")
    assert_exact(dW, oracle.wgrad(X, dY, L.FH, L.FW, L.stride, L.padding), "cfg1 wgrad full")
    Cs = nan_like((1, 1, L.IC, L.FH, L.FW, L.OC))
    dX2 = nan_like(X.shape)
    cks.cks_kernel_split(dev(W), Cs, 1)
    cks.cks_deconv2d_presplit(dev(dY), Cs, dX2, L.FH, L.FW, L.stride, L.padding)
    Wtt = nan_like((L.FH, L.FW, L.IC, L.OC))
    Y2 = nan_like(dY.shape)
    cks.cks_filter_transpose(dev(W), Wtt)
    cks.cks_conv2d_fwd_transposed(dev(X), Wtt, Y2, L.stride, L.padding)
    torch.cuda.synchronize()
    assert_exact(dX2.cpu().numpy(), want_dX, "cfg1 deconv on the pre-split filter, full")
    assert_exact(Y2.cpu().numpy(), oracle.conv_fwd(X, W, L.stride, L.padding), "cfg1 fwd on the transposed filter, full")


STAGE1 = [(40, 3, 3, 36, 2), (7, 7, 7, 3, 2), (33, 4, 4, 65, 2), (8, 5, 3, 12, 3), (16, 3, 3, 16, 1), (4, 1, 1, 4, 2)]   # OC, FH, FW, IC, stride


def test_stage_entry_points(cks, oracle):
    """Stage 1 (kernel split) and the filter transposition against the oracle's
    data-movement definitions."""
    import torch

    rng = np.random.default_rng(5)
    for (OC, FH, FW, IC, s) in STAGE1:
        W = rng.standard_normal((OC, FH, FW, IC)).astype(np.float32)
        Wd = dev(W)
        Cs = nan_like((s, s, IC, -(-FH // s), -(-FW // s), OC))
        cks.cks_kernel_split(Wd, Cs, s)
        Wt = nan_like((FH, FW, IC, OC))
        cks.cks_filter_transpose(Wd, Wt)
        torch.cuda.synchronize()
        # the library keeps the paper's 6-D tensor with the two channel axes exchanged
        want = np.transpose(oracle.kernel_split(W, s), (0, 1, 5, 3, 4, 2))
        assert np.array_equal(Cs.cpu().numpy().view(np.uint32), want.view(np.uint32)), (OC, FH, FW, IC, s)
        assert np.array_equal(Wt.cpu().numpy(), oracle.filter_transpose(W))


# Stage 1 once, Stage 2&3 on the split filter (Section V.A: the filter operations before the loop), with one
# stride for both axes and per axis: scalar, 16-byte, whole-chunk and LDS-direct loads, narrow and wide tiles
PRESPLIT = [
    ("presplit_vec", 40, 12, 9, 8, 20, 3, 3, 2, 1),
    ("presplit_scalar", 17, 5, 9, 10, 7, 3, 2, 2, 0),
    ("presplit_lds_direct_wide", 70, 64, 11, 12, 96, 3, 3, 2, 1),
    ("presplit_lds_direct_narrow", 130, 24, 10, 9, 64, 4, 4, 2, 1),
    ("presplit_hw_s23", 64, 36, 13, 11, 96, 4, 5, (2, 3), (1, 2)),
    ("presplit_hw_s31_scalar", 33, 21, 11, 9, 20, 3, 5, (3, 1), (0, 2)),
    ("presplit_hw_lds_direct", 66, 52, 9, 12, 64, 3, 3, (1, 2), (1, 0)),
]


@pytest.mark.parametrize("geo", PRESPLIT, ids=[g[0] for g in PRESPLIT])
def test_presplit_mode(cks, oracle, geo):
    import torch
    from paper_2306_15951_amd import synth

    L = synth.Layer(*geo)
    print("geometry", geo, flush=True)
    hw = isinstance(L.stride, tuple)
    (sh, sw), pd = synth.pair(L.stride), synth.pair(L.padding)
    for kind in ("int", "normal"):
        X, W, dY = synth.make_inputs(L, kind, 40)
        Cs = nan_like((sh, sw, L.IC, -(-L.FH // sh), -(-L.FW // sw), L.OC))
        assert Cs.numel() * 4 == (cks.cks_kernel_split_bytes_hw(L.IC, L.OC, L.FH, L.FW, (sh, sw)) if hw
                                  else cks.cks_kernel_split_bytes(L.IC, L.OC, L.FH, L.FW, sh))
        dX = nan_like(X.shape)
        if hw:
            cks.cks_kernel_split_hw(dev(W), Cs, (sh, sw))
            cks.cks_deconv2d_presplit_hw(dev(dY), Cs, dX, L.FH, L.FW, (sh, sw), pd)
        else:
            cks.cks_kernel_split(dev(W), Cs, sh)
            cks.cks_deconv2d_presplit(dev(dY), Cs, dX, L.FH, L.FW, sh, pd[0])
        torch.cuda.synchronize()
        want = oracle.deconv(dY, W, L.IH, L.IW, L.stride, L.padding)
        if kind == "int":
            want_Cs = np.transpose(oracle.kernel_split(W, L.stride), (0, 1, 5, 3, 4, 2))
            assert np.array_equal(Cs.cpu().numpy().view(np.uint32), want_Cs.view(np.uint32)), "Stage 1"
            assert_exact(dX.cpu().numpy(), want, L.name + " int")
        else:
            bound = oracle.deconv(np.abs(dY), np.abs(W), L.IH, L.IW, L.stride, L.padding)
            assert_close(dX.cpu().numpy(), want, bound, L.name + " normal")


# ConvV2 on the transposed filter (Section IV.A: filter transposition before the convolution): 64-column tiles
# loaded straight into LDS, narrow outputs on the 128x32 tile, ragged batch / channel tiles, strides, per-axis
# geometry, padding beyond the filter, one tap
FWD_TRANSPOSED = [
    ("fwdt_s1", 70, 64, 7, 8, 100, 3, 3, 1, 1),
    ("fwdt_s2_two_chunks", 96, 64, 11, 9, 96, 3, 3, 2, 1),
    ("fwdt_narrow_output", 130, 32, 9, 9, 40, 3, 3, 1, 1),
    ("fwdt_5x4_s3", 33, 32, 13, 11, 128, 5, 4, 3, 2),
    ("fwdt_pad_ge_filter", 12, 32, 5, 6, 8, 2, 2, 1, 3),
    ("fwdt_one_by_one", 200, 96, 5, 5, 68, 1, 1, 1, 0),
    ("fwdt_per_axis", 64, 32, 9, 12, 64, 3, 3, (1, 2), (1, 0)),
    ("fwdt_per_axis_narrow", 40, 64, 13, 11, 20, 4, 5, (2, 3), (1, 2)),
]


@pytest.mark.parametrize("geo", FWD_TRANSPOSED, ids=[g[0] for g in FWD_TRANSPOSED])
def test_forward_on_the_transposed_filter(cks, oracle, geo):
    import torch
    from paper_2306_15951_amd import synth

    L = synth.Layer(*geo)
    print("geometry", geo, flush=True)
    hw = isinstance(L.stride, tuple)
    for kind in ("int", "normal"):
        X, W, _ = synth.make_inputs(L, kind, 55)
        Wtt = nan_like((L.FH, L.FW, L.IC, L.OC))
        cks.cks_filter_transpose(dev(W), Wtt)
        OH, OW = synth.out_hw(L)
        Y = nan_like((L.N, OH, OW, L.OC))
        if hw:
            cks.cks_conv2d_fwd_transposed_hw(dev(X), Wtt, Y, synth.pair(L.stride), synth.pair(L.padding))
        else:
            cks.cks_conv2d_fwd_transposed(dev(X), Wtt, Y, L.stride, L.padding)
        torch.cuda.synchronize()
        want = oracle.conv_fwd(X, W, L.stride, L.padding)
        if kind == "int":
            assert_exact(Y.cpu().numpy(), want, L.name + " int")
        else:
            assert_close(Y.cpu().numpy(), want, oracle.conv_fwd(np.abs(X), np.abs(W), L.stride, L.padding), L.name + " normal")


def test_forward_on_the_transposed_filter_says_what_it_cannot_do(cks):
    import torch

    X = torch.zeros((4, 6, 6, 36), device="cuda")          # 36 input channels: no whole 32-channel chunks
    Wtt = torch.zeros((3, 3, 36, 8), device="cuda")
    Y = torch.full((4, 6, 6, 8), 7.0, device="cuda")
    with pytest.raises(cks.CksError) as e:
        cks.cks_conv2d_fwd_transposed(X, Wtt, Y, 1, 1)
    assert e.value.status == cks.CKS_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())


# Plain convolution, KS-deconv (Algorithm 2) and Sk-dilated (Algorithm 3) -- trimming off, kernel split and
# leaping access kept -- as the ablation of bench.py runs them: the same entry points on tensors whose zero
# border is written out.  Must equal the oracle like the trimmed operators do.
UNTRIMMED = [
    ("untrimmed_s1", 40, 36, 7, 6, 64, 3, 3, 1, 1),
    ("untrimmed_s2_4x4", 33, 24, 10, 9, 32, 4, 4, 2, 1),
    ("untrimmed_s3_pad", 20, 8, 11, 13, 12, 5, 4, 3, 2),
    ("untrimmed_s2_remainder_pad0", 16, 12, 8, 9, 20, 3, 3, 2, 0),
    ("untrimmed_pad_ge_filter", 12, 4, 5, 6, 8, 2, 2, 1, 3),
    ("untrimmed_per_axis", 17, 20, 9, 12, 32, 3, 5, (2, 1), (1, 2)),
]


@pytest.mark.parametrize("geo", UNTRIMMED, ids=[g[0] for g in UNTRIMMED])
def test_untrimmed_algorithms_through_the_same_kernels(cks, oracle, geo):
    import torch
    from paper_2306_15951_amd import synth, untrimmed

    L = synth.Layer(*geo)
    print("geometry", geo, flush=True)
    X, W, dY = synth.make_inputs(L, "int", 77)
    Y, dX, dW = nan_like(dY.shape), nan_like(X.shape), nan_like(W.shape)
    for call in (untrimmed.prepare_conv2d_fwd(cks, dev(X), dev(W), Y, L.stride, L.padding),
                 untrimmed.prepare_deconv2d(cks, dev(dY), dev(W), dX, L.stride, L.padding),
                 untrimmed.prepare_dilated_conv2d_wgrad(cks, dev(X), dev(dY), dW, L.stride, L.padding)):
        call()
    torch.cuda.synchronize()
    want = oracle_three(oracle, L, X, W, dY)
    for got, w, nm in zip((Y, dX, dW), want, ("conv", "KS-deconv", "Sk-dilated")):
        assert_exact(got.cpu().numpy(), w, "%s untrimmed %s" % (L.name, nm))


# The same three algorithms as kernel variants with the trimming compiled out (the library's *_untrimmed entry
# points): whole windows, the cells outside the data fetched as zeros by the loads themselves.  They exist for
# 32-multiple channel counts only (and, for the filter gradient, a batch that is a multiple of 32).
TRIM_OFF = [
    ("trimoff_s1", 64, 64, 7, 6, 64, 3, 3, 1, 1),
    ("trimoff_s2_4x4", 96, 64, 10, 9, 96, 4, 4, 2, 1),
    ("trimoff_s3_pad_ragged_batch", 40, 64, 11, 13, 64, 5, 4, 3, 2),
    ("trimoff_s2_remainder_pad0", 32, 96, 8, 9, 64, 3, 3, 2, 0),
    ("trimoff_pad_ge_filter", 32, 64, 5, 6, 64, 2, 2, 1, 3),
    ("trimoff_per_axis_ragged_batch", 70, 64, 9, 12, 128, 3, 5, (2, 1), (1, 2)),
    ("trimoff_stride_gt_filter", 32, 64, 9, 9, 64, 2, 2, 3, 0),
]


@pytest.mark.parametrize("geo", TRIM_OFF, ids=[g[0] for g in TRIM_OFF])
def test_kernels_with_trimming_compiled_out(cks, oracle, geo):
    import torch
    from paper_2306_15951_amd import synth

    L = synth.Layer(*geo)
    print("geometry", geo, flush=True)
    s, p = synth.pair(L.stride), synth.pair(L.padding)
    for kind in ("int", "normal"):
        X, W, dY = synth.make_inputs(L, kind, 78)
        Y, dX, dW = nan_like(dY.shape), nan_like(X.shape), nan_like(W.shape)
        cks.cks_conv2d_fwd_untrimmed_hw(dev(X), dev(W), Y, s, p)
        cks.cks_deconv2d_untrimmed_hw(dev(dY), dev(W), dX, s, p)
        ws = torch.empty(max(cks.cks_dilated_conv2d_wgrad_workspace_hw(L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, s, p), 4) // 4,
                         dtype=torch.float32, device="cuda")
        got = [Y, dX]
        if L.N % 32 == 0:
            cks.cks_dilated_conv2d_wgrad_untrimmed_hw(dev(X), dev(dY), dW, s, p, ws)
            got.append(dW)
        else:   # no whole 32-image chunks: the variant does not exist, and says so
            with pytest.raises(cks.CksError) as e:
                cks.cks_dilated_conv2d_wgrad_untrimmed_hw(dev(X), dev(dY), dW, s, p, ws)
            assert e.value.status == cks.CKS_ERR_UNSUPPORTED
        torch.cuda.synchronize()
        want = oracle_three(oracle, L, X, W, dY)
        mags = oracle_three(oracle, L, np.abs(X), np.abs(W), np.abs(dY)) if kind == "normal" else want
        for g, w, m, nm in zip(got, want, mags, ("conv", "KS-deconv", "Sk-dilated")):
            if kind == "int":
                assert_exact(g.cpu().numpy(), w, "%s trim-off %s" % (L.name, nm))
            else:
                assert_close(g.cpu().numpy(), w, m, "%s trim-off %s" % (L.name, nm))


def test_trim_off_variants_say_what_they_cannot_do(cks):
    import torch

    X = torch.zeros((32, 6, 6, 36), device="cuda")          # 36 channels: no whole 32-channel chunks
    W = torch.zeros((64, 3, 3, 36), device="cuda")
    Y = torch.zeros((32, 6, 6, 64), device="cuda")
    X40, Y40 = torch.zeros((40, 6, 6, 36), device="cuda"), torch.zeros((40, 6, 6, 64), device="cuda")   # 40 images: no whole 32-image chunks
    for call in (lambda: cks.cks_conv2d_fwd_untrimmed_hw(X, W, Y, (1, 1), (1, 1)),
                 lambda: cks.cks_deconv2d_untrimmed_hw(Y, W, X, (1, 1), (1, 1)),
                 lambda: cks.cks_dilated_conv2d_wgrad_untrimmed_hw(X40, Y40, W, (1, 1), (1, 1), torch.zeros(1 << 20, device="cuda"))):
        with pytest.raises(cks.CksError) as e:
            call()
        assert e.value.status == cks.CKS_ERR_UNSUPPORTED


GUARD = [
    ("guards", 37, 8, 7, 9, 12, 3, 3, 2, 1),
    ("guards_stem", 5, 3, 23, 26, 64, 7, 7, 2, 3),
    ("guards_rgb", 7, 3, 10, 19, 12, 3, 3, 1, 1),
]


@pytest.mark.parametrize("guard_geo", GUARD, ids=[g[0] for g in GUARD])
def test_no_write_outside_outputs_and_unaligned_pointers(cks, oracle, guard_geo):
    """Outputs, inputs and workspaces sit inside guard bands; offsets of one
    float make every pointer 4-byte aligned only (scalar load path)."""
    import torch
    from paper_2306_15951_amd import synth

    L = synth.Layer(*guard_geo)
    print("geometry", guard_geo, flush=True)
    g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding)
    X, W, dY = synth.make_inputs(L, "int", 2)
    OH, OW = cks.cks_out_dims(L.IH, L.IW, L.FH, L.FW, L.stride, L.padding)
    want = oracle_three(oracle, L, X, W, dY)
    SENT = 12345.0
    for off in (64, 1):
        def guarded(n):
            buf = torch.full((n + 2 * off,), SENT, dtype=torch.float32, device="cuda")
            return buf, buf[off:off + n]

        def inside(a):
            buf, v = guarded(a.size)
            v.copy_(dev(a).reshape(-1))
            return v.view(a.shape)

        Xd, Wd, dYd = inside(X), inside(W), inside(dY)
        bY, vY = guarded(L.N * OH * OW * L.OC)
        bX, vX = guarded(X.size)
        bW, vW = guarded(W.size)
        b1, v1 = guarded(cks.cks_deconv2d_workspace(*g) // 4)
        b2, v2 = guarded(max(cks.cks_dilated_conv2d_wgrad_workspace(*g) // 4, 1))
        cks.cks_conv2d_fwd(Xd, Wd, vY.view(L.N, OH, OW, L.OC), L.stride, L.padding)
        cks.cks_deconv2d(dYd, Wd, vX.view(X.shape), L.stride, L.padding, v1)
        cks.cks_dilated_conv2d_wgrad(Xd, dYd, vW.view(W.shape), L.stride, L.padding, v2)
        torch.cuda.synchronize()
        for b, v, w, nm in ((bY, vY, want[0], "Y"), (bX, vX, want[1], "dX"), (bW, vW, want[2], "dW")):
            assert_exact(v.cpu().numpy().reshape(w.shape), w, "%s off=%d" % (nm, off))
        for b in (bY, bX, bW, b1, b2):
            h = b.cpu().numpy()
            assert np.all(h[:off] == SENT) and np.all(h[-off:] == SENT), "guard band overwritten (off=%d)" % off


def test_wgrad_is_reproducible_bit_for_bit(cks):
    """The split contraction axis is reduced in a fixed order."""
    import torch
    from paper_2306_15951_amd import synth

    L = synth.LAYERS["cfg2"]
    g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding)
    assert cks.cks_dilated_conv2d_wgrad_segments(*g) > 1
    X, W, dY = synth.make_inputs(L, "normal", 4)
    Xd, dYd = dev(X), dev(dY)
    ws = torch.empty(cks.cks_dilated_conv2d_wgrad_workspace(*g) // 4, device="cuda")
    outs = []
    for _ in range(3):
        dW = nan_like(W.shape)
        ws.fill_(float("nan"))
        cks.cks_dilated_conv2d_wgrad(Xd, dYd, dW, L.stride, L.padding, ws)
        torch.cuda.synchronize()
        outs.append(dW.cpu().numpy().view(np.uint32))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


WGRAD_STAGES = [
    ("general", 130, 40, 11, 12, 68, 3, 3, 2, 1),        # one tile per tap, many segments
    ("patch", 40, 16, 9, 10, 70, 3, 3, 1, 1),            # all taps in one tile
    ("stem", 6, 3, 40, 37, 64, 7, 7, 2, 3),              # input strip in LDS, one segment per workgroup
]


@pytest.mark.parametrize("geo", WGRAD_STAGES, ids=[g[0] for g in WGRAD_STAGES])
def test_wgrad_stage_entry_points(cks, oracle, geo):
    """Map step and reduce step of the filter gradient on their own: the segments' partial sums add
    up to the oracle's result (exactly, on integer inputs); on real inputs the reduce kernel returns
    their sum to fp32 rounding, the same bits every time."""
    import torch
    from paper_2306_15951_amd import synth

    L = synth.Layer(*geo)
    g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding)
    gz = cks.cks_dilated_conv2d_wgrad_segments(*g)
    print("geometry", geo, "segments", gz, flush=True)
    for kind in ("int", "normal"):
        X, W, dY = synth.make_inputs(L, kind, 11)
        part = nan_like((gz, L.OC, L.FH, L.FW, L.IC))
        cks.cks_dilated_conv2d_wgrad_partials(dev(X), dev(dY), part, L.FH, L.FW, L.stride, L.padding)
        dW, dW2 = nan_like(W.shape), nan_like(W.shape)
        cks.cks_reduce_partials(part, dW)
        cks.cks_reduce_partials(part, dW2)
        torch.cuda.synchronize()
        ph = part.cpu().numpy().astype(np.float64)
        assert np.isfinite(ph).all(), "a segment left part of its slice unwritten"
        got = dW.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), dW2.cpu().numpy().view(np.uint32))
        if kind == "int":
            want = oracle.wgrad(X, dY, L.FH, L.FW, L.stride, L.padding)
            assert_exact(ph.sum(0).astype(np.float32), want, "%s: sum of the partial slices" % L.name)
            assert_exact(got, want, "%s: reduce" % L.name)
        else:
            err = np.abs(got - ph.sum(0))
            assert (err <= gz * 2.0 ** -24 * np.abs(ph).sum(0) + 1e-30).all(), "reduce differs from the sum of the slices"


def test_stem_deconv_is_reproducible_bit_for_bit(cks):
    """The few-channel input gradient composes its sums in a fixed order (no atomics)."""
    import torch
    from paper_2306_15951_amd import synth

    L = synth.Layer("stem_repro", 40, 3, 48, 224, 64, 7, 7, 2, 3)   # workgroup runs start inside bands
    g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding)
    X, W, dY = synth.make_inputs(L, "normal", 5)
    ws = torch.empty(max(cks.cks_deconv2d_workspace(*g) // 4, 1), device="cuda")
    outs = []
    for _ in range(3):
        dX = nan_like(X.shape)
        ws.fill_(float("nan"))
        cks.cks_deconv2d(dev(dY), dev(W), dX, L.stride, L.padding, ws)
        torch.cuda.synchronize()
        outs.append(dX.cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    assert np.isfinite(outs[0]).all()


def test_deconv_without_workspace_where_none_is_used(cks, oracle):
    """A call whose sub-kernels are read from the filter in place (OC a multiple of 32, C of 4, aligned
    tensors) uses no workspace and accepts none; a call that needs Stage 1 is refused without one."""
    import torch
    from paper_2306_15951_amd import synth

    L = synth.Layer("inplace_no_ws", 70, 36, 11, 12, 96, 3, 3, 2, 1)
    X, W, dY = synth.make_inputs(L, "int", 8)
    dX = nan_like(X.shape)
    cks.cks_deconv2d(dev(dY), dev(W), dX, L.stride, L.padding, None)
    torch.cuda.synchronize()
    assert_exact(dX.cpu().numpy(), oracle.deconv(dY, W, L.IH, L.IW, L.stride, L.padding), "in place, no workspace")
    L2 = synth.Layer("split_needs_ws", 17, 5, 9, 10, 7, 3, 2, 2, 0)
    X2, W2, dY2 = synth.make_inputs(L2, "int", 8)
    with pytest.raises(cks.CksError) as e:
        cks.cks_deconv2d(dev(dY2), dev(W2), nan_like(X2.shape), L2.stride, L2.padding, None)
    assert e.value.status == cks.CKS_ERR_WORKSPACE


def test_errors_on_device(cks):
    import torch

    X = torch.zeros((2, 8, 8, 4), device="cuda")
    W = torch.zeros((4, 3, 3, 4), device="cuda")
    dX = torch.zeros_like(X)
    dY = torch.zeros((2, 8, 8, 4), device="cuda")
    small = torch.zeros(3, device="cuda")
    with pytest.raises(cks.CksError) as e:
        cks.cks_deconv2d(dY, W, dX, 1, 1, small)
    assert e.value.status == cks.CKS_ERR_WORKSPACE
    with pytest.raises(ValueError):
        cks.cks_conv2d_fwd(X, W, torch.zeros((2, 7, 8, 4), device="cuda"), 1, 1)


def planned_calls():
    """Every call this module makes on the GPU, as (CKS_OP_* number, layer tuple, mask of pointer arguments that
    are only 4-byte aligned).  tests/test_dispatch_coverage.py asks the library, on the host, which kernels
    these calls select, and fails if a kernel the library was built with is selected by none of them."""
    from paper_2306_15951_amd import synth

    FWD, DECONV, WGRAD, SPLIT, PRESPLIT_OP, TRANSPOSE, PARTIALS, REDUCE, FWD_T, FWD_U, DECONV_U, WGRAD_U = range(12)
    calls = []
    three = [tuple(synth.LAYERS["cfg0"])] + MID + RANDOM + ASYM + RANDOM_ASYM + RANDOM_STEM + WIDE_TILE
    three += [tuple(synth.LAYERS[n]) for n in FULL] + [("beyond_2GiB", 9, 64, 1024, 1024, 16, 3, 3, 1, 1)]
    for geo in three:
        calls += [(op, geo, 0) for op in (FWD, DECONV, WGRAD)]
    for geo in GUARD:                                    # once aligned, once with every pointer one float off
        calls += [(op, geo, m) for op in (FWD, DECONV, WGRAD) for m in (0, 15)]
    calls += [(op, tuple(synth.LAYERS["cfg1"]), 0) for op in (SPLIT, PRESPLIT_OP, TRANSPOSE, FWD_T)]
    for geo in FWD_TRANSPOSED:
        calls += [(op, geo, 0) for op in (TRANSPOSE, FWD_T)]
    for (OC, FH, FW, IC, s) in STAGE1:
        calls += [(op, ("stage1", 1, IC, FH, FW, OC, FH, FW, s, 0), 0) for op in (SPLIT, TRANSPOSE)]
    for geo in PRESPLIT:
        calls += [(op, geo, 0) for op in (SPLIT, PRESPLIT_OP)]
    for geo in WGRAD_STAGES:
        calls += [(op, geo, 0) for op in (PARTIALS, REDUCE)]
    for geo in TRIM_OFF:
        calls += [(op, geo, 0) for op in ((FWD_U, DECONV_U, WGRAD_U) if geo[1] % 32 == 0 else (FWD_U, DECONV_U))]
    calls.append((WGRAD, tuple(synth.LAYERS["cfg2"]), 0))
    calls.append((DECONV, ("stem_repro", 40, 3, 48, 224, 64, 7, 7, 2, 3), 0))
    return calls
