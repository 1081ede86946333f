"""Pins for the CPU oracle (no GPU needed).

The oracle (oracle/cks_oracle.c) is what every GPU result is compared with, so
it is tied here to things that are not itself: a brute-force scatter loop, an
independent library convolution (PyTorch CPU, float64), the adjoint identities,
finite differences, closed forms, and the numbers the paper prints for its
worked example.
"""
import itertools
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_int(rng, shape):
    return rng.integers(-3, 4, size=shape).astype(np.float32)


def geometry_sweep():
    """(N, IC, IH, IW, OC, FH, FW, s, p): non-square maps and filters, strides
    1-3, pad 0 .. >= filter, stride > filter, remainder rows."""
    out = []
    for (IH, IW), (FH, FW), s, p in itertools.product(
        [(3, 5), (4, 4), (5, 8), (7, 4)], [(1, 1), (2, 3), (3, 3), (4, 2), (5, 5)], [1, 2, 3], [0, 1, 2, 3]
    ):
        if IH + 2 * p < FH or IW + 2 * p < FW:
            continue
        out.append((2, 3, IH, IW, 2, FH, FW, s, p))
    return out


SWEEP = geometry_sweep()


def odims(g):
    N, IC, IH, IW, OC, FH, FW, s, p = g
    return (IH + 2 * p - FH) // s + 1, (IW + 2 * p - FW) // s + 1


def make(g, seed, integer=True):
    N, IC, IH, IW, OC, FH, FW, s, p = g
    OH, OW = odims(g)
    rng = np.random.default_rng(seed)
    if integer:
        return (rand_int(rng, (N, IH, IW, IC)), rand_int(rng, (OC, FH, FW, IC)), rand_int(rng, (N, OH, OW, OC)))
    return tuple(rng.standard_normal(sh).astype(np.float32)
                 for sh in ((N, IH, IW, IC), (OC, FH, FW, IC), (N, OH, OW, OC)))


def test_sweep_is_wide():
    assert len(SWEEP) > 150
    assert any(g[7] > g[5] for g in SWEEP)          # stride larger than filter
    assert any(g[8] >= g[5] for g in SWEEP)         # padding >= filter
    assert any((g[2] + 2 * g[8] - g[5]) % g[7] for g in SWEEP)   # remainder rows


def test_out_dim(oracle):
    # Table III / configurations: 16->8 (3x3 s2 p1), 224->112 (7x7 s2 p3), 32->16 (4x4 s2 p1)
    assert oracle.out_dim(16, 3, 2, 1) == 8
    assert oracle.out_dim(224, 7, 2, 3) == 112
    assert oracle.out_dim(32, 4, 2, 1) == 16
    assert oracle.out_dim(4, 3, 2, 1) == 2
    assert oracle.out_dim(7, 3, 1, 1) == 7


@pytest.mark.parametrize("chunk", range(4))
def test_brute_force_equals_oracle_exactly(oracle, chunk):
    for i, g in enumerate(SWEEP[chunk::4]):
        X, W, dY = make(g, 1000 + i)
        N, IC, IH, IW, OC, FH, FW, s, p = g
        Yb, dXb, dWb = oracle.brute(X, W, dY, s, p)
        assert np.array_equal(oracle.conv_fwd(X, W, s, p), Yb), g
        assert np.array_equal(oracle.deconv(dY, W, IH, IW, s, p), dXb), g
        assert np.array_equal(oracle.wgrad(X, dY, FH, FW, s, p), dWb), g


def test_against_library_convolution(oracle):
    """PyTorch's CPU convolution and its autograd, in float64, are an
    implementation that shares nothing with the oracle."""
    torch = pytest.importorskip("torch")
    for i, g in enumerate(SWEEP[::5]):
        N, IC, IH, IW, OC, FH, FW, s, p = g
        X, W, dY = make(g, 2000 + i, integer=False)
        xt = torch.from_numpy(X.astype(np.float64)).permute(0, 3, 1, 2).clone().requires_grad_(True)
        wt = torch.from_numpy(W.astype(np.float64)).permute(0, 3, 1, 2).clone().requires_grad_(True)
        yt = torch.nn.functional.conv2d(xt, wt, stride=s, padding=p)
        gy = torch.from_numpy(dY.astype(np.float64)).permute(0, 3, 1, 2)
        yt.backward(gy)
        Yl = yt.detach().permute(0, 2, 3, 1).numpy()
        dXl = xt.grad.permute(0, 2, 3, 1).numpy()
        dWl = wt.grad.permute(0, 2, 3, 1).numpy()
        np.testing.assert_allclose(oracle.conv_fwd(X, W, s, p), Yl, rtol=0, atol=1e-12)
        np.testing.assert_allclose(oracle.deconv(dY, W, IH, IW, s, p), dXl, rtol=0, atol=1e-12)
        np.testing.assert_allclose(oracle.wgrad(X, dY, FH, FW, s, p), dWl, rtol=0, atol=1e-11)


def test_library_transposed_convolution_layer(oracle):
    """A deconvolution layer's forward pass is Eq. (2) (Section II.A): compare
    with the library's conv_transpose2d when (IH+2p-FH) is a multiple of s."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(7)
    N, IC, OC, F, s, p, OH = 2, 3, 5, 4, 2, 1, 6
    IH = (OH - 1) * s + F - 2 * p
    dY = rng.standard_normal((N, OH, OH, OC)).astype(np.float32)
    W = rng.standard_normal((OC, F, F, IC)).astype(np.float32)
    ref = torch.nn.functional.conv_transpose2d(
        torch.from_numpy(dY.astype(np.float64)).permute(0, 3, 1, 2),
        torch.from_numpy(W.astype(np.float64)).permute(0, 3, 1, 2), stride=s, padding=p)
    assert ref.shape[2] == IH
    np.testing.assert_allclose(oracle.deconv(dY, W, IH, IH, s, p), ref.permute(0, 2, 3, 1).numpy(), atol=1e-12)


def test_adjoint_identities_exact(oracle):
    """<conv(X,W),R> = <X,deconv(R,W)> = <W,wgrad(X,R)>, exactly, on integers."""
    for i, g in enumerate(SWEEP[::3]):
        N, IC, IH, IW, OC, FH, FW, s, p = g
        X, W, R = make(g, 3000 + i)
        a = np.sum(oracle.conv_fwd(X, W, s, p) * R)
        b = np.sum(X * oracle.deconv(R, W, IH, IW, s, p))
        c = np.sum(W * oracle.wgrad(X, R, FH, FW, s, p))
        assert a == b == c, g


def test_finite_differences(oracle):
    """The operators are linear, so central differences of f = <conv(X,W),R>
    give deconv / wgrad up to rounding."""
    g = (2, 2, 5, 4, 3, 3, 2, 2, 1)
    N, IC, IH, IW, OC, FH, FW, s, p = g
    X, W, R = make(g, 11, integer=False)
    dX = oracle.deconv(R, W, IH, IW, s, p)
    dW = oracle.wgrad(X, R, FH, FW, s, p)
    h = 0.5  # exact in float32; f is linear in each argument
    rng = np.random.default_rng(5)

    def f(Xa, Wa):
        return float(np.sum(oracle.conv_fwd(Xa, Wa, s, p) * R))

    for _ in range(25):
        idx = tuple(rng.integers(0, d) for d in X.shape)
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += h
        Xm[idx] -= h
        assert abs((f(Xp, W) - f(Xm, W)) / (2 * h) - dX[idx]) < 1e-5 * (1 + abs(dX[idx]))
        idx = tuple(rng.integers(0, d) for d in W.shape)
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += h
        Wm[idx] -= h
        assert abs((f(X, Wp) - f(X, Wm)) / (2 * h) - dW[idx]) < 1e-5 * (1 + abs(dW[idx]))


def test_one_by_one_filter_is_a_matrix_product(oracle):
    rng = np.random.default_rng(3)
    X = rng.standard_normal((3, 4, 5, 6)).astype(np.float32)
    W = rng.standard_normal((7, 1, 1, 6)).astype(np.float32)
    R = rng.standard_normal((3, 4, 5, 7)).astype(np.float32)
    Xm, Wm, Rm = X.reshape(-1, 6).astype(np.float64), W.reshape(7, 6).astype(np.float64), R.reshape(-1, 7).astype(np.float64)
    np.testing.assert_allclose(oracle.conv_fwd(X, W, 1, 0).reshape(-1, 7), Xm @ Wm.T, atol=1e-12)
    np.testing.assert_allclose(oracle.deconv(R, W, 4, 5, 1, 0).reshape(-1, 6), Rm @ Wm, atol=1e-12)
    np.testing.assert_allclose(oracle.wgrad(X, R, 1, 1, 1, 0).reshape(7, 6), Rm.T @ Xm, atol=1e-12)


def test_all_ones_counts_the_real_taps(oracle):
    """With X = W = 1 every output equals IC x (number of taps over real input),
    which pins the padding convention at every border."""
    N, IC, IH, IW, OC, FH, FW, s, p = 1, 3, 7, 6, 2, 3, 5, 2, 2
    Y = oracle.conv_fwd(np.ones((N, IH, IW, IC)), np.ones((OC, FH, FW, IC)), s, p)
    OH, OW = Y.shape[1:3]
    for oh in range(OH):
        for ow in range(OW):
            rows = sum(1 for fh in range(FH) if 0 <= oh * s - p + fh < IH)
            cols = sum(1 for fw in range(FW) if 0 <= ow * s - p + fw < IW)
            assert np.all(Y[0, oh, ow] == IC * rows * cols)


def test_delta_input_copies_the_filter(oracle):
    """A single 1 in X at (ih,iw): Y[oh,ow,oc] = W[oc, ih+p-oh*s, iw+p-ow*s]."""
    rng = np.random.default_rng(9)
    IH, IW, FH, FW, s, p, OC = 6, 7, 3, 4, 2, 1, 3
    W = rng.standard_normal((OC, FH, FW, 1)).astype(np.float32)
    X = np.zeros((1, IH, IW, 1), np.float32)
    ih, iw = 3, 4
    X[0, ih, iw, 0] = 1
    Y = oracle.conv_fwd(X, W, s, p)
    for oh in range(Y.shape[1]):
        for ow in range(Y.shape[2]):
            fh, fw = ih + p - oh * s, iw + p - ow * s
            want = W[:, fh, fw, 0] if 0 <= fh < FH and 0 <= fw < FW else np.zeros(OC)
            assert np.array_equal(Y[0, oh, ow], want.astype(np.float64))
    # and the mirror statement for Eq. (2): a single 1 in dY spreads the filter into dX
    dY = np.zeros_like(Y, dtype=np.float32)
    dY[0, 1, 2, 1] = 1
    dX = oracle.deconv(dY, W, IH, IW, s, p)
    want = np.zeros((IH, IW))
    for fh in range(FH):
        for fw in range(FW):
            a, b = 1 * s - p + fh, 2 * s - p + fw
            if 0 <= a < IH and 0 <= b < IW:
                want[a, b] = W[1, fh, fw, 0]
    assert np.array_equal(dX[0, :, :, 0], want)


def test_remainder_rows_get_zero_gradient(oracle):
    """(IH+2p-FH) mod s != 0: the last input rows are never read, so dX there is 0."""
    g = (1, 2, 8, 8, 2, 3, 3, 2, 0)   # OH = 3, rows 0..6 used, row 7 untouched
    X, W, dY = make(g, 4)
    dX = oracle.deconv(dY, W, 8, 8, 2, 0)
    assert np.all(dX[:, 7] == 0) and np.all(dX[:, :, 7] == 0)
    assert np.any(dX[:, 6] != 0)


def test_sampled_mode_equals_full_mode(oracle):
    g = (2, 3, 7, 5, 4, 3, 3, 2, 1)
    N, IC, IH, IW, OC, FH, FW, s, p = g
    X, W, dY = make(g, 21, integer=False)
    rng = np.random.default_rng(1)
    for full, fn in ((oracle.conv_fwd(X, W, s, p), lambda sm: oracle.conv_fwd(X, W, s, p, sample=sm)),
                     (oracle.deconv(dY, W, IH, IW, s, p), lambda sm: oracle.deconv(dY, W, IH, IW, s, p, sample=sm)),
                     (oracle.wgrad(X, dY, FH, FW, s, p), lambda sm: oracle.wgrad(X, dY, FH, FW, s, p, sample=sm))):
        sm = rng.integers(0, full.size, size=50)
        assert np.array_equal(fn(sm), full.ravel()[sm])


def test_mac_counts_closed_forms(oracle):
    # Table III (with the batch factor restored in T_Dilated)
    N, IC, IH, IW, OC, FH, FW, s, p = 3, 5, 16, 12, 7, 3, 5, 2, 1
    OH, OW = (IH + 2 * p - FH) // s + 1, (IW + 2 * p - FW) // s + 1
    c = oracle.mac_counts(N, IC, IH, IW, OC, FH, FW, s, p)
    assert 2 * c["dense"] == 2 * (OC * N * OH * OW * FH * FW * IC)
    assert 2 * c["nominal_deconv"] == 2 * (IC * N * IH * IW * FH * FW * OC)
    OHp, OWp = OH + (OH - 1) * (s - 1), OW + (OW - 1) * (s - 1)
    assert 2 * c["nominal_dilated"] == 2 * (N * OC * FH * FW * IC * OHp * OWp)
    # 3x3, stride 1, pad 1: S = 3*I - 2 per axis
    for I in (4, 7, 32):
        c = oracle.mac_counts(2, 3, I, I, 5, 3, 3, 1, 1)
        assert c["useful"] == 2 * 3 * 5 * (3 * I - 2) ** 2
        assert c["dense"] == 2 * 3 * 5 * 9 * I * I
    # no padding: nothing to trim
    c = oracle.mac_counts(1, 1, 9, 9, 1, 3, 3, 2, 0)
    assert c["useful"] == c["dense"]


def test_paper_worked_example(oracle):
    """The one example the paper works through (Figs. 1, 4-8)."""
    from oracle import algorithms as alg

    gold = json.load(open(os.path.join(GOLDEN, "worked_example.json")))
    g = gold["geometry"]
    geo = (g["N"], g["IC"], g["IH"], g["IW"], g["OC"], g["FH"], g["FW"], g["stride"], g["padding"])
    N, IC, IH, IW, OC, FH, FW, s, p = geo
    assert [oracle.out_dim(IH, FH, s, p), oracle.out_dim(IW, FW, s, p)] == gold["output_hw"]
    c = oracle.mac_counts(*geo)
    assert 2 * c["dense"] == gold["dense_flops"]
    assert 2 * c["useful"] == gold["trimmed_flops"]
    X, W, dY = make(geo, 77)
    # each algorithm performs exactly the printed number of operations ...
    Y, m = alg.conv_v2(X, W, s, p)
    assert 2 * m == gold["trimmed_flops"]
    C = oracle.kernel_split(W, s)
    assert list(C.shape[0:2]) + list(C.shape[3:5]) == gold["split_tensor_shape_spatial"]
    for key, ext in gold["subkernel_extents"].items():
        y, x = int(key[0]), int(key[1])
        assert [alg.subkernel_extent(FH, y, s), alg.subkernel_extent(FW, x, s)] == ext
        nz = np.argwhere(C[y, x, 0, :, :, 0] != 0)
        assert nz[:, 0].max(initial=-1) < ext[0] and nz[:, 1].max(initial=-1) < ext[1]
    dX0, m0, _ = alg.ks_deconv(dY, C, IH, IW, FH, FW, s, p, trim=False)
    dX1, m1, _ = alg.ks_deconv(dY, C, IH, IW, FH, FW, s, p, trim=True)
    assert (2 * m0, 2 * m1) == (gold["dense_flops"], gold["trimmed_flops"])
    dW0, k0 = alg.sk_dilated(X, dY, FH, FW, s, p, trim=False)
    dW1, k1 = alg.sk_dilated(X, dY, FH, FW, s, p, trim=True)
    assert (2 * k0, 2 * k1) == (gold["dense_flops"], gold["trimmed_flops"])
    # ... and reaches the textbook result
    assert np.array_equal(Y, oracle.conv_fwd(X, W, s, p))
    assert np.array_equal(dX0, oracle.deconv(dY, W, IH, IW, s, p)) and np.array_equal(dX1, dX0)
    assert np.array_equal(dW0, oracle.wgrad(X, dY, FH, FW, s, p)) and np.array_equal(dW1, dW0)


def test_literal_upper_bound_of_algorithm_2b_contradicts_the_worked_example():
    """Algorithm 2B as printed bounds the trimmed sub-kernel range above by the outer padding oph = extent - 1.
    Counted that way the worked example (4x4 map, 3x3 filter, stride 2, padding 1) costs 8 operations; the
    paper prints 50, which is what the sub-kernel extent as the bound gives."""
    from oracle import algorithms as alg

    gold = json.load(open(os.path.join(GOLDEN, "worked_example.json")))
    g = gold["geometry"]
    I, F, s, p = g["IH"], g["FH"], g["stride"], g["padding"]
    O = (I + 2 * p - F) // s + 1

    def taps_per_axis(literal):
        total = 0
        for i in range(I):
            q, y = divmod(i + p, s)
            ext = alg.subkernel_extent(F, y, s)
            start = q - (ext - 1)
            lo, hi = max(-start, 0), min(O - start, ext - 1 if literal else ext)
            total += max(hi - lo, 0)
        return total

    assert 2 * taps_per_axis(False) ** 2 == gold["trimmed_flops"] == 50
    assert 2 * taps_per_axis(True) ** 2 == 8


def test_appendix_algorithms_reach_the_textbook_result(oracle):
    """Algorithms 1, 2+2B, 3+3B (with the readings listed in oracle/algorithms.py)
    against the explicit-zero operators, exactly, over the geometry sweep; all
    three skip the same number of multiply-adds; every dX element is written by
    exactly one sub-kernel class."""
    from oracle import algorithms as alg

    for i, g in enumerate(SWEEP[::2]):
        N, IC, IH, IW, OC, FH, FW, s, p = g
        g = (1, 2, IH, IW, 2, FH, FW, s, p)
        N, IC, OC = 1, 2, 2
        X, W, dY = make(g, 5000 + i)
        useful = oracle.mac_counts(*g)["useful"]
        Y, m = alg.conv_v2(X, W, s, p)
        assert np.array_equal(Y, oracle.conv_fwd(X, W, s, p)) and m == useful, g
        C = oracle.kernel_split(W, s)
        dX, m, writes = alg.ks_deconv(dY, C, IH, IW, FH, FW, s, p, trim=True)
        assert np.all(writes == 1), g
        assert np.array_equal(dX, oracle.deconv(dY, W, IH, IW, s, p)) and m == useful, g
        dX, _, _ = alg.ks_deconv(dY, C, IH, IW, FH, FW, s, p, trim=False)
        assert np.array_equal(dX, oracle.deconv(dY, W, IH, IW, s, p)), g
        dW, m = alg.sk_dilated(X, dY, FH, FW, s, p, trim=True)
        assert np.array_equal(dW, oracle.wgrad(X, dY, FH, FW, s, p)) and m == useful, g


def test_kernel_split_is_a_rotated_partition_of_the_filter(oracle):
    """Every filter tap lands in exactly one sub-kernel entry, at the place the
    rotation puts it; the padded entries stay zero."""
    rng = np.random.default_rng(12)
    for FH, FW, s in [(3, 3, 2), (4, 4, 2), (7, 7, 2), (5, 3, 3), (3, 3, 1), (1, 1, 2), (2, 5, 4)]:
        OC, IC = 2, 3
        W = (rng.permutation(OC * FH * FW * IC) + 1).astype(np.float32).reshape(OC, FH, FW, IC)
        C = oracle.kernel_split(W, s)
        assert C.shape == (s, s, OC, -(-FH // s), -(-FW // s), IC)
        assert sorted(C[C != 0].tolist()) == sorted(W.ravel().tolist())
        Wr = W[:, ::-1, ::-1, :]          # rot180
        for y in range(s):
            for x in range(s):
                # taps of the rotated filter seen by class (y,x), in order
                rows = sorted(FH - 1 - fh for fh in range(FH) if fh % s == y)
                cols = sorted(FW - 1 - fw for fw in range(FW) if fw % s == x)
                got = C[y, x, :, :len(rows), :len(cols), :]
                if rows and cols:
                    assert np.array_equal(got, Wr[:, rows][:, :, cols]), (FH, FW, s, y, x)
                mask = np.ones(C.shape[3:5], bool)
                mask[:len(rows), :len(cols)] = False
                assert np.all(C[y, x][:, mask] == 0)


# ---------------------------------------------------------------- per-axis stride and padding
# Table I writes stride and padding as <sh sw> and <ph pw>.  The same pins, on geometries whose two
# axes differ in everything: a mistake that swaps the axes anywhere fails them.

def asym_sweep():
    """(N, IC, IH, IW, OC, FH, FW, (sh, sw), (ph, pw)) with sh != sw or ph != pw."""
    out = []
    for (IH, IW), (FH, FW), st, pd in itertools.product(
        [(5, 8), (7, 4), (6, 6)], [(3, 3), (2, 3), (4, 1), (5, 2)],
        [(1, 2), (2, 1), (2, 3), (3, 1), (4, 2)], [(0, 1), (1, 0), (2, 1), (1, 3), (0, 0), (3, 3)]
    ):
        if st[0] == st[1] and pd[0] == pd[1]:
            continue
        if IH + 2 * pd[0] < FH or IW + 2 * pd[1] < FW:
            continue
        out.append((2, 3, IH, IW, 2, FH, FW, st, pd))
    return out


ASYM = asym_sweep()


def make_asym(g, seed, integer=True):
    N, IC, IH, IW, OC, FH, FW, (sh, sw), (ph, pw) = g
    OH, OW = (IH + 2 * ph - FH) // sh + 1, (IW + 2 * pw - FW) // sw + 1
    rng = np.random.default_rng(seed)
    shapes = ((N, IH, IW, IC), (OC, FH, FW, IC), (N, OH, OW, OC))
    if integer:
        return tuple(rand_int(rng, sh_) for sh_ in shapes)
    return tuple(rng.standard_normal(sh_).astype(np.float32) for sh_ in shapes)


def test_asymmetric_sweep_is_wide():
    assert len(ASYM) > 250
    assert any(g[7][0] > g[5] or g[7][1] > g[6] for g in ASYM)      # a stride larger than the filter
    assert any((g[2] + 2 * g[8][0] - g[5]) % g[7][0] for g in ASYM)   # remainder rows


@pytest.mark.parametrize("chunk", range(4))
def test_asymmetric_brute_force_equals_oracle_exactly(oracle, chunk):
    for i, g in enumerate(ASYM[chunk::4]):
        X, W, dY = make_asym(g, 7000 + i)
        N, IC, IH, IW, OC, FH, FW, st, pd = g
        Yb, dXb, dWb = oracle.brute(X, W, dY, st, pd)
        assert np.array_equal(oracle.conv_fwd(X, W, st, pd), Yb), g
        assert np.array_equal(oracle.deconv(dY, W, IH, IW, st, pd), dXb), g
        assert np.array_equal(oracle.wgrad(X, dY, FH, FW, st, pd), dWb), g


def test_asymmetric_against_library_convolution(oracle):
    torch = pytest.importorskip("torch")
    for i, g in enumerate(ASYM[::7]):
        N, IC, IH, IW, OC, FH, FW, st, pd = g
        X, W, dY = make_asym(g, 8000 + i, integer=False)
        xt = torch.from_numpy(X.astype(np.float64)).permute(0, 3, 1, 2).clone().requires_grad_(True)
        wt = torch.from_numpy(W.astype(np.float64)).permute(0, 3, 1, 2).clone().requires_grad_(True)
        yt = torch.nn.functional.conv2d(xt, wt, stride=st, padding=pd)
        yt.backward(torch.from_numpy(dY.astype(np.float64)).permute(0, 3, 1, 2))
        np.testing.assert_allclose(oracle.conv_fwd(X, W, st, pd), yt.detach().permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(oracle.deconv(dY, W, IH, IW, st, pd), xt.grad.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(oracle.wgrad(X, dY, FH, FW, st, pd), wt.grad.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-11)


def test_asymmetric_all_ones_counts_the_real_taps(oracle):
    """With X = W = 1 an output is IC times the number of its taps over real input: per axis the
    trimmed range of Algorithm 1 with that axis' own stride and padding."""
    N, IC, IH, IW, OC, FH, FW, (sh, sw), (ph, pw) = 1, 3, 7, 9, 2, 4, 3, (3, 2), (2, 1)
    Y = oracle.conv_fwd(np.ones((N, IH, IW, IC), np.float32), np.ones((OC, FH, FW, IC), np.float32), (sh, sw), (ph, pw))
    OH, OW = (IH + 2 * ph - FH) // sh + 1, (IW + 2 * pw - FW) // sw + 1
    assert Y.shape == (N, OH, OW, OC)
    for oh in range(OH):
        for ow in range(OW):
            th = min(IH - (oh * sh - ph), FH) - max(ph - oh * sh, 0)
            tw = min(IW - (ow * sw - pw), FW) - max(pw - ow * sw, 0)
            assert np.all(Y[0, oh, ow] == IC * th * tw)
    c = oracle.mac_counts(N, IC, IH, IW, OC, FH, FW, (sh, sw), (ph, pw))
    assert c["useful"] == int(Y.sum())   # N*IC*OC*S_h*S_w
    assert c["dense"] == N * IC * OC * OH * OW * FH * FW
    assert c["nominal_dilated"] == N * IC * OC * FH * FW * ((OH - 1) * sh + 1) * ((OW - 1) * sw + 1)


def test_asymmetric_appendix_algorithms_reach_the_textbook_result(oracle):
    from oracle import algorithms as alg

    for i, g in enumerate(ASYM[::5]):
        _, _, IH, IW, _, FH, FW, st, pd = g
        g = (1, 2, IH, IW, 2, FH, FW, st, pd)
        X, W, dY = make_asym(g, 9000 + i)
        useful = oracle.mac_counts(*g)["useful"]
        Y, m = alg.conv_v2(X, W, st, pd)
        assert np.array_equal(Y, oracle.conv_fwd(X, W, st, pd)) and m == useful, g
        C = oracle.kernel_split(W, st)
        assert C.shape == (st[0], st[1], 2, -(-FH // st[0]), -(-FW // st[1]), 2)
        dX, m, writes = alg.ks_deconv(dY, C, IH, IW, FH, FW, st, pd, trim=True)
        assert np.all(writes == 1), g
        assert np.array_equal(dX, oracle.deconv(dY, W, IH, IW, st, pd)) and m == useful, g
        dW, m = alg.sk_dilated(X, dY, FH, FW, st, pd, trim=True)
        assert np.array_equal(dW, oracle.wgrad(X, dY, FH, FW, st, pd)) and m == useful, g


def test_asymmetric_kernel_split_partitions_the_filter(oracle):
    rng = np.random.default_rng(13)
    for FH, FW, sh, sw in [(3, 3, 2, 1), (4, 5, 2, 3), (7, 7, 3, 2), (2, 5, 4, 1), (1, 3, 2, 2)]:
        OC, IC = 2, 3
        W = (rng.permutation(OC * FH * FW * IC) + 1).astype(np.float32).reshape(OC, FH, FW, IC)
        C = oracle.kernel_split(W, (sh, sw))
        assert sorted(C[C != 0].tolist()) == sorted(W.ravel().tolist())
        Wr = W[:, ::-1, ::-1, :]
        for y in range(sh):
            for x in range(sw):
                rows = sorted(FH - 1 - fh for fh in range(FH) if fh % sh == y)
                cols = sorted(FW - 1 - fw for fw in range(FW) if fw % sw == x)
                if rows and cols:
                    assert np.array_equal(C[y, x, :, :len(rows), :len(cols), :], Wr[:, rows][:, :, cols]), (FH, FW, sh, sw, y, x)


def test_filter_transpose(oracle):
    rng = np.random.default_rng(2)
    W = rng.standard_normal((5, 3, 2, 7)).astype(np.float32)
    assert np.array_equal(oracle.filter_transpose(W), np.transpose(W, (1, 2, 3, 0)))


def test_oracle_rejects_bad_geometry(oracle):
    X = np.zeros((1, 2, 2, 1), np.float32)
    W = np.zeros((1, 5, 5, 1), np.float32)
    with pytest.raises(ValueError):
        oracle.conv_fwd(X, W, 1, 1)   # 2 + 2*1 < 5
