"""The zero-skipping operators of the paper as index-set contractions, for SMALL inputs.

TEST INFRASTRUCTURE ONLY (see the package docstring).  ``cks_oracle.c`` is the textbook definition with
every zero written out.  This module states what Sections IV.A-IV.C do instead -- ConvV2 (Algorithm 1),
KS-deconv and KS-deconv-V2 (Algorithm 2 / 2B), Sk-dilated and Sk-dilated-V2 (Algorithm 3 / 3B) -- in one
common form: every output block is the contraction of two dense sub-arrays, chosen by the overlap of a
window with the real data, so that no operand is ever a padded or inserted zero.  The tests check that
these contractions reach exactly the textbook result and perform exactly the number of multiply-adds the
paper prints for its worked example (72 untrimmed, 50 trimmed: Figs. 4-8).

One rule serves all three operators.  A window of ``length`` cells that starts at cell ``start`` of an axis
holding ``limit`` real cells meets real data on the cells

    overlap(start, length, limit) = [max(-start, 0), min(limit - start, length))

(window-relative; empty if lo >= hi).  For ConvV2 the window is the filter over the input (Algorithm 1's
fh_s, fh_e), for KS-deconv-V2 it is a sub-kernel over the dense gradient (Algorithm 2B's ch_s, ch_e) and for
Sk-dilated-V2 it is, per filter tap, the run of output rows whose leaped-to input row exists (Algorithm 3B's
oh_s, oh_e, the same overlap divided by the stride with the ceilings taken towards +infinity).

Readings of the printed algorithms that this module takes (each is checked by a test):
  * Algorithm 2B bounds the trimmed sub-kernel range above by the outer padding ``oph``; that drops the last
    tap (8 instead of 50 operations on the worked example).  The bound is the sub-kernel extent oph + 1.
  * Algorithm 2B sums over ``ic``; the contraction runs over the output channels.
  * A sub-kernel whose extent is <= 0 (stride larger than the filter) is empty; its dX class is 0.
The untrimmed algorithms (trim=False) contract over the whole window; cells outside the data are zeros,
which are materialised here and counted as operations, as the paper's figures count them.

Every function returns (result as float64, number of multiply-adds); ks_deconv also returns how often each
dX position was written.
"""
from __future__ import annotations

import numpy as np


def _pair(v):
    """<sh sw> / <ph pw> of Table I; an int applies to both axes."""
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def _ceil_div(a, b):
    """Ceiling of a/b towards +infinity, b > 0, any integer a."""
    return -((-a) // b)


def overlap(start, length, limit, trim=True):
    """Cells [lo, hi) of a window of `length` cells starting at `start` that lie inside [0, limit).
    trim=False: the whole window."""
    if not trim:
        return 0, max(length, 0)
    lo, hi = max(-start, 0), min(limit - start, length)
    return (lo, hi) if hi > lo else (0, 0)


def subkernel_extent(F, y, s):
    """Taps of a filter axis of F taps that are congruent to y modulo s: ceil((F - y)/s), at least 0."""
    return max(_ceil_div(F - y, s), 0)


def _grown(A, before, after):
    """A[N, H, W, C] with zero rows / columns added: before = (top, left), after = (bottom, right)."""
    return np.pad(A, ((0, 0), (before[0], after[0]), (before[1], after[1]), (0, 0)))


def conv_v2(X, W, s, p):
    """Algorithm 1: at output position (oh, ow) the filter window starts at input cell (oh*sh - ph,
    ow*sw - pw); only its overlap with the input is contracted."""
    N, IH, IW, IC = X.shape
    OC, FH, FW, _ = W.shape
    (sh, sw), (ph, pw) = _pair(s), _pair(p)
    OH, OW = (IH + 2 * ph - FH) // sh + 1, (IW + 2 * pw - FW) // sw + 1
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    Y = np.zeros((N, OH, OW, OC))
    macs = 0
    for oh in range(OH):
        top = oh * sh - ph
        h0, h1 = overlap(top, FH, IH)
        for ow in range(OW):
            left = ow * sw - pw
            w0, w1 = overlap(left, FW, IW)
            patch = Xd[:, top + h0:top + h1, left + w0:left + w1, :]
            Y[:, oh, ow, :] = np.einsum("nhwc,ohwc->no", patch, Wd[:, h0:h1, w0:w1, :])
            macs += N * OC * IC * (h1 - h0) * (w1 - w0)
    return Y, macs


def ks_deconv(dY, C, IH, IW, FH, FW, s, p, trim):
    """Algorithm 2 Stage 2&3 (trim=False) / Algorithm 2B (trim=True) on the Stage-1 tensor
    ``C[sh, sw, OC, ceil(FH/sh), ceil(FW/sw), IC]`` (the paper's layout).

    Sub-kernel (y, x) serves the dX cells with (ih + ph) mod sh = y and (iw + pw) mod sw = x.  For such a
    cell, ih + ph = y + qh*sh, and its unit-stride window over the dense dY has the sub-kernel's extent CH
    and ends at row qh: it starts at qh - (CH - 1).  Stage 3 is the assignment into the interleaved place."""
    N, OH, OW, OC = dY.shape
    IC = C.shape[5]
    (sh, sw), (ph, pw) = _pair(s), _pair(p)
    CHmax, CWmax = C.shape[3], C.shape[4]
    # untrimmed: the gradient with a border of zeros wide enough for every window (Stage 2's outer padding)
    qh_max, qw_max = (IH - 1 + ph) // sh, (IW - 1 + pw) // sw
    bh, bw = max(CHmax - 1, 0), max(CWmax - 1, 0)
    G = _grown(dY.astype(np.float64), (bh, bw), (max(qh_max + 1 - OH, 0), max(qw_max + 1 - OW, 0)))
    Cd = C.astype(np.float64)
    dX = np.full((N, IH, IW, IC), np.nan)
    writes = np.zeros((IH, IW), dtype=np.int64)
    macs = 0
    for ih in range(IH):
        qh, y = divmod(ih + ph, sh)
        CH = subkernel_extent(FH, y, sh)
        top = qh - (CH - 1)
        h0, h1 = overlap(top, CH, OH, trim)
        for iw in range(IW):
            qw, x = divmod(iw + pw, sw)
            CW = subkernel_extent(FW, x, sw)
            left = qw - (CW - 1)
            w0, w1 = overlap(left, CW, OW, trim)
            window = G[:, bh + top + h0:bh + top + h1, bw + left + w0:bw + left + w1, :]
            dX[:, ih, iw, :] = np.einsum("nhwo,ohwc->nc", window, Cd[y, x, :, h0:h1, w0:w1, :])
            writes[ih, iw] += 1
            macs += N * OC * IC * (h1 - h0) * (w1 - w0)
    return dX, macs, writes


def sk_dilated(X, dY, FH, FW, s, p, trim):
    """Algorithm 3 (trim=False) / Algorithm 3B (trim=True): dY is used as it is; tap (fh, fw) meets the input
    cells (fh - ph + oh*sh, fw - pw + ow*sw), a leap of the stride per output cell.  The output rows whose
    input row exists are those of the overlap of the leaped-over stretch with the input, counted in leaps."""
    N, IH, IW, IC = X.shape
    _, OH, OW, OC = dY.shape
    (sh, sw), (ph, pw) = _pair(s), _pair(p)
    # untrimmed: the input with its zero border (and whatever the last leap reaches beyond it)
    reach_h, reach_w = (OH - 1) * sh + FH, (OW - 1) * sw + FW
    Xg = _grown(X.astype(np.float64), (ph, pw), (max(reach_h - IH - ph, 0), max(reach_w - IW - pw, 0)))
    dYd = dY.astype(np.float64)
    dW = np.zeros((OC, FH, FW, IC))
    macs = 0

    def leaps(first, step, count, limit):
        """Leap numbers [lo, hi) of first + k*step, k < count, that land inside [0, limit)."""
        if not trim:
            return 0, count
        lo, hi = max(_ceil_div(-first, step), 0), min(count, _ceil_div(limit - first, step))
        return (lo, hi) if hi > lo else (0, 0)

    for fh in range(FH):
        a0, a1 = leaps(fh - ph, sh, OH, IH)
        for fw in range(FW):
            b0, b1 = leaps(fw - pw, sw, OW, IW)
            rows = slice(fh + a0 * sh, fh + (a1 - 1) * sh + 1, sh) if a1 > a0 else slice(0, 0)
            cols = slice(fw + b0 * sw, fw + (b1 - 1) * sw + 1, sw) if b1 > b0 else slice(0, 0)
            dW[:, fh, fw, :] = np.einsum("nhwo,nhwc->oc", dYd[:, a0:a1, b0:b1, :], Xg[:, rows, cols, :])
            macs += N * OC * IC * (a1 - a0) * (b1 - b0)
    return dW, macs
