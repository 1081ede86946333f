"""The zero-skipping algorithms of the appendix, step by step, for TINY inputs.

TEST INFRASTRUCTURE ONLY (see the package docstring).  These are slow Python
loops in the paper's notation.  They exist to check, on the CPU, that the
index algebra the paper gives (with the readings listed below) reaches exactly
the textbook result of ``cks_oracle.c`` while touching only non-zero operands,
and to count the multiply-adds each algorithm performs (the paper prints these
counts for its worked example, Figs. 4-8).

Readings of the printed algorithms that are used here:
  * Algorithm 2B bounds the trimmed sub-kernel range with ``oph``/``opw``; that
    drops the last tap.  The upper bound must be the sub-kernel extent
    ``C_H = oph + 1`` (the analogue of ``min(I_H - ih_s, F_H)`` in Algorithm 1).
  * Algorithm 2B sums over ``ic``; the contraction index is ``oc``.
  * Ceilings of negative numerators are mathematical ceilings.
  * A sub-kernel whose extent is <= 0 (stride larger than the filter) is empty
    and the dX elements of its class are 0.
Every function returns (result as float64, number of multiply-adds).
"""
from __future__ import annotations

import numpy as np


def _cdiv(a, b):
    """Mathematical ceiling of a/b for b > 0 and any integer a."""
    return -((-a) // b)


def _pair(v):
    """<sh sw> / <ph pw> of Table I; an int applies to both axes."""
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def _out_dim(I, F, s, p):
    return (I + 2 * p - F) // s + 1


def conv_v2(X, W, s, p):
    """Algorithm 1 (ConvV2): per output position the filter is cut down to
    [fh_s, fh_e) x [fw_s, fw_e), the part that lies over real input."""
    N, IH, IW, IC = X.shape
    OC, FH, FW, _ = W.shape
    (sh, sw), (ph, pw) = _pair(s), _pair(p)
    OH, OW = _out_dim(IH, FH, sh, ph), _out_dim(IW, FW, sw, pw)
    Y = np.zeros((N, OH, OW, OC))
    macs = 0
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    for n in range(N):
        for oh in range(OH):
            for ow in range(OW):
                ih_s, iw_s = oh * sh - ph, ow * sw - pw
                fh_s, fh_e = max(-ih_s, 0), min(IH - ih_s, FH)
                fw_s, fw_e = max(-iw_s, 0), min(IW - iw_s, FW)
                for oc in range(OC):
                    acc = 0.0
                    for fh in range(fh_s, fh_e):
                        for fw in range(fw_s, fw_e):
                            for ic in range(IC):
                                acc += Xd[n, ih_s + fh, iw_s + fw, ic] * Wd[oc, fh, fw, ic]
                                macs += 1
                    Y[n, oh, ow, oc] = acc
    return Y, macs


def subkernel_extent(F, y, s):
    """ceil((F - y)/s), clamped at 0: taps of the filter congruent to y mod s."""
    return max(_cdiv(F - y, s), 0)


def ks_deconv(dY, C, IH, IW, FH, FW, s, p, trim):
    """Algorithm 2 Stage 2&3 (trim=False) / Algorithm 2B (trim=True).

    ``C`` is the Stage-1 tensor in the paper's layout [sh,sw,OC,CHp,CWp,IC].
    Class (y,x) owns the dX elements with (ih+ph) mod sh == y, (iw+pw) mod sw == x.
    Also returns how often each dX element was written (must be exactly once)."""
    N, OH, OW, OC = dY.shape
    IC = C.shape[5]
    (sh, sw), (ph, pw) = _pair(s), _pair(p)
    dX = np.full((N, IH, IW, IC), np.nan)
    writes = np.zeros((IH, IW), dtype=np.int64)
    macs = 0
    dYd, Cd = dY.astype(np.float64), C.astype(np.float64)
    for y in range(sh):
        for x in range(sw):
            CH, CW = subkernel_extent(FH, y, sh), subkernel_extent(FW, x, sw)
            oph, opw = CH - 1, CW - 1
            ih_s, iw_s = y - ph, x - pw
            if ih_s < 0:
                ih_s += _cdiv(-ih_s, sh) * sh
            if iw_s < 0:
                iw_s += _cdiv(-iw_s, sw) * sw
            for u in range(_cdiv(IH, sh)):
                for v in range(_cdiv(IW, sw)):
                    ih, iw = u * sh + ih_s, v * sw + iw_s
                    if not (0 <= ih < IH and 0 <= iw < IW):
                        continue
                    assert (ih + ph - y) % sh == 0 and (iw + pw - x) % sw == 0
                    oh_s = (ih + ph - y) // sh - oph
                    ow_s = (iw + pw - x) // sw - opw
                    if trim:
                        ch_s, ch_e = max(-oh_s, 0), min(OH - oh_s, CH)
                        cw_s, cw_e = max(-ow_s, 0), min(OW - ow_s, CW)
                    else:
                        ch_s, ch_e, cw_s, cw_e = 0, CH, 0, CW
                    writes[ih, iw] += 1
                    for n in range(N):
                        for ic in range(IC):
                            acc = 0.0
                            for ch in range(ch_s, ch_e):
                                for cw in range(cw_s, cw_e):
                                    oh, ow = oh_s + ch, ow_s + cw
                                    if not trim and not (0 <= oh < OH and 0 <= ow < OW):
                                        macs += OC  # Alg. 2 as printed skips these; Fig. 5 counts them
                                        continue
                                    for oc in range(OC):
                                        acc += dYd[n, oh, ow, oc] * Cd[y, x, oc, ch, cw, ic]
                                        macs += 1
                            dX[n, ih, iw, ic] = acc
    return dX, macs, writes


def sk_dilated(X, dY, FH, FW, s, p, trim):
    """Algorithm 3 (trim=False) / Algorithm 3B (trim=True): dY is used as it is,
    X is read with a leaping step (sh, sw)."""
    N, IH, IW, IC = X.shape
    _, OH, OW, OC = dY.shape
    (sh, sw), (ph, pw) = _pair(s), _pair(p)
    dW = np.zeros((OC, FH, FW, IC))
    macs = 0
    Xd, dYd = X.astype(np.float64), dY.astype(np.float64)
    for fh in range(FH):
        for fw in range(FW):
            ih_s, iw_s = fh - ph, fw - pw
            if trim:
                oh_s, oh_e = max(_cdiv(-ih_s, sh), 0), min(OH, _cdiv(IH - ih_s, sh))
                ow_s, ow_e = max(_cdiv(-iw_s, sw), 0), min(OW, _cdiv(IW - iw_s, sw))
            else:
                oh_s, oh_e, ow_s, ow_e = 0, OH, 0, OW
            for oc in range(OC):
                for ic in range(IC):
                    acc = 0.0
                    for n in range(N):
                        for oh in range(oh_s, oh_e):
                            for ow in range(ow_s, ow_e):
                                ih, iw = oh * sh + ih_s, ow * sw + iw_s
                                if not trim and not (0 <= ih < IH and 0 <= iw < IW):
                                    macs += 1  # Alg. 3 as printed skips these; Fig. 7 counts them
                                    continue
                                acc += Xd[n, ih, iw, ic] * dYd[n, oh, ow, oc]
                                macs += 1
                    dW[oc, fh, fw, ic] = acc
    return dW, macs
