"""The operators before trimming -- plain convolution, KS-deconv (Algorithm 2) and Sk-dilated
(Algorithm 3) -- run through the library's own kernels, for the ablation the paper describes
(Sections IV.A-IV.C: what filter trimming adds on top of kernel split and leaping access).

The V2 kernels shorten their loops to the taps that lie over real data.  Given tensors whose zero border
is written out, with the padding argument lowered (convolution, filter gradient) or raised (input
gradient) to match, every trimmed range is the full one: the same kernels then multiply exactly the zeros
that the untrimmed algorithms' out-of-range loads supply, while kernel split and leaping access stay as
they are.  Each prepare_* function writes the border once (torch is used for that copy only; it is outside
any timed region) and returns a callable that makes just the library call.

    convolution       Xp = X with a border of p zeros;            cks_conv2d_fwd(Xp, W, padding 0)
    input gradient    dYq = dY with a border of q zeros;          cks_deconv2d(dYq, W, padding p + q*s)
    filter gradient   Xp as above;                                cks_dilated_conv2d_wgrad(Xp, dY, padding 0)

For the input gradient q >= ceil(F/s) - 1 = oph of Algorithm 2 on the low side and enough rows on the
high side that the last dX row's window ends inside dYq; the sub-kernels still have their own
ceil((F-y)/s) taps, so the multiply-adds are those of Algorithm 2: N*IC*OC*IH*IW*(taps of the class).
"""
from __future__ import annotations


def _pair(v):
    return (int(v[0]), int(v[1])) if isinstance(v, (tuple, list)) else (int(v), int(v))


def gradient_border(I, F, s, p):
    """Zeros to put on each side of one axis of dY so that no position's sub-kernel range is cut."""
    O = (I + 2 * p - F) // s + 1
    low = -(-F // s) - 1                       # oph of the largest sub-kernel
    high = (I - 1 + p) // s + 1 - O            # last window's end beyond dY
    return max(low, high, 0)


def prepare_conv2d_fwd(cks, X, Wt, Y, stride, padding):
    import torch.nn.functional as F

    (sh, sw), (ph, pw) = _pair(stride), _pair(padding)
    Xp = F.pad(X, (0, 0, pw, pw, ph, ph)).contiguous()
    return lambda: cks.cks_conv2d_fwd_hw(Xp, Wt, Y, (sh, sw), (0, 0))


def prepare_deconv2d(cks, dY, Wt, dX, stride, padding):
    import torch
    import torch.nn.functional as F

    (sh, sw), (ph, pw) = _pair(stride), _pair(padding)
    N, H, W, C = dX.shape
    OC, FH, FW, _ = Wt.shape
    qh, qw = gradient_border(H, FH, sh, ph), gradient_border(W, FW, sw, pw)
    dYq = F.pad(dY, (0, 0, qw, qw, qh, qh)).contiguous()
    pad2 = (ph + qh * sh, pw + qw * sw)
    need = cks.cks_deconv2d_workspace_hw(N, C, H, W, OC, FH, FW, (sh, sw), pad2)
    ws = torch.empty(max(need // 4, 1), device=dY.device)
    return lambda: cks.cks_deconv2d_hw(dYq, Wt, dX, (sh, sw), pad2, ws)


def prepare_dilated_conv2d_wgrad(cks, X, dY, dW, stride, padding):
    import torch
    import torch.nn.functional as F

    (sh, sw), (ph, pw) = _pair(stride), _pair(padding)
    N, H, W, C = X.shape
    OC, FH, FW, _ = dW.shape
    Xp = F.pad(X, (0, 0, pw, pw, ph, ph)).contiguous()
    need = cks.cks_dilated_conv2d_wgrad_workspace_hw(N, C, H + 2 * ph, W + 2 * pw, OC, FH, FW, (sh, sw), (0, 0))
    ws = torch.empty(max(need // 4, 1), device=X.device)
    return lambda: cks.cks_dilated_conv2d_wgrad_hw(Xp, dY, dW, (sh, sw), (0, 0), ws)
