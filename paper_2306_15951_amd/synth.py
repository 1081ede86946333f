"""Seeded synthetic inputs and the benchmark layer geometries.

This module holds no arithmetic of the method: it only names layer shapes and
draws random tensors.  Both the GPU tests/benchmark and the CPU oracle's tests
take their inputs from here, so that both sides see identical bits.

Layouts (paper, Section IV, paragraph before Eq. (1)):
    X  [N, IH, IW, IC]     W [OC, FH, FW, IC]     dY [N, OH, OW, OC]     float32
"""
from __future__ import annotations

from collections import namedtuple

import numpy as np

# stride / padding: an int (both axes) or a pair (vertical, horizontal)
Layer = namedtuple("Layer", "name N IC IH IW OC FH FW stride padding")

# Canonical conv-layer parameters of the benchmark configurations.  "cfg4a" is
# the deconvolution-layer upsampler (16x16x256 -> 32x32x128, 4x4, s2, p1)
# written from the convolution side: its forward pass is the deconvolution
# operator, its input gradient the convolution operator.  Its He-normal filter
# is drawn like every other layer's, with the fan-in of the convolution side:
# std = sqrt(2 / (FH*FW*IC)) with IC = 128 (the 32x32 side's channels), not the
# 256 channels that feed the layer when it is used as an upsampler.  The choice
# only scales W; timings and parity bars do not depend on it.
LAYERS = {
    "cfg0": Layer("cfg0", 2, 4, 8, 8, 4, 3, 3, 1, 1),
    "cfg1": Layer("cfg1", 128, 64, 32, 32, 64, 3, 3, 1, 1),
    "cfg2": Layer("cfg2", 128, 128, 16, 16, 256, 3, 3, 2, 1),
    "cfg3a": Layer("cfg3a", 256, 512, 7, 7, 512, 3, 3, 1, 1),
    "cfg3b": Layer("cfg3b", 256, 512, 4, 4, 512, 3, 3, 1, 1),
    "cfg4a": Layer("cfg4a", 64, 128, 32, 32, 256, 4, 4, 2, 1),
    "cfg4b": Layer("cfg4b", 64, 3, 224, 224, 64, 7, 7, 2, 3),
}

BASE_SEED = 230615951


def pair(v):
    """Stride or padding of a Layer as (vertical, horizontal); an int applies to both axes."""
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def out_hw(L):
    (sh, sw), (ph, pw) = pair(L.stride), pair(L.padding)
    return (L.IH + 2 * ph - L.FH) // sh + 1, (L.IW + 2 * pw - L.FW) // sw + 1


def shapes(L):
    OH, OW = out_hw(L)
    return (L.N, L.IH, L.IW, L.IC), (L.OC, L.FH, L.FW, L.IC), (L.N, OH, OW, L.OC)


def make_inputs(L, kind="normal", seed=0):
    """Return (X, W, dY) as float32 numpy arrays.

    kind = "normal":  X, dY ~ N(0,1); W ~ N(0, 2/(FH*FW*IC))  (He-normal)
           "uniform": all three uniform in [-1, 1]
           "int":     all three integers uniform in {-3..3}, stored as float32
                      (every partial sum of every operator is then exact in
                      float32 as long as 9 * K < 2^24)
    """
    xs, ws, ys = shapes(L)
    rng = [np.random.default_rng([BASE_SEED, seed, i]) for i in range(3)]
    if kind == "normal":
        X = rng[0].standard_normal(xs, dtype=np.float32)
        W = rng[1].standard_normal(ws, dtype=np.float32) * np.float32(np.sqrt(2.0 / (L.FH * L.FW * L.IC)))
        dY = rng[2].standard_normal(ys, dtype=np.float32)
    elif kind == "uniform":
        X, W, dY = (r.uniform(-1.0, 1.0, size=s).astype(np.float32) for r, s in zip(rng, (xs, ws, ys)))
    elif kind == "int":
        X, W, dY = (r.integers(-3, 4, size=s).astype(np.float32) for r, s in zip(rng, (xs, ws, ys)))
    else:
        raise ValueError(kind)
    return X, W.astype(np.float32), dY

