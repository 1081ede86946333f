"""CPU oracle for the C-K-S conv-layer operators -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  It never touches the GPU library and shares no code with it.

The arithmetic lives in ``cks_oracle.c`` (plain C, double accumulation; the
textbook operators of Section IV Eq. (1)-(3) with padding, zero insertion and
dilation made explicit).  This module only builds that file with gcc, loads it
with ctypes and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cks_oracle.c")
_LIB = os.path.join(_HERE, "libcks_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile cks_oracle.c -> libcks_oracle.so (gcc -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        geo = [ctypes.c_int] * 11   # N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw
        for name in ("cko_conv_fwd", "cko_deconv", "cko_wgrad"):
            f = getattr(lib, name)
            f.argtypes = [fp, fp, dp] + geo + [ip, ctypes.c_int64]
            f.restype = ctypes.c_int
        lib.cko_brute.argtypes = [fp, fp, fp, dp, dp, dp] + geo
        lib.cko_brute.restype = ctypes.c_int
        lib.cko_filter_transpose.argtypes = [fp, fp] + [ctypes.c_int] * 4
        lib.cko_filter_transpose.restype = ctypes.c_int
        lib.cko_kernel_split.argtypes = [fp, fp] + [ctypes.c_int] * 6
        lib.cko_kernel_split.restype = ctypes.c_int
        lib.cko_mac_counts.argtypes = [ip] + geo
        lib.cko_mac_counts.restype = ctypes.c_int
        lib.cko_num_threads.argtypes = []
        lib.cko_num_threads.restype = ctypes.c_int
        lib.cko_out_dim.argtypes = [ctypes.c_int] * 4
        lib.cko_out_dim.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.shape != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), a.shape))
    return a


def _fptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _sample(sample):
    if sample is None:
        return None, None, 0
    s = np.ascontiguousarray(sample, dtype=np.int64).ravel()
    return s, s.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), s.size


def pair(v):
    """Stride or padding as (vertical, horizontal): an int applies to both axes
    (Table I writes them as <sh sw> and <ph pw>)."""
    if isinstance(v, (tuple, list)):
        a, b = v
        return int(a), int(b)
    return int(v), int(v)


def out_dim(I, F, s, p):
    """floor((I + 2p - F)/s) + 1."""
    return _load().cko_out_dim(I, F, s, p)


def _check(rc):
    if rc != 0:
        raise ValueError("oracle rejected the geometry (code %d)" % rc)


def conv_fwd(X, W, stride, padding, sample=None):
    """Eq. (1): Y[N,OH,OW,OC] (float64) from X[N,IH,IW,IC], W[OC,FH,FW,IC].

    With ``sample`` (flat indices into Y) only those elements are returned."""
    N, IH, IW, IC = X.shape
    OC, FH, FW, _ = W.shape
    X = _f32(X, (N, IH, IW, IC)); W = _f32(W, (OC, FH, FW, IC))
    lib = _load()
    (sh, sw), (ph, pw) = pair(stride), pair(padding)
    OH, OW = out_dim(IH, FH, sh, ph), out_dim(IW, FW, sw, pw)
    s, sp, ns = _sample(sample)
    out = np.empty(ns if s is not None else (N, OH, OW, OC), dtype=np.float64)
    _check(lib.cko_conv_fwd(_fptr(X), _fptr(W), _dptr(out), N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, sp, ns))
    return out


def deconv(dY, W, IH, IW, stride, padding, sample=None):
    """Eq. (2): dX[N,IH,IW,IC] (float64) from dY[N,OH,OW,OC], W[OC,FH,FW,IC]."""
    OC, FH, FW, IC = W.shape
    N = dY.shape[0]
    (sh, sw), (ph, pw) = pair(stride), pair(padding)
    OH, OW = out_dim(IH, FH, sh, ph), out_dim(IW, FW, sw, pw)
    dY = _f32(dY, (N, OH, OW, OC)); W = _f32(W, (OC, FH, FW, IC))
    lib = _load()
    s, sp, ns = _sample(sample)
    out = np.empty(ns if s is not None else (N, IH, IW, IC), dtype=np.float64)
    _check(lib.cko_deconv(_fptr(dY), _fptr(W), _dptr(out), N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, sp, ns))
    return out


def wgrad(X, dY, FH, FW, stride, padding, sample=None):
    """Eq. (3): dW[OC,FH,FW,IC] (float64) from X[N,IH,IW,IC], dY[N,OH,OW,OC]."""
    N, IH, IW, IC = X.shape
    OC = dY.shape[3]
    (sh, sw), (ph, pw) = pair(stride), pair(padding)
    OH, OW = out_dim(IH, FH, sh, ph), out_dim(IW, FW, sw, pw)
    X = _f32(X, (N, IH, IW, IC)); dY = _f32(dY, (N, OH, OW, OC))
    lib = _load()
    s, sp, ns = _sample(sample)
    out = np.empty(ns if s is not None else (OC, FH, FW, IC), dtype=np.float64)
    _check(lib.cko_wgrad(_fptr(X), _fptr(dY), _dptr(out), N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, sp, ns))
    return out


def brute(X, W, dY, stride, padding):
    """7-deep scatter loop; returns (Y, dX, dW) as float64.  Tiny inputs only."""
    N, IH, IW, IC = X.shape
    OC, FH, FW, _ = W.shape
    (sh, sw), (ph, pw) = pair(stride), pair(padding)
    OH, OW = out_dim(IH, FH, sh, ph), out_dim(IW, FW, sw, pw)
    X = _f32(X, (N, IH, IW, IC)); W = _f32(W, (OC, FH, FW, IC)); dY = _f32(dY, (N, OH, OW, OC))
    Y = np.empty((N, OH, OW, OC)); dX = np.empty((N, IH, IW, IC)); dW = np.empty((OC, FH, FW, IC))
    _check(_load().cko_brute(_fptr(X), _fptr(W), _fptr(dY), _dptr(Y), _dptr(dX), _dptr(dW),
                             N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw))
    return Y, dX, dW


def filter_transpose(W):
    """Section IV.A: W[OC,FH,FW,IC] -> [FH,FW,IC,OC] (float32)."""
    OC, FH, FW, IC = W.shape
    W = _f32(W, (OC, FH, FW, IC))
    out = np.empty((FH, FW, IC, OC), dtype=np.float32)
    _check(_load().cko_filter_transpose(_fptr(W), _fptr(out), OC, FH, FW, IC))
    return out


def kernel_split(W, stride):
    """Algorithm 2 Stage 1 in the paper's layout C[sh,sw,OC,ceil(FH/sh),ceil(FW/sw),IC] (float32)."""
    OC, FH, FW, IC = W.shape
    W = _f32(W, (OC, FH, FW, IC))
    sh, sw = pair(stride)
    out = np.empty((sh, sw, OC, -(-FH // sh), -(-FW // sw), IC), dtype=np.float32)
    _check(_load().cko_kernel_split(_fptr(W), _fptr(out), OC, FH, FW, IC, sh, sw))
    return out


def mac_counts(N, IC, IH, IW, OC, FH, FW, stride, padding):
    """dict(dense, useful, nominal_deconv, nominal_dilated) in multiply-adds, by enumeration."""
    c = np.zeros(4, dtype=np.int64)
    (sh, sw), (ph, pw) = pair(stride), pair(padding)
    _check(_load().cko_mac_counts(c.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                  N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw))
    return dict(dense=int(c[0]), useful=int(c[1]), nominal_deconv=int(c[2]), nominal_dilated=int(c[3]))


def num_threads():
    """OpenMP threads the operators run on."""
    return _load().cko_num_threads()
