"""Thin Python binding over libcks.so (include/cks.h): argument marshalling only.

Every function has the name of the C entry point it calls.  Tensors are
contiguous float32 torch tensors on a ROCm device; PyTorch supplies device
memory and the current stream, all arithmetic happens in the library's kernels.
There is no fallback: if libcks.so is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcks.so")
_lib = None

CKS_OK, CKS_ERR_NULL, CKS_ERR_SHAPE, CKS_ERR_WORKSPACE, CKS_ERR_HIP, CKS_ERR_UNSUPPORTED, CKS_ERR_SCRATCH = 0, -1, -2, -3, -4, -5, -6
CKS_STATIC_SCRATCH_BYTES = 32 << 20
(CKS_OP_CONV2D_FWD, CKS_OP_DECONV2D, CKS_OP_DILATED_CONV2D_WGRAD, CKS_OP_KERNEL_SPLIT, CKS_OP_DECONV2D_PRESPLIT,
 CKS_OP_FILTER_TRANSPOSE, CKS_OP_WGRAD_PARTIALS, CKS_OP_REDUCE_PARTIALS, CKS_OP_CONV2D_FWD_TRANSPOSED,
 CKS_OP_CONV2D_FWD_UNTRIMMED, CKS_OP_DECONV2D_UNTRIMMED, CKS_OP_WGRAD_UNTRIMMED) = range(12)

_GEO = [ctypes.c_int] * 9
_GEO_HW = [ctypes.c_int] * 11   # N, C, H, W, OC, FH, FW, sh, sw, ph, pw
_OP_TAIL = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_PROTOTYPES = {
    "cks_out_dims_hw": ([ctypes.c_int] * 8 + [ctypes.POINTER(ctypes.c_int)] * 2, ctypes.c_int),
    "cks_useful_macs_hw": (_GEO_HW, ctypes.c_int64),
    "cks_conv2d_fwd_workspace_hw": (_GEO_HW, ctypes.c_size_t),
    "cks_deconv2d_workspace_hw": (_GEO_HW, ctypes.c_size_t),
    "cks_dilated_conv2d_wgrad_workspace_hw": (_GEO_HW, ctypes.c_size_t),
    "cks_conv2d_fwd_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + _OP_TAIL, ctypes.c_int),
    "cks_deconv2d_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + _OP_TAIL, ctypes.c_int),
    "cks_dilated_conv2d_wgrad_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + _OP_TAIL, ctypes.c_int),
    "cks_out_dims": ([ctypes.c_int] * 6 + [ctypes.POINTER(ctypes.c_int)] * 2, ctypes.c_int),
    "cks_useful_macs": (_GEO, ctypes.c_int64),
    "cks_conv2d_fwd_workspace": (_GEO, ctypes.c_size_t),
    "cks_deconv2d_workspace": (_GEO, ctypes.c_size_t),
    "cks_dilated_conv2d_wgrad_workspace": (_GEO, ctypes.c_size_t),
    "cks_dilated_conv2d_wgrad_segments": (_GEO, ctypes.c_int),
    "cks_conv2d_fwd": ([ctypes.c_void_p] * 3 + _GEO + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p], ctypes.c_int),
    "cks_deconv2d": ([ctypes.c_void_p] * 3 + _GEO + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p], ctypes.c_int),
    "cks_dilated_conv2d_wgrad": ([ctypes.c_void_p] * 3 + _GEO + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p], ctypes.c_int),
    "cks_dilated_conv2d_wgrad_partials": ([ctypes.c_void_p] * 3 + _GEO + [ctypes.c_void_p], ctypes.c_int),
    "cks_reduce_partials": ([ctypes.c_void_p] * 2 + [ctypes.c_int64, ctypes.c_int, ctypes.c_void_p], ctypes.c_int),
    "cks_kernel_split_bytes": ([ctypes.c_int] * 5, ctypes.c_size_t),
    "cks_kernel_split": ([ctypes.c_void_p] * 2 + [ctypes.c_int] * 5 + [ctypes.c_void_p], ctypes.c_int),
    "cks_deconv2d_presplit": ([ctypes.c_void_p] * 3 + _GEO + [ctypes.c_void_p], ctypes.c_int),
    "cks_filter_transpose": ([ctypes.c_void_p] * 2 + [ctypes.c_int] * 4 + [ctypes.c_void_p], ctypes.c_int),
    "cks_kernel_split_bytes_hw": ([ctypes.c_int] * 6, ctypes.c_size_t),
    "cks_kernel_split_hw": ([ctypes.c_void_p] * 2 + [ctypes.c_int] * 6 + [ctypes.c_void_p], ctypes.c_int),
    "cks_deconv2d_presplit_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + [ctypes.c_void_p], ctypes.c_int),
    "cks_dilated_conv2d_wgrad_segments_hw": (_GEO_HW, ctypes.c_int),
    "cks_dilated_conv2d_wgrad_partials_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + [ctypes.c_void_p], ctypes.c_int),
    "cks_dilated_conv2d_wgrad_noalloc_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + [ctypes.c_void_p], ctypes.c_int),
    "cks_conv2d_fwd_transposed": ([ctypes.c_void_p] * 3 + _GEO + [ctypes.c_void_p], ctypes.c_int),
    "cks_conv2d_fwd_transposed_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + [ctypes.c_void_p], ctypes.c_int),
    "cks_conv2d_fwd_untrimmed_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + [ctypes.c_void_p], ctypes.c_int),
    "cks_deconv2d_untrimmed_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + [ctypes.c_void_p], ctypes.c_int),
    "cks_dilated_conv2d_wgrad_untrimmed_hw": ([ctypes.c_void_p] * 3 + _GEO_HW + _OP_TAIL, ctypes.c_int),
    "cks_plan_hw": ([ctypes.c_int] + _GEO_HW + [ctypes.c_uint, ctypes.c_char_p, ctypes.c_size_t], ctypes.c_int),
    "cks_strerror": ([ctypes.c_int], ctypes.c_char_p),
    "cks_last_hip_error": ([], ctypes.c_int),
}
EXPORTS = tuple(_PROTOTYPES)


class CksError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().cks_strerror(status).decode()
        if status == CKS_ERR_HIP:
            msg += " [hipError_t %d]" % lib().cks_last_hip_error()
        super().__init__("%s: %s (status %d)" % (where, msg, status))


def lib():
    """Load libcks.so (built in-tree by paper_2306_15951_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libcks.so is not built: run `python -m paper_2306_15951_amd.build` "
                              "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        for name, (argtypes, restype) in _PROTOTYPES.items():
            f = getattr(L, name)
            f.argtypes = argtypes
            f.restype = restype
        _lib = L
    return _lib


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, name, shape=None):
    import torch

    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous float32 tensor on the GPU" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return ctypes.c_void_p(t.data_ptr())


def _ws(ws):
    import torch

    if ws is None:
        return None, 0
    if not (isinstance(ws, torch.Tensor) and ws.is_cuda and ws.is_contiguous()):
        raise TypeError("workspace must be a contiguous tensor on the GPU")
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def _check(rc, where):
    if rc != CKS_OK:
        raise CksError(rc, where)


def cks_out_dims(H, W, FH, FW, stride, padding):
    oh, ow = ctypes.c_int(), ctypes.c_int()
    _check(lib().cks_out_dims(H, W, FH, FW, stride, padding, ctypes.byref(oh), ctypes.byref(ow)), "cks_out_dims")
    return oh.value, ow.value


def cks_useful_macs(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_useful_macs(N, C, H, W, OC, FH, FW, stride, padding)


def cks_conv2d_fwd_workspace(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_conv2d_fwd_workspace(N, C, H, W, OC, FH, FW, stride, padding)


def cks_deconv2d_workspace(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_deconv2d_workspace(N, C, H, W, OC, FH, FW, stride, padding)


def cks_dilated_conv2d_wgrad_workspace(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_dilated_conv2d_wgrad_workspace(N, C, H, W, OC, FH, FW, stride, padding)


def cks_dilated_conv2d_wgrad_segments(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_dilated_conv2d_wgrad_segments(N, C, H, W, OC, FH, FW, stride, padding)


def cks_kernel_split_bytes(C, OC, FH, FW, stride):
    return lib().cks_kernel_split_bytes(C, OC, FH, FW, stride)


def cks_conv2d_fwd(X, Wt, Y, stride, padding, ws=None):
    """Y[N,OH,OW,OC] <- ConvV2(X[N,H,W,C], Wt[OC,FH,FW,C]) on the current stream."""
    N, H, W, C = X.shape
    OC, FH, FW, _ = Wt.shape
    OH, OW = cks_out_dims(H, W, FH, FW, stride, padding)
    wp, wb = _ws(ws)
    _check(lib().cks_conv2d_fwd(_ptr(X, "X"), _ptr(Wt, "Wt", (OC, FH, FW, C)), _ptr(Y, "Y", (N, OH, OW, OC)),
                                N, C, H, W, OC, FH, FW, stride, padding, wp, wb, _stream()), "cks_conv2d_fwd")
    return Y


def cks_deconv2d(dY, Wt, dX, stride, padding, ws):
    """dX[N,H,W,C] <- KS-deconv-V2(dY[N,OH,OW,OC], Wt[OC,FH,FW,C]); H, W are taken from dX."""
    N, H, W, C = dX.shape
    OC, FH, FW, _ = Wt.shape
    OH, OW = cks_out_dims(H, W, FH, FW, stride, padding)
    wp, wb = _ws(ws)
    _check(lib().cks_deconv2d(_ptr(dY, "dY", (N, OH, OW, OC)), _ptr(Wt, "Wt", (OC, FH, FW, C)), _ptr(dX, "dX"),
                              N, C, H, W, OC, FH, FW, stride, padding, wp, wb, _stream()), "cks_deconv2d")
    return dX


def cks_dilated_conv2d_wgrad(X, dY, dW, stride, padding, ws):
    """dW[OC,FH,FW,C] <- Sk-dilated-V2(X[N,H,W,C], dY[N,OH,OW,OC])."""
    N, H, W, C = X.shape
    OC, FH, FW, _ = dW.shape
    OH, OW = cks_out_dims(H, W, FH, FW, stride, padding)
    wp, wb = _ws(ws)
    _check(lib().cks_dilated_conv2d_wgrad(_ptr(X, "X"), _ptr(dY, "dY", (N, OH, OW, OC)), _ptr(dW, "dW", (OC, FH, FW, C)),
                                          N, C, H, W, OC, FH, FW, stride, padding, wp, wb, _stream()),
           "cks_dilated_conv2d_wgrad")
    return dW


def cks_kernel_split(Wt, Cs, stride):
    """Cs[s,s,C,ceil(FH/s),ceil(FW/s),OC] <- Stage 1 of KS-deconv on Wt[OC,FH,FW,C]."""
    OC, FH, FW, C = Wt.shape
    s = stride
    _check(lib().cks_kernel_split(_ptr(Wt, "Wt"), _ptr(Cs, "Cs", (s, s, C, -(-FH // s), -(-FW // s), OC)),
                                  C, OC, FH, FW, s, _stream()), "cks_kernel_split")
    return Cs


def cks_deconv2d_presplit(dY, Cs, dX, FH, FW, stride, padding):
    N, H, W, C = dX.shape
    OC = dY.shape[3]
    s = stride
    OH, OW = cks_out_dims(H, W, FH, FW, stride, padding)
    _check(lib().cks_deconv2d_presplit(_ptr(dY, "dY", (N, OH, OW, OC)),
                                       _ptr(Cs, "Cs", (s, s, C, -(-FH // s), -(-FW // s), OC)), _ptr(dX, "dX"),
                                       N, C, H, W, OC, FH, FW, stride, padding, _stream()), "cks_deconv2d_presplit")
    return dX


def cks_filter_transpose(Wt, Wout):
    OC, FH, FW, C = Wt.shape
    _check(lib().cks_filter_transpose(_ptr(Wt, "Wt"), _ptr(Wout, "Wout", (FH, FW, C, OC)), C, OC, FH, FW, _stream()),
           "cks_filter_transpose")
    return Wout


def cks_dilated_conv2d_wgrad_partials(X, dY, part, FH, FW, stride, padding):
    """part[G_Z,OC,FH,FW,C] <- per-segment partial filter gradients."""
    N, H, W, C = X.shape
    OC = dY.shape[3]
    OH, OW = cks_out_dims(H, W, FH, FW, stride, padding)
    gz = cks_dilated_conv2d_wgrad_segments(N, C, H, W, OC, FH, FW, stride, padding)
    _check(lib().cks_dilated_conv2d_wgrad_partials(_ptr(X, "X"), _ptr(dY, "dY", (N, OH, OW, OC)),
                                                   _ptr(part, "part", (gz, OC, FH, FW, C)),
                                                   N, C, H, W, OC, FH, FW, stride, padding, _stream()),
           "cks_dilated_conv2d_wgrad_partials")
    return part


def cks_reduce_partials(part, dW):
    _check(lib().cks_reduce_partials(_ptr(part, "part"), _ptr(dW, "dW", tuple(part.shape[1:])),
                                     dW.numel(), part.shape[0], _stream()), "cks_reduce_partials")
    return dW


# ---- stride and padding per axis: stride = (sh, sw), padding = (ph, pw)

def cks_out_dims_hw(H, W, FH, FW, stride, padding):
    (sh, sw), (ph, pw) = stride, padding
    oh, ow = ctypes.c_int(), ctypes.c_int()
    _check(lib().cks_out_dims_hw(H, W, FH, FW, sh, sw, ph, pw, ctypes.byref(oh), ctypes.byref(ow)), "cks_out_dims_hw")
    return oh.value, ow.value


def cks_useful_macs_hw(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_useful_macs_hw(N, C, H, W, OC, FH, FW, *stride, *padding)


def cks_conv2d_fwd_workspace_hw(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_conv2d_fwd_workspace_hw(N, C, H, W, OC, FH, FW, *stride, *padding)


def cks_deconv2d_workspace_hw(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_deconv2d_workspace_hw(N, C, H, W, OC, FH, FW, *stride, *padding)


def cks_dilated_conv2d_wgrad_workspace_hw(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_dilated_conv2d_wgrad_workspace_hw(N, C, H, W, OC, FH, FW, *stride, *padding)


def cks_conv2d_fwd_hw(X, Wt, Y, stride, padding, ws=None):
    N, H, W, C = X.shape
    OC, FH, FW, _ = Wt.shape
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    wp, wb = _ws(ws)
    _check(lib().cks_conv2d_fwd_hw(_ptr(X, "X"), _ptr(Wt, "Wt", (OC, FH, FW, C)), _ptr(Y, "Y", (N, OH, OW, OC)),
                                   N, C, H, W, OC, FH, FW, *stride, *padding, wp, wb, _stream()), "cks_conv2d_fwd_hw")
    return Y


def cks_deconv2d_hw(dY, Wt, dX, stride, padding, ws):
    N, H, W, C = dX.shape
    OC, FH, FW, _ = Wt.shape
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    wp, wb = _ws(ws)
    _check(lib().cks_deconv2d_hw(_ptr(dY, "dY", (N, OH, OW, OC)), _ptr(Wt, "Wt", (OC, FH, FW, C)), _ptr(dX, "dX"),
                                 N, C, H, W, OC, FH, FW, *stride, *padding, wp, wb, _stream()), "cks_deconv2d_hw")
    return dX


def cks_dilated_conv2d_wgrad_hw(X, dY, dW, stride, padding, ws):
    N, H, W, C = X.shape
    OC, FH, FW, _ = dW.shape
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    wp, wb = _ws(ws)
    _check(lib().cks_dilated_conv2d_wgrad_hw(_ptr(X, "X"), _ptr(dY, "dY", (N, OH, OW, OC)), _ptr(dW, "dW", (OC, FH, FW, C)),
                                             N, C, H, W, OC, FH, FW, *stride, *padding, wp, wb, _stream()),
           "cks_dilated_conv2d_wgrad_hw")
    return dW


def cks_kernel_split_bytes_hw(C, OC, FH, FW, stride):
    return lib().cks_kernel_split_bytes_hw(C, OC, FH, FW, *stride)


def cks_kernel_split_hw(Wt, Cs, stride):
    """Cs[sh,sw,C,ceil(FH/sh),ceil(FW/sw),OC] <- Stage 1 of KS-deconv on Wt[OC,FH,FW,C]."""
    OC, FH, FW, C = Wt.shape
    sh, sw = stride
    _check(lib().cks_kernel_split_hw(_ptr(Wt, "Wt"), _ptr(Cs, "Cs", (sh, sw, C, -(-FH // sh), -(-FW // sw), OC)),
                                     C, OC, FH, FW, sh, sw, _stream()), "cks_kernel_split_hw")
    return Cs


def cks_deconv2d_presplit_hw(dY, Cs, dX, FH, FW, stride, padding):
    N, H, W, C = dX.shape
    OC = dY.shape[3]
    sh, sw = stride
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    _check(lib().cks_deconv2d_presplit_hw(_ptr(dY, "dY", (N, OH, OW, OC)),
                                          _ptr(Cs, "Cs", (sh, sw, C, -(-FH // sh), -(-FW // sw), OC)), _ptr(dX, "dX"),
                                          N, C, H, W, OC, FH, FW, *stride, *padding, _stream()), "cks_deconv2d_presplit_hw")
    return dX


def cks_dilated_conv2d_wgrad_segments_hw(N, C, H, W, OC, FH, FW, stride, padding):
    return lib().cks_dilated_conv2d_wgrad_segments_hw(N, C, H, W, OC, FH, FW, *stride, *padding)


def cks_dilated_conv2d_wgrad_partials_hw(X, dY, part, FH, FW, stride, padding):
    N, H, W, C = X.shape
    OC = dY.shape[3]
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    gz = cks_dilated_conv2d_wgrad_segments_hw(N, C, H, W, OC, FH, FW, stride, padding)
    _check(lib().cks_dilated_conv2d_wgrad_partials_hw(_ptr(X, "X"), _ptr(dY, "dY", (N, OH, OW, OC)),
                                                      _ptr(part, "part", (gz, OC, FH, FW, C)),
                                                      N, C, H, W, OC, FH, FW, *stride, *padding, _stream()),
           "cks_dilated_conv2d_wgrad_partials_hw")
    return part


def cks_plan_hw(op, N, C, H, W, OC, FH, FW, stride, padding, only_4byte_aligned=0):
    """The kernels entry point `op` (CKS_OP_*) would enqueue for this geometry and pointer alignment, as a
    list of (kernel name with template arguments, launch shape) pairs.  Host only."""
    buf = ctypes.create_string_buffer(4096)
    _check(lib().cks_plan_hw(op, N, C, H, W, OC, FH, FW, *stride, *padding, only_4byte_aligned, buf, len(buf)), "cks_plan_hw")
    out = []
    for line in buf.value.decode().splitlines():
        name, _, shape = line.partition(" [")
        out.append((name, "[" + shape))
    return out


def cks_dilated_conv2d_wgrad_noalloc_hw(X, dY, dW, stride, padding):
    """dW <- Sk-dilated-V2(X, dY) with the partial sums in the library's static scratch array."""
    N, H, W, C = X.shape
    OC, FH, FW, _ = dW.shape
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    _check(lib().cks_dilated_conv2d_wgrad_noalloc_hw(_ptr(X, "X"), _ptr(dY, "dY", (N, OH, OW, OC)), _ptr(dW, "dW", (OC, FH, FW, C)),
                                                     N, C, H, W, OC, FH, FW, *stride, *padding, _stream()),
           "cks_dilated_conv2d_wgrad_noalloc_hw")
    return dW


def cks_conv2d_fwd_transposed(X, Wtt, Y, stride, padding):
    """Y[N,OH,OW,OC] <- ConvV2(X[N,H,W,C], Wtt[FH,FW,C,OC]), the filter as cks_filter_transpose writes it."""
    N, H, W, C = X.shape
    FH, FW, _, OC = Wtt.shape
    OH, OW = cks_out_dims(H, W, FH, FW, stride, padding)
    _check(lib().cks_conv2d_fwd_transposed(_ptr(X, "X"), _ptr(Wtt, "Wtt", (FH, FW, C, OC)), _ptr(Y, "Y", (N, OH, OW, OC)),
                                           N, C, H, W, OC, FH, FW, stride, padding, _stream()), "cks_conv2d_fwd_transposed")
    return Y


def cks_conv2d_fwd_transposed_hw(X, Wtt, Y, stride, padding):
    N, H, W, C = X.shape
    FH, FW, _, OC = Wtt.shape
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    _check(lib().cks_conv2d_fwd_transposed_hw(_ptr(X, "X"), _ptr(Wtt, "Wtt", (FH, FW, C, OC)), _ptr(Y, "Y", (N, OH, OW, OC)),
                                              N, C, H, W, OC, FH, FW, *stride, *padding, _stream()), "cks_conv2d_fwd_transposed_hw")
    return Y


# ---- trimming switched off (ablation): stride = (sh, sw), padding = (ph, pw)

def cks_conv2d_fwd_untrimmed_hw(X, Wt, Y, stride, padding):
    N, H, W, C = X.shape
    OC, FH, FW, _ = Wt.shape
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    _check(lib().cks_conv2d_fwd_untrimmed_hw(_ptr(X, "X"), _ptr(Wt, "Wt", (OC, FH, FW, C)), _ptr(Y, "Y", (N, OH, OW, OC)),
                                             N, C, H, W, OC, FH, FW, *stride, *padding, _stream()), "cks_conv2d_fwd_untrimmed_hw")
    return Y


def cks_deconv2d_untrimmed_hw(dY, Wt, dX, stride, padding):
    N, H, W, C = dX.shape
    OC, FH, FW, _ = Wt.shape
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    _check(lib().cks_deconv2d_untrimmed_hw(_ptr(dY, "dY", (N, OH, OW, OC)), _ptr(Wt, "Wt", (OC, FH, FW, C)), _ptr(dX, "dX"),
                                           N, C, H, W, OC, FH, FW, *stride, *padding, _stream()), "cks_deconv2d_untrimmed_hw")
    return dX


def cks_dilated_conv2d_wgrad_untrimmed_hw(X, dY, dW, stride, padding, ws):
    N, H, W, C = X.shape
    OC, FH, FW, _ = dW.shape
    OH, OW = cks_out_dims_hw(H, W, FH, FW, stride, padding)
    wp, wb = _ws(ws)
    _check(lib().cks_dilated_conv2d_wgrad_untrimmed_hw(_ptr(X, "X"), _ptr(dY, "dY", (N, OH, OW, OC)), _ptr(dW, "dW", (OC, FH, FW, C)),
                                                       N, C, H, W, OC, FH, FW, *stride, *padding, wp, wb, _stream()),
           "cks_dilated_conv2d_wgrad_untrimmed_hw")
    return dW
