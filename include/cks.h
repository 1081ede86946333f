/*
 * cks.h -- C ABI of the C-K-S convolution-layer operators for AMD MI355X (gfx950).
 *
 * The three operators of a 2-D convolutional layer (paper: Section IV,
 * Eq. (1)-(3)), computed without ever multiplying a padded or inserted zero:
 *
 *   cks_conv2d_fwd            Y  = conv2D(X, W)             ConvV2, Algorithm 1
 *   cks_deconv2d              dX = deconv2D(dY, rot180(W))  KS-deconv-V2, Algorithm 2 / 2B
 *   cks_dilated_conv2d_wgrad  dW = dilated_conv2D(X, dY)    Sk-dilated-V2, Algorithm 3B
 *
 * Tensors (Section IV, paragraph before Eq. (1); notation of Table I).  All are
 * dense, row-major, float32, in DEVICE memory of the current HIP device:
 *
 *   X, dX   [N][H][W][C]          input feature maps / their gradient   (C = I_C)
 *   Wt, dW  [OC][FH][FW][C]       filters / their gradient
 *   Y, dY   [N][OH][OW][OC]       output feature maps / their gradient
 *   OH = floor((H + 2*padding - FH) / stride) + 1, OW likewise (cks_out_dims).
 *
 * Common arguments: N batch, C input channels, H x W the size of X (always the
 * larger, input side -- also for cks_deconv2d, whose output size cannot be
 * recovered from OH when (H + 2*padding - FH) is not a multiple of stride),
 * OC output channels, FH x FW filter size, stride and padding applied to both
 * axes (the *_hw entry points further down take them per axis).
 *
 * Ownership: the caller owns every buffer, workspaces included; the library
 * never allocates or frees device memory and keeps no device state.  Inputs are
 * never written; outputs are completely overwritten (elements whose trimmed
 * range is empty receive +0.0); inputs, outputs and workspace must not overlap.
 * Pointers must be 4-byte aligned; 16-byte aligned pointers with C and OC
 * multiples of 4 take the vector-load path.
 *
 * Execution: asynchronous on `stream` (a hipStream_t passed as void*, NULL is
 * the default stream).  Calls on different streams are independent.
 *
 * Errors: every function returns a cks_status (0 = success, negative = error).
 * On error nothing has been enqueued.  CKS_ERR_HIP means a HIP call failed;
 * cks_last_hip_error() returns that hipError_t value (per calling thread).
 */
#ifndef CKS_H
#define CKS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CKS_OK = 0,
    CKS_ERR_NULL = -1,        /* a required pointer is NULL */
    CKS_ERR_SHAPE = -2,       /* dimension <= 0, stride < 1, padding < 0, filter larger
                                 than the padded input, or a tensor of 2^31 or more elements */
    CKS_ERR_WORKSPACE = -3,   /* workspace NULL or smaller than the *_workspace() size */
    CKS_ERR_HIP = -4,         /* a HIP runtime call failed; see cks_last_hip_error() */
    CKS_ERR_UNSUPPORTED = -5, /* valid geometry that this entry point has no kernel for
                                 (cks_conv2d_fwd_transposed, the *_untrimmed entry points;
                                 unknown op of cks_plan_hw) */
    CKS_ERR_SCRATCH = -6      /* cks_dilated_conv2d_wgrad_noalloc_hw: the call needs more than
                                 CKS_STATIC_SCRATCH_BYTES of scratch memory */
} cks_status;

/* Output size of Eq. (1).  OH, OW may be NULL.  Returns CKS_ERR_SHAPE if the
 * padded input is smaller than the filter. */
int cks_out_dims(int H, int W, int FH, int FW, int stride, int padding, int *OH, int *OW);

/* Multiply-adds that touch no padded / inserted zero: N*C*OC*S_h*S_w with
 * S_h = sum over oh of (fh_e - fh_s) of Algorithm 1, S_w likewise.  All three
 * operators of a layer perform exactly this many.  -1 on bad geometry. */
int64_t cks_useful_macs(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding);

/* Bytes of workspace each operator needs for this geometry (0 = none; then
 * ws may be NULL).  Returns 0 on bad geometry as well. */
size_t cks_conv2d_fwd_workspace(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding);
size_t cks_deconv2d_workspace(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding);
size_t cks_dilated_conv2d_wgrad_workspace(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding);

/* ConvV2 (Section IV.A, Algorithm 1).  For every output position the filter is
 * cut to [fh_s,fh_e) x [fw_s,fw_e), the taps that lie over real input:
 *   Y[n,oh,ow,oc] = sum_{fh,fw in the trimmed range, c} X[n,oh*s-p+fh,ow*s-p+fw,c] * Wt[oc,fh,fw,c]
 * X [N,H,W,C] in, Wt [OC,FH,FW,C] in, Y [N,OH,OW,OC] out. */
int cks_conv2d_fwd(const float *X, const float *Wt, float *Y,
                   int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                   void *ws, size_t ws_bytes, void *stream);

/* KS-deconv-V2 (Section IV.B; Algorithm 2 Stage 1, Algorithm 2B Stage 2&3).
 * The sub-kernels of Stage 1 are either taken straight from Wt (sub-kernel
 * (y,x)'s tap (ch,cw) is filter tap (y + (CH-1-ch) s, x + (CW-1-cw) s); used when
 * OC is a multiple of 32, C a multiple of 4 and dY, Wt are 16-byte aligned), or
 * written to the workspace by cks_kernel_split and consumed by
 * cks_deconv2d_presplit.  Layers with C < 8 and OC <= 64 run Stage 2&3
 * tap-stationary and compose the result in on-chip memory; they use the
 * workspace for the rows and columns neighbouring workgroups share.
 * cks_deconv2d_workspace is what the call needs whatever the alignment of its
 * pointers; a call whose sub-kernels are read from Wt in place uses no
 * workspace and accepts ws = NULL, any other call returns CKS_ERR_WORKSPACE
 * without it.  The result does not depend on which variant runs beyond
 * rounding, and every variant is reproducible bit for bit.
 * dY [N,OH,OW,OC] in, Wt [OC,FH,FW,C] in, dX [N,H,W,C] out. */
int cks_deconv2d(const float *dY, const float *Wt, float *dX,
                 int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                 void *ws, size_t ws_bytes, void *stream);

/* Sk-dilated-V2 (Section IV.C, Algorithm 3B) with the split of the contraction
 * axis G_K = N*OH*OW into segments and a final aggregation (Section IV.C,
 * paragraph on map-reduce).  dY is read as it is, X with a leaping step equal
 * to the stride; per filter tap only the (oh,ow) whose X element exists are
 * visited.  The partial sums live in the workspace and are added in a fixed
 * order, so results are reproducible bit for bit.
 * X [N,H,W,C] in, dY [N,OH,OW,OC] in, dW [OC,FH,FW,C] out. */
int cks_dilated_conv2d_wgrad(const float *X, const float *dY, float *dW,
                             int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                             void *ws, size_t ws_bytes, void *stream);

/* ---- stride and padding given per axis ----
 *
 * Table I writes the strides as <sh sw> and the padding as <ph pw>, and
 * Algorithms 1-3B are printed with both.  The *_hw entry points take them in
 * that order: sh, ph act on the H axis (rows), sw, pw on the W axis (columns);
 * OH = floor((H + 2*ph - FH) / sh) + 1, OW = floor((W + 2*pw - FW) / sw) + 1.
 * Everything else -- tensors, layouts, ownership, execution, errors, the role
 * of the workspace -- is as for the entry point of the same name without the
 * suffix, which is the special case sh = sw = stride, ph = pw = padding (and
 * calls it).  CKS_ERR_SHAPE if sh or sw < 1, ph or pw < 0, or the padded input
 * is smaller than the filter on either axis.  KS-deconv then splits the
 * filter into sh*sw sub-kernels; sub-kernel (y,x), y < sh, x < sw, has
 * ceil((FH-y)/sh) x ceil((FW-x)/sw) taps (Section IV.B with the two strides
 * kept apart), and Sk-dilated leaps sh rows and sw columns (Section IV.C).
 * Geometries whose two axes differ always run the general kernels. */
int cks_out_dims_hw(int H, int W, int FH, int FW, int sh, int sw, int ph, int pw, int *OH, int *OW);
int64_t cks_useful_macs_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw);
size_t cks_conv2d_fwd_workspace_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw);
size_t cks_deconv2d_workspace_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw);
size_t cks_dilated_conv2d_wgrad_workspace_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw);
/* ConvV2, Algorithm 1: X [N,H,W,C] in, Wt [OC,FH,FW,C] in, Y [N,OH,OW,OC] out. */
int cks_conv2d_fwd_hw(const float *X, const float *Wt, float *Y,
                      int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                      void *ws, size_t ws_bytes, void *stream);
/* KS-deconv-V2, Algorithms 2 / 2B: dY [N,OH,OW,OC] in, Wt [OC,FH,FW,C] in, dX [N,H,W,C] out;
 * ws must hold cks_deconv2d_workspace_hw bytes. */
int cks_deconv2d_hw(const float *dY, const float *Wt, float *dX,
                    int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                    void *ws, size_t ws_bytes, void *stream);
/* Sk-dilated-V2, Algorithm 3B: X [N,H,W,C] in, dY [N,OH,OW,OC] in, dW [OC,FH,FW,C] out;
 * ws must hold cks_dilated_conv2d_wgrad_workspace_hw bytes. */
int cks_dilated_conv2d_wgrad_hw(const float *X, const float *dY, float *dW,
                                int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                void *ws, size_t ws_bytes, void *stream);

/* ---- for callers that cannot allocate ----
 *
 * cks_dilated_conv2d_wgrad_hw for code that must not call hipMalloc and has no
 * workspace to hand over: work recorded under HIP graph capture, tight serving
 * or training loops, harnesses that forbid allocation.  Same kernels, same
 * number of segments and therefore the same bits in dW; the partial sums of
 * the segments go to a scratch array of CKS_STATIC_SCRATCH_BYTES that is part
 * of the library's device code: every GPU the library runs on holds its own
 * copy from the first use until the process ends.  The call allocates and
 * frees nothing (the first call on a device looks the array's address up).
 * X, dY in, dW out as for cks_dilated_conv2d_wgrad_hw; inputs and output are
 * still the caller's.  Returns CKS_ERR_SCRATCH, with nothing enqueued, if the
 * geometry needs more than CKS_STATIC_SCRATCH_BYTES
 * (cks_dilated_conv2d_wgrad_workspace_hw tells how much).  All calls on one
 * GPU share that GPU's array, which keeps the last call's contents (nothing
 * needs clearing: every partial sum is written before it is read): calls that
 * overlap in time on one GPU -- on different streams, from different threads
 * -- race with each other; calls on one stream are ordered and safe. */
#define CKS_STATIC_SCRATCH_BYTES (32u << 20)
int cks_dilated_conv2d_wgrad_noalloc_hw(const float *X, const float *dY, float *dW,
                                        int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                        void *stream);

/* ---- the stages on their own (what the three calls above are made of) ----
 *
 * Section V.A measures the operators also with "the filter operations done
 * before the loop": cks_kernel_split once, cks_deconv2d_presplit per step.
 * Each stage exists with one stride / padding and, suffixed _hw, with
 * <sh sw>, <ph pw> per axis (Table I), the former calling the latter. */

/* Stage 1 of KS-deconv (Section IV.B, Algorithm 2 Stage 1): rotate the filter
 * by 180 degrees and split it into sh*sw sub-kernels.  Sub-kernel (y,x)
 * holds the taps fh = y + (oph-ch)*sh, fw = x + (opw-cw)*sw with
 * oph = ceil((FH-y)/sh) - 1, opw = ceil((FW-x)/sw) - 1.  The result is the
 * paper's zero-padded 6-D tensor with the two channel axes exchanged, so that
 * the contraction index (ch,cw,oc) of Stage 2 is contiguous:
 *   Cs[sh][sw][C][ceil(FH/sh)][ceil(FW/sw)][OC]
 * cks_kernel_split_bytes gives its size (0 on bad arguments).  Every element
 * of Cs is written.  Wt [OC,FH,FW,C] in, Cs out, both in device memory. */
size_t cks_kernel_split_bytes(int C, int OC, int FH, int FW, int stride);
size_t cks_kernel_split_bytes_hw(int C, int OC, int FH, int FW, int sh, int sw);
int cks_kernel_split(const float *Wt, float *Cs, int C, int OC, int FH, int FW, int stride, void *stream);
int cks_kernel_split_hw(const float *Wt, float *Cs, int C, int OC, int FH, int FW, int sh, int sw, void *stream);

/* Stage 2&3 of KS-deconv-V2 (Algorithm 2B) on an already split filter:
 * dY [N,OH,OW,OC] in, Cs (as written by cks_kernel_split for the same
 * strides) in, dX [N,H,W,C] out.  No workspace. */
int cks_deconv2d_presplit(const float *dY, const float *Cs, float *dX,
                          int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                          void *stream);
int cks_deconv2d_presplit_hw(const float *dY, const float *Cs, float *dX,
                             int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                             void *stream);

/* Filter transposition of Section IV.A (last paragraph):
 * Wt[OC][FH][FW][C] -> Wout[FH][FW][C][OC]. */
int cks_filter_transpose(const float *Wt, float *Wout, int C, int OC, int FH, int FW, void *stream);

/* ConvV2 (Algorithm 1) on the transposed filter, the arrangement Section IV.A
 * describes for large inputs: cks_filter_transpose once (a temporary the caller
 * owns), then this call per step.  X [N,H,W,C] in, Wtt [FH,FW,C,OC] in (as
 * written by cks_filter_transpose), Y [N,OH,OW,OC] out; the same result as
 * cks_conv2d_fwd up to the order of the fp32 sums.  No workspace.  The kernel
 * stages 32-channel chunks of the filter as they lie, so it exists only for
 * C a multiple of 32, OC a multiple of 4 and 16-byte aligned X, Wtt: any other
 * call returns CKS_ERR_UNSUPPORTED with nothing enqueued (cks_conv2d_fwd, which
 * reads the filter in its given layout, serves every geometry). */
int cks_conv2d_fwd_transposed(const float *X, const float *Wtt, float *Y,
                              int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                              void *stream);
int cks_conv2d_fwd_transposed_hw(const float *X, const float *Wtt, float *Y,
                                 int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                 void *stream);

/* Number of segments the contraction axis of cks_dilated_conv2d_wgrad is split
 * into for this geometry (the paper's G_Z); 0 on bad geometry. */
int cks_dilated_conv2d_wgrad_segments(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding);
int cks_dilated_conv2d_wgrad_segments_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw);

/* The "map" half of Sk-dilated-V2 (Section IV.C): segment z of the contraction
 * axis writes its partial filter gradient to part[z], with
 * part [G_Z][OC][FH][FW][C], G_Z = cks_dilated_conv2d_wgrad_segments(...).
 * Every element of part is written. */
int cks_dilated_conv2d_wgrad_partials(const float *X, const float *dY, float *part,
                                      int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                                      void *stream);
int cks_dilated_conv2d_wgrad_partials_hw(const float *X, const float *dY, float *part,
                                         int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                         void *stream);

/* The "reduce" half: dW[e] = part[0][e] + part[1][e] + ... in that order,
 * for e < elems (= OC*FH*FW*C), segments >= 1. */
int cks_reduce_partials(const float *part, float *dW, int64_t elems, int segments, void *stream);

/* ---- the operators with filter trimming switched off (for the ablation) ----
 *
 * Sections IV.A-IV.C introduce each operator first without trimming -- the plain
 * convolution, KS-deconv (Algorithm 2: kernel split only) and Sk-dilated
 * (Algorithm 3: leaping access only) -- and then its V2 with the filter / range
 * trimmed (Algorithms 1, 2B, 3B).  These entry points run the former through the
 * same kernels, work lists and segment counts as the library's operators: every
 * position (every tap) contracts its whole window, and the cells of the window
 * that lie outside the data are fetched as zeros and multiplied.  Results equal
 * those of the trimmed operators up to the order of the fp32 sums (exactly, on
 * integer-valued inputs).  They exist for the kernels that load their operands
 * straight into LDS only.  Forward and input gradient: C and OC multiples of 32,
 * a tile 64 columns wide (OC >= 48 forward, C >= 48 input gradient), 16-byte
 * aligned tensors.  Filter gradient: N a multiple of 32, C and OC multiples of 4,
 * 16-byte aligned tensors, and a geometry for which the library's own filter
 * gradient takes its general kernel (not the one for small images).  Any other
 * call returns CKS_ERR_UNSUPPORTED with nothing enqueued.  Tensors, H/W convention, stream and
 * (filter gradient) workspace as for cks_conv2d_fwd_hw, cks_deconv2d_hw (no
 * workspace: the filter is read in place) and cks_dilated_conv2d_wgrad_hw. */
int cks_conv2d_fwd_untrimmed_hw(const float *X, const float *Wt, float *Y,
                                int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                void *stream);
int cks_deconv2d_untrimmed_hw(const float *dY, const float *Wt, float *dX,
                              int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                              void *stream);
int cks_dilated_conv2d_wgrad_untrimmed_hw(const float *X, const float *dY, float *dW,
                                          int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                          void *ws, size_t ws_bytes, void *stream);

/* ---- which kernels a call would enqueue (host only, no device is touched) ----
 *
 * Which kernel variant serves a call is a function of the geometry and of the
 * alignment of the pointers (Section IV.E describes the paper's own library
 * choosing between kernels in the same way).  cks_plan_hw runs the code path of
 * the entry point named by `op` up to, but not including, the launches and
 * writes one line per kernel to `text` (host memory, text_bytes long, always
 * terminated):  name<template arguments> [workgroups x threads, lds bytes]
 * Bit i of only_4byte_aligned marks the i-th pointer argument of that entry
 * point (bit 3: the workspace) as 4-byte aligned only; others count as
 * 16-byte aligned.  CKS_OP_REDUCE_PARTIALS is planned for elems = OC*FH*FW*C
 * and the geometry's own number of segments.  Returns CKS_ERR_SHAPE on bad
 * geometry, CKS_ERR_NULL without a buffer, CKS_ERR_WORKSPACE if the text did
 * not fit, CKS_ERR_UNSUPPORTED for an unknown op (or what the entry point itself
 * would answer). */
typedef enum {
    CKS_OP_CONV2D_FWD = 0,
    CKS_OP_DECONV2D = 1,
    CKS_OP_DILATED_CONV2D_WGRAD = 2,
    CKS_OP_KERNEL_SPLIT = 3,
    CKS_OP_DECONV2D_PRESPLIT = 4,
    CKS_OP_FILTER_TRANSPOSE = 5,
    CKS_OP_WGRAD_PARTIALS = 6,
    CKS_OP_REDUCE_PARTIALS = 7,
    CKS_OP_CONV2D_FWD_TRANSPOSED = 8,
    CKS_OP_CONV2D_FWD_UNTRIMMED = 9,
    CKS_OP_DECONV2D_UNTRIMMED = 10,
    CKS_OP_WGRAD_UNTRIMMED = 11
} cks_op;
int cks_plan_hw(int op, int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                unsigned only_4byte_aligned, char *text, size_t text_bytes);

const char *cks_strerror(int status);
int cks_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CKS_H */
