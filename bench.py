#!/usr/bin/env python3
"""Benchmark of the C-K-S conv-layer hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch of a layer: ConvV2 forward, KS-deconv-V2
input gradient and Sk-dilated-V2 filter gradient (segments + aggregation), inputs resident in HBM.  The
default run times every benchmark layer (cfg1 ... cfg4b) and prints ONE JSON line:

  value / ms_per_step   the step on the headline layer (--config, default cfg3a: the largest layer by
                        useful FLOPs), exactly --steps steps between two events, median of --repeats
  configs               per layer: step and per-operator ms (median and min of the repeats), useful
                        TFLOP/s, % of the fp32 matrix peak, the kernels each call launches, the
                        main kernels' own launch times, the input gradient with the filter split
                        beforehand and the forward pass on the filter transposed beforehand (Section V.A /
                        IV.A, pack excluded / included), and that layer's roofline
  min_pct_fp32_mfma_peak the lowest per-operator figure over all layers, with the layer and operator
  roofline              the headline layer's dominant kernel against 157.3 TFLOP/s
  cpu_baseline          the CPU oracle on a bounded sample of the headline layer

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg3a] [--layers cfg1,cfg2,...]
    python bench.py --ablation | --sweep | --mfma-probe | --copy-probe
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X published dense fp32 matrix peak
METRIC = "useful TFLOPS per operator (ConvV2 / KS-deconv / Sk-dilated), % fp32 MFMA peak"
BENCH_LAYERS = ["cfg1", "cfg2", "cfg3a", "cfg3b", "cfg4a", "cfg4b"]
SETTLE_MS = 250.0               # load put on the GPU before a layer is timed, whatever --warmup says
OPS = ("conv2d_fwd", "deconv2d", "dilated_conv2d_wgrad")


def describe(L):
    return ("%s: N=%d C=%d H=W=%dx%d OC=%d %dx%d stride %d pad %d, fp32 NHWC; X,dY~N(0,1), W He-normal"
            % (L.name, L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding))


class LayerBench:
    """Device buffers of one layer and the calls of its hot path."""

    def __init__(self, L, seed=0):
        import torch
        from paper_2306_15951_amd import binding as cks
        from paper_2306_15951_amd import synth

        self.L, self.cks, self.torch = L, cks, torch
        self.g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding)
        self.g_hw = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, (L.stride,) * 2, (L.padding,) * 2)
        self.host = synth.make_inputs(L, "normal", seed)
        X, W, dY = self.host
        d = "cuda:0"
        self.X, self.W, self.dY = (torch.from_numpy(a).to(d) for a in (X, W, dY))
        self.Y = torch.empty_like(self.dY)
        self.dX = torch.empty_like(self.X)
        self.dW = torch.empty_like(self.W)
        self.gz = cks.cks_dilated_conv2d_wgrad_segments(*self.g)
        self.ws_deconv = torch.empty(max(cks.cks_deconv2d_workspace(*self.g) // 4, 1), device=d)
        self.ws_wgrad = torch.empty(max(cks.cks_dilated_conv2d_wgrad_workspace(*self.g) // 4, 1), device=d)
        s = L.stride
        self.Cs = torch.empty((s, s, L.IC, -(-L.FH // s), -(-L.FW // s), L.OC), device=d)
        self.part = torch.empty((self.gz, L.OC, L.FH, L.FW, L.IC), device=d)
        self.Wtt = torch.empty((L.FH, L.FW, L.IC, L.OC), device=d)
        self.useful_flops = 2 * cks.cks_useful_macs(*self.g)

    def plan(self, op):
        """Names of the kernels entry point `op` launches for this layer (host-side query of the library)."""
        return [k for k, _ in self.cks.cks_plan_hw(op, *self.g_hw)]

    # the three operators as a user calls them
    def fwd(self):
        self.cks.cks_conv2d_fwd(self.X, self.W, self.Y, self.L.stride, self.L.padding)

    def deconv(self):
        self.cks.cks_deconv2d(self.dY, self.W, self.dX, self.L.stride, self.L.padding, self.ws_deconv)

    def wgrad(self):
        self.cks.cks_dilated_conv2d_wgrad(self.X, self.dY, self.dW, self.L.stride, self.L.padding, self.ws_wgrad)

    def step(self):
        self.fwd()
        self.deconv()
        self.wgrad()

    # single stages (stage entry points)
    def k_split(self):
        self.cks.cks_kernel_split(self.W, self.Cs, self.L.stride)

    def k_deconv_presplit(self):
        self.cks.cks_deconv2d_presplit(self.dY, self.Cs, self.dX, self.L.FH, self.L.FW, self.L.stride, self.L.padding)

    def k_transpose(self):
        self.cks.cks_filter_transpose(self.W, self.Wtt)

    def k_fwd_transposed(self):
        self.cks.cks_conv2d_fwd_transposed(self.X, self.Wtt, self.Y, self.L.stride, self.L.padding)

    def k_wgrad_main(self):
        self.cks.cks_dilated_conv2d_wgrad_partials(self.X, self.dY, self.part, self.L.FH, self.L.FW,
                                                   self.L.stride, self.L.padding)

    def k_reduce(self):
        self.cks.cks_reduce_partials(self.part, self.dW)

    def settle(self, ms=SETTLE_MS):
        """Keep the GPU under this layer's load for `ms`: after an idle spell (allocating and filling the
        tensors is one) the board needs some tens of milliseconds before timings are steady."""
        torch = self.torch
        busy, batch = 0.0, 3
        while busy < ms:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(batch):
                self.step()
            e1.record()
            torch.cuda.synchronize()
            t = max(e0.elapsed_time(e1), 1e-3)
            busy += t
            batch = max(3, min(int(batch * 50.0 / t), 2000))      # batches of about 50 ms

    def time_ms(self, fn, iters, warmup, repeats=1):
        """Milliseconds per call, one figure per repeat: `iters` calls between two events on the stream the
        library launches on (torch's current stream is the one handed to it), a device sync on both sides."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        out = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / iters)
        return out


def hbm_traffic(layer, kernel):
    """HBM bytes per launch of `kernel` on `layer` from the committed rocprofv3 counter summary
    (profiles/hbm_traffic.txt: FETCH_SIZE / WRITE_SIZE runs of this script, scaled by a copy kernel of
    known size), or None.  Not a measurement of the present run."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.rstrip("\n").split("\t")
        if len(f) == 4 and f[0] == layer and f[1].replace(" ", "") == kernel.replace(" ", ""):
            return float(f[2]) + float(f[3])
    return None


def mfma_probe(fn=None, busy_ms=30.0):
    """What the fp32 matrix cores sustain on this machine (bench_probe/libcks_probe.so), each case run back to
    back for busy_ms after 20 ms of the same load, with the shader clock sampled from a second stream
    meanwhile.  With fn (a callable that launches work on the current stream) only the clock under that
    load is measured."""
    import ctypes
    import torch

    path = os.path.join(ROOT, "bench_probe", "libcks_probe.so")
    if not os.path.exists(path):
        raise ImportError("bench_probe/libcks_probe.so is not built: run __graft_entry__.build()")
    P = ctypes.CDLL(path)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    P.cks_probe_mfma_registers.argtypes = [vp, ci, ci, ci, vp]
    P.cks_probe_mfma_lds.argtypes = [vp, ci, ci, ci, ci, vp]
    P.cks_probe_clock_samples.argtypes = [vp, ci, ci, vp]
    out = torch.zeros(256, device="cuda:0")
    side = torch.cuda.Stream()
    n = 600                                     # samples about 27 us apart: 16 ms
    stamps = torch.zeros(2 * n, dtype=torch.int64, device="cuda:0")
    st = lambda: ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def run(launch):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); launch(); launch(); e1.record(); torch.cuda.synchronize()
        per = max(e0.elapsed_time(e1) / 2, 1e-3)
        for _ in range(int(20.0 / per) + 1):
            launch()
        reps = int(busy_ms / per) + 1
        assert P.cks_probe_clock_samples(stamps.data_ptr(), n, 8, ctypes.c_void_p(side.cuda_stream)) == 0
        e0.record()
        for _ in range(reps):
            launch()
        e1.record()
        torch.cuda.synchronize()
        h = stamps.cpu().numpy().reshape(n, 2)
        ghz = float(h[-1, 1] - h[0, 1]) / (float(h[-1, 0] - h[0, 0]) / 100e6) / 1e9
        return e0.elapsed_time(e1) / reps, ghz

    if fn is not None:
        ms, ghz = run(fn)
        return {"ms_per_call": ms, "shader_clock_ghz": ghz}
    res = {}
    iters, chunks, items = 4096, 18, 64
    cases = (
        ("registers_constant_operands", 1024.0 * 4 * iters * 8, lambda: P.cks_probe_mfma_registers(out.data_ptr(), 1024, iters, 0, st())),
        ("registers_varying_operands", 1024.0 * 4 * iters * 8, lambda: P.cks_probe_mfma_registers(out.data_ptr(), 1024, iters, 1, st())),
        ("lds_fed_k_loop_constant_operands", 1024.0 * 4 * items * chunks * 16, lambda: P.cks_probe_mfma_lds(out.data_ptr(), 1024, chunks, items, 0, st())),
        ("lds_fed_k_loop_varying_operands", 1024.0 * 4 * items * chunks * 16, lambda: P.cks_probe_mfma_lds(out.data_ptr(), 1024, chunks, items, 1, st())),
    )
    for name, mfmas, launch in cases:
        ms, ghz = run(launch)
        tf = mfmas * 4096 / ms / 1e9
        res[name] = {"tflops": tf, "pct_of_published_peak": 100 * tf / PEAK_FP32_MFMA_TFLOPS, "shader_clock_ghz": ghz}
    return res


def cpu_baseline(L, host, useful_flops, budget_s=6.0):
    """The oracle as it stands, on a random sample of outputs of each operator (indices drawn with
    replacement), sized from a short calibration so that each operator takes about budget_s."""
    import numpy as np
    import oracle

    X, W, dY = host
    rng = np.random.default_rng(1)
    ops = (("conv_fwd", dY.size, lambda sm: oracle.conv_fwd(X, W, L.stride, L.padding, sample=sm)),
           ("deconv", X.size, lambda sm: oracle.deconv(dY, W, L.IH, L.IW, L.stride, L.padding, sample=sm)),
           ("wgrad", W.size, lambda sm: oracle.wgrad(X, dY, L.FH, L.FW, L.stride, L.padding, sample=sm)))
    flops = secs = 0.0
    parts = []
    for name, size, fn in ops:
        n0 = max(min(size // 1000, 2000), 16)
        t = time.time(); fn(rng.integers(0, size, n0)); t0 = time.time() - t    # includes materialising the zeros
        t = time.time(); fn(rng.integers(0, size, 4 * n0)); t1 = time.time() - t
        per = max((t1 - t0) / (3 * n0), 1e-9)
        n = int(min(size, max(n0, (budget_s - min(t0, budget_s / 2)) / per)))
        t = time.time(); fn(rng.integers(0, size, n)); dt = time.time() - t
        flops += useful_flops * n / size
        secs += dt
        parts.append("%s %d of %d outputs in %.2fs" % (name, n, size, dt))
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%s: " % L.name + "; ".join(parts) + " (random output elements drawn with replacement, useful FLOPs "
                      "pro rata, time includes building the padded / zero-inserted tensors)"}


def pct(tflops):
    return 100.0 * tflops / PEAK_FP32_MFMA_TFLOPS


def timing(ms_list, flops):
    med, lo = statistics.median(ms_list), min(ms_list)
    tf = flops / med / 1e9
    return {"ms_median": med, "ms_min": lo, "useful_tflops": tf, "pct_fp32_mfma_peak": pct(tf),
            "pct_fp32_mfma_peak_best": pct(flops / lo / 1e9)}


def bench_layer(L, steps, warmup, repeats, settle_ms=SETTLE_MS):
    """All timings of one layer.  Returns (LayerBench, dict)."""
    B = LayerBench(L)
    cks = B.cks
    out = {"workload": describe(L), "useful_gflop_per_operator": B.useful_flops / 1e9, "segments_G_Z": B.gz}
    B.settle(settle_ms)
    out["step"] = timing(B.time_ms(B.step, steps, warmup, repeats), 3 * B.useful_flops)
    ops = {}
    for name, fn, op in (("conv2d_fwd", B.fwd, cks.CKS_OP_CONV2D_FWD), ("deconv2d", B.deconv, cks.CKS_OP_DECONV2D),
                         ("dilated_conv2d_wgrad", B.wgrad, cks.CKS_OP_DILATED_CONV2D_WGRAD)):
        ops[name] = timing(B.time_ms(fn, steps, warmup, repeats), B.useful_flops)
        ops[name]["kernels"] = B.plan(op)
    out["operators"] = ops
    # Main kernels on their own.  Forward and input gradient are one main launch each (the few-channel input
    # gradient adds a short second one, timed with it); the filter gradient's main kernel and its aggregation
    # are timed through the stage entry points.  These are event timings of back-to-back launches, so each
    # includes the gap between two launches (3-5 us) that a profiler's kernel duration does not.
    B.k_wgrad_main()
    mains = {
        ops["conv2d_fwd"]["kernels"][0]: ops["conv2d_fwd"]["ms_median"],
        ops["deconv2d"]["kernels"][0]: ops["deconv2d"]["ms_median"],
        B.plan(cks.CKS_OP_WGRAD_PARTIALS)[0]: statistics.median(B.time_ms(B.k_wgrad_main, steps, warmup, repeats)),
    }
    out["main_kernels"] = {k: {"ms": v, "useful_tflops": B.useful_flops / v / 1e9, "frac_of_peak": B.useful_flops / v / 1e9 / PEAK_FP32_MFMA_TFLOPS}
                           for k, v in mains.items()}
    if B.gz > 1:
        out["reduce_slices_ms"] = statistics.median(B.time_ms(B.k_reduce, steps, warmup, repeats))
    # The filter operations done before the loop (Section V.A): Stage 1 once, Stage 2&3 on the split filter.
    B.k_split()
    split_ms = statistics.median(B.time_ms(B.k_split, steps, warmup, repeats))
    pre_ms = statistics.median(B.time_ms(B.k_deconv_presplit, steps, warmup, repeats))
    out["deconv2d_filter_split_beforehand"] = {
        "kernel_split_ms": split_ms, "stage2and3_ms": pre_ms, "kernels": B.plan(cks.CKS_OP_DECONV2D_PRESPLIT),
        "pct_fp32_mfma_peak_pack_excluded": pct(B.useful_flops / pre_ms / 1e9),
        "pct_fp32_mfma_peak_pack_included": pct(B.useful_flops / (pre_ms + split_ms) / 1e9),
    }
    # ... and the forward pass on the transposed filter (Section IV.A: the filter is transposed first when the
    # input is large); the kernel exists for whole 32-channel chunks of C only
    B.k_transpose()
    tr_ms = statistics.median(B.time_ms(B.k_transpose, steps, warmup, repeats))
    try:
        B.k_fwd_transposed()
        ft_ms = statistics.median(B.time_ms(B.k_fwd_transposed, steps, warmup, repeats))
        out["conv2d_fwd_filter_transposed_beforehand"] = {
            "filter_transpose_ms": tr_ms, "conv2d_fwd_transposed_ms": ft_ms, "kernels": B.plan(cks.CKS_OP_CONV2D_FWD_TRANSPOSED),
            "pct_fp32_mfma_peak_pack_excluded": pct(B.useful_flops / ft_ms / 1e9),
            "pct_fp32_mfma_peak_pack_included": pct(B.useful_flops / (ft_ms + tr_ms) / 1e9),
            "speedup_over_conv2d_fwd_pack_excluded": ops["conv2d_fwd"]["ms_median"] / ft_ms,
        }
    except cks.CksError as e:
        if e.status != cks.CKS_ERR_UNSUPPORTED:
            raise
        out["conv2d_fwd_filter_transposed_beforehand"] = {"filter_transpose_ms": tr_ms, "conv2d_fwd_transposed_ms": None,
                                                          "note": "no kernel for this geometry (C is not a multiple of 32)"}
    dom = max(mains, key=mains.get)
    achieved = B.useful_flops / mains[dom] / 1e9
    out["roofline"] = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                       "frac": achieved / PEAK_FP32_MFMA_TFLOPS, "traffic": hbm_traffic(L.name, dom),
                       "traffic_unit": "HBM bytes per launch, read from profiles/hbm_traffic.txt (rocprofv3 FETCH_SIZE + WRITE_SIZE "
                                       "of an earlier run of this script; not measured in this run)"}
    return B, out


# Invented stand-ins for the paper's first experiment (its 16 shapes per operator are not disclosed):
# two filter sets, eight shapes each with shrinking maps and growing channels, and a stride series.
SWEEP = (
    [("3x3p1_%d" % i, n, c, hw, hw, c, 3, 3, 1, 1) for i, (n, c, hw) in enumerate(
        [(64, 64, 64), (128, 64, 32), (64, 128, 32), (128, 128, 16), (64, 256, 16), (128, 256, 8), (128, 512, 8), (256, 512, 4)])] +
    [("5x5p2_%d" % i, n, c, hw, hw, c, 5, 5, 1, 2) for i, (n, c, hw) in enumerate(
        [(64, 64, 64), (128, 64, 32), (64, 128, 32), (128, 128, 16), (64, 256, 16), (128, 256, 8), (128, 512, 8), (256, 512, 4)])] +
    [("5x5p2_s%d" % st, 64, 128, 32, 32, 128, 5, 5, st, 2) for st in (2, 3, 4)]
)


def sweep(steps, warmup, repeats):
    """Useful TFLOP/s of the three operators over the SWEEP shapes."""
    import torch
    from paper_2306_15951_amd import synth

    rows = {}
    for geo in SWEEP:
        B = LayerBench(synth.Layer(*geo))
        B.settle()
        r = {}
        for name, fn in (("conv2d_fwd", B.fwd), ("deconv2d", B.deconv), ("dilated_conv2d_wgrad", B.wgrad)):
            t = timing(B.time_ms(fn, steps, warmup, repeats), B.useful_flops)
            r[name] = {"ms": t["ms_median"], "pct_fp32_mfma_peak": t["pct_fp32_mfma_peak"]}
        rows[geo[0]] = {"geometry": geo[1:], "useful_gflop": B.useful_flops / 1e9, "operators": r}
        del B
        torch.cuda.empty_cache()
    return rows


def ablation(L, steps, warmup):
    """What each zero-skipping step is worth, per operator, with the library's own kernels throughout:

      skip       the operator as the library runs it (ConvV2, KS-deconv-V2, Sk-dilated-V2)
      untrimmed  trimming off, kernel split / leaping access kept: plain convolution, KS-deconv
                 (Algorithm 2), Sk-dilated (Algorithm 3) -- the library's *_untrimmed entry points: the
                 same kernels built without the trimming, on the same tensors; the window cells outside
                 the data are fetched as zeros by the loads and multiplied
      untrimmed_materialised
                 the same three algorithms through the library's ordinary entry points, on tensors
                 whose zero border is written out (paper_2306_15951_amd/untrimmed.py)
      dense      the textbook form that multiplies every zero: padded input; stride-inserted zeros on a
                 canvas + rotated filter at unit stride; the dilated gradient as a filter -- all through
                 cks_conv2d_fwd with padding 0
    """
    import torch
    import torch.nn.functional as F
    from paper_2306_15951_amd import untrimmed

    B = LayerBench(L)
    B.settle()
    cks, s, p = B.cks, L.stride, L.padding
    OH, OW = cks.cks_out_dims(L.IH, L.IW, L.FH, L.FW, s, p)
    out = {"useful_gflop": B.useful_flops / 1e9, "dense_gflop": 2e-9 * cks.cks_useful_macs(L.N, L.IC, L.IH + 2 * p, L.IW + 2 * p, L.OC, L.FH, L.FW, s, 0)}

    def timed(fns):
        # alternate the forms three times and keep each one's best: buffers run slower for their first
        # launches and the order of measurement must not decide a 5 % difference
        best = [float("inf")] * len(fns)
        for _ in range(3):
            for i, fn in enumerate(fns):
                best[i] = min(best[i], B.time_ms(fn, steps, warmup)[0])
        return best

    def close(a, b):
        return float((a - b).abs().max() / max(float(b.abs().max()), 1e-30))

    def row(skip, untrim, mat, dense, got_untrim, got_mat, got_dense, want):
        skip(); untrim(); mat(); dense()
        torch.cuda.synchronize()
        d = {"max_rel_diff_untrimmed": close(got_untrim(), want()), "max_rel_diff_untrimmed_materialised": close(got_mat(), want()),
             "max_rel_diff_dense": close(got_dense(), want())}
        d["skip_ms"], d["untrimmed_ms"], d["untrimmed_materialised_ms"], d["dense_ms"] = timed((skip, untrim, mat, dense))
        d["gain_of_trimming"] = d["untrimmed_ms"] / d["skip_ms"]
        d["gain_over_dense"] = d["dense_ms"] / d["skip_ms"]
        return d

    sp, pp = (s, s), (p, p)

    # ConvV2 | plain convolution = the dense form: the padded input, padding 0
    Xp = F.pad(B.X, (0, 0, p, p, p, p)).contiguous()
    Y2 = torch.empty_like(B.Y)
    Y1 = torch.empty_like(B.Y)
    plain = lambda: cks.cks_conv2d_fwd(Xp, B.W, Y2, s, 0)
    out["conv2d_fwd"] = row(B.fwd, lambda: cks.cks_conv2d_fwd_untrimmed_hw(B.X, B.W, Y1, sp, pp), plain, plain,
                            lambda: Y1, lambda: Y2, lambda: Y2, lambda: B.Y)
    # KS-deconv-V2 | KS-deconv (Algorithm 2) | zero-inserted gradient on a zero canvas, rotated filter, unit stride
    dX1, dX0 = torch.empty_like(B.dX), torch.empty_like(B.dX)
    alg2 = untrimmed.prepare_deconv2d(cks, B.dY, B.W, dX1, s, p)
    Z = torch.zeros((L.N, L.IH + L.FH - 1, L.IW + L.FW - 1, L.OC), device=B.X.device)
    o = (L.FH - 1 - p, L.FW - 1 - p)
    hs, ws = (OH - 1) * s + 1, (OW - 1) * s + 1
    ih = torch.arange(0, hs, s, device=B.X.device) + o[0]
    iw = torch.arange(0, ws, s, device=B.X.device) + o[1]
    mh, mw = (ih >= 0) & (ih < Z.shape[1]), (iw >= 0) & (iw < Z.shape[2])
    Z[:, ih[mh][:, None], iw[mw][None, :], :] = B.dY[:, mh][:, :, mw]
    Wr = B.W.flip(1, 2).permute(3, 1, 2, 0).contiguous()      # [IC, FH, FW, OC]
    dX2 = torch.empty_like(B.dX)
    out["deconv2d"] = row(B.deconv, lambda: cks.cks_deconv2d_untrimmed_hw(B.dY, B.W, dX0, sp, pp), alg2,
                          lambda: cks.cks_conv2d_fwd(Z, Wr, dX2, 1, 0), lambda: dX0, lambda: dX1, lambda: dX2, lambda: B.dX)
    # Sk-dilated-V2 | Sk-dilated (Algorithm 3) | the dilated gradient as the filter of a unit-stride convolution
    # over the padded input (image axis and channel axis change places: the contraction runs over n)
    dW1, dW0 = torch.empty_like(B.dW), torch.empty_like(B.dW)
    alg3 = untrimmed.prepare_dilated_conv2d_wgrad(cks, B.X, B.dY, dW1, s, p)
    D = torch.zeros((L.N, hs, ws, L.OC), device=B.X.device)
    D[:, ::s, ::s, :] = B.dY
    need_h, need_w = hs + L.FH - 1, ws + L.FW - 1                    # padded rows the FH x FW output uses
    Xq = Xp[:, :need_h, :need_w, :].permute(3, 1, 2, 0).contiguous()   # [IC, rows, cols, N]
    Dq = D.permute(3, 1, 2, 0).contiguous()                            # [OC, hs, ws, N]
    dWq = torch.empty((L.IC, L.FH, L.FW, L.OC), device=B.X.device)
    out["dilated_conv2d_wgrad"] = row(B.wgrad, lambda: cks.cks_dilated_conv2d_wgrad_untrimmed_hw(B.X, B.dY, dW0, sp, pp, B.ws_wgrad), alg3,
                                      lambda: cks.cks_conv2d_fwd(Xq, Dq, dWq, 1, 0),
                                      lambda: dW0, lambda: dW1, lambda: dWq.permute(3, 1, 2, 0), lambda: B.dW)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20, help="untimed calls before each timed series (on top of %.0f ms of load per layer)" % SETTLE_MS)
    ap.add_argument("--repeats", type=int, default=5, help="timed series of --steps calls each; median and min are reported")
    ap.add_argument("--config", default="cfg3a", help="headline layer (value, ms_per_step, roofline, cpu_baseline)")
    ap.add_argument("--layers", default=",".join(BENCH_LAYERS), help="layers to time (the headline layer is always included)")
    ap.add_argument("--settle-ms", type=float, default=SETTLE_MS, help="load put on the GPU before a layer is timed (profiler runs use less)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true", help="skip the sustained-rate / clock probes")
    ap.add_argument("--sweep", action="store_true", help="only: the three operators over a sweep of invented shapes")
    ap.add_argument("--ablation", action="store_true",
                    help="only: zeros skipped / trimming off / zeros multiplied, same kernels, on the benchmark layers")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="only: the fp32 matrix rate this box sustains (registers / LDS-fed loop, constant / varying operands)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run only a plain 1 GiB -> 1 GiB streaming kernel (calibrates the HBM byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2306_15951_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if a.copy_probe:
        # out = in * 1: every launch reads 1 GiB and writes 1 GiB, nothing else
        n = 1 << 28
        src = torch.ones(n, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe": "torch.mul(src, 1.0, out=dst), float32", "bytes_read_per_launch": 4 * n,
                          "bytes_written_per_launch": 4 * n, "launches": 5}))
        return
    if a.mfma_probe:
        LayerBench(synth.LAYERS["cfg1"]).settle(500.0)
        print(json.dumps({"mfma_probe": mfma_probe(), "unit": "TFLOP/s", "published_peak": PEAK_FP32_MFMA_TFLOPS}))
        return
    if a.sweep:
        print(json.dumps({"sweep": sweep(a.steps, a.warmup, a.repeats), "steps": a.steps, "warmup": a.warmup,
                          "repeats": a.repeats, "data": "synthetic, invented shapes"}))
        return
    if a.ablation:
        res = {}
        for name in ("cfg1", "cfg2", "cfg3a", "cfg3b", "cfg4a"):
            res[name] = ablation(synth.LAYERS[name], a.steps, a.warmup)
            torch.cuda.empty_cache()
        print(json.dumps({"ablation": res, "steps": a.steps, "warmup": a.warmup, "data": "synthetic"}))
        return

    names = [n for n in a.layers.split(",") if n]
    if a.config not in names:
        names.append(a.config)
    configs, head = {}, None
    for name in names:
        B, r = bench_layer(synth.LAYERS[name], a.steps, a.warmup, a.repeats, a.settle_ms)
        configs[name] = r
        if name == a.config:
            head = (B.L, B.host, B.useful_flops)
        if not a.no_probe:
            # shader clock while this layer's dominant kernel runs back to back (sampled from a second stream), and the
            # kernel's rate against the matrix peak at that clock: what is left is the kernel's, the rest the board's
            k = r["roofline"]["kernel"]
            fn = B.fwd if k == r["operators"]["conv2d_fwd"]["kernels"][0] else (
                B.deconv if k == r["operators"]["deconv2d"]["kernels"][0] else B.k_wgrad_main)
            clk = mfma_probe(fn)
            r["roofline"]["clock_under_dominant_kernel"] = clk
            r["roofline"]["frac_of_peak_at_that_clock"] = r["roofline"]["frac"] * 2.4 / clk["shader_clock_ghz"]
        del B
        torch.cuda.empty_cache()
    H = configs[a.config]
    lowest = min(((r["operators"][op]["pct_fp32_mfma_peak"], name, op) for name, r in configs.items() for op in OPS))
    line = {
        "metric": METRIC, "value": H["step"]["useful_tflops"], "unit": "TFLOP/s", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": H["step"]["ms_median"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": H["workload"], "step": "conv2d_fwd + deconv2d + dilated_conv2d_wgrad",
                   "useful_gflop_per_operator": H["useful_gflop_per_operator"], "segments_G_Z": H["segments_G_Z"],
                   "timing": "median of %d series of %d steps, each after %d untimed steps; %.0f ms of load per layer first"
                             % (a.repeats, a.steps, a.warmup, a.settle_ms)},
        "pct_fp32_mfma_peak": H["step"]["pct_fp32_mfma_peak"],
        "min_pct_fp32_mfma_peak": {"value": lowest[0], "layer": lowest[1], "operator": lowest[2],
                                   "over": "every operator of " + ", ".join(configs)},
        "pct_fp32_mfma_peak_by_layer": {name: {op: round(r["operators"][op]["pct_fp32_mfma_peak"], 2) for op in OPS}
                                        for name, r in configs.items()},
        "roofline": dict(H["roofline"]),
        "configs": configs,
    }
    if not a.no_probe:
        # the same rate against what the matrix cores sustain here with operands that vary (the published
        # peak assumes back-to-back issue at 2.4 GHz)
        probe = mfma_probe()
        line["roofline"]["peak_sustained"] = {
            "what": "fp32 MFMA rate measured on this box, TFLOP/s: LDS-fed K loop of the general kernels without its global "
                    "side / registers only; constant / varying operands",
            "probe": probe,
            "frac_of_lds_fed_varying": H["roofline"]["achieved"] / probe["lds_fed_k_loop_varying_operands"]["tflops"]}
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(*head)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
