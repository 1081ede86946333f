#!/usr/bin/env python3
"""Benchmark of the C-K-S conv-layer hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch of a layer:
ConvV2 forward, KS-deconv-V2 input gradient (kernel split + Stage 2&3) and
Sk-dilated-V2 filter gradient (segments + reduction), inputs resident in HBM.
Prints ONE JSON line: useful (zero-free) TFLOP/s of the step, the roofline of
the dominant kernel measured with events on the launch stream, and the CPU
oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg1] [--all]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X published dense fp32 matrix peak
METRIC = "useful TFLOPS per operator (ConvV2 / KS-deconv / Sk-dilated), % fp32 MFMA peak"


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
        self.useful_flops = 2 * cks.cks_useful_macs(*self.g)

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

    # single kernels (stage entry points)
    def k_split(self):
        self.cks.cks_kernel_split(self.W, self.Cs, self.L.stride)

    def k_deconv_main(self):
        self.cks.cks_deconv2d_presplit(self.dY, self.Cs, self.dX, self.L.FH, self.L.FW, self.L.stride, self.L.padding)

    def k_wgrad_main(self):
        self.cks.cks_dilated_conv2d_wgrad_partials(self.X, self.dY, self.part, self.L.FH, self.L.FW,
                                                   self.L.stride, self.L.padding)

    def k_reduce(self):
        self.cks.cks_reduce_partials(self.part, self.dW)

    def time_ms(self, fn, iters, warmup):
        """Average milliseconds per call: events on the stream the library launches on."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()          # torch's current stream == the stream handed to the library
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters


def measured_traffic(workload, kernel_prefix):
    """HBM bytes per launch of a kernel, from the committed rocprofv3 counter
    summary of this workload (profiles/bench_<workload>_traffic.txt), or None."""
    path = os.path.join(ROOT, "profiles", "bench_%s_traffic.txt" % workload)
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("#"):
            continue
        f = line.rstrip("\n").split("\t")
        if len(f) == 3 and f[0].startswith(kernel_prefix):
            return float(f[1]) + float(f[2])
    return None


def mfma_probe(fn=None, busy_ms=30.0):
    """What the fp32 matrix cores sustain on this machine (libcks_probe.so, include/cks_probe.h), each case run
    back to back for busy_ms after 20 ms of the same load, with the shader clock sampled from a second
    stream meanwhile.  With fn (a callable that launches work on the current stream) only the clock under
    that load is measured."""
    import ctypes
    import numpy as np
    import torch

    path = os.path.join(ROOT, "paper_2306_15951_amd", "libcks_probe.so")
    if not os.path.exists(path):
        raise ImportError("libcks_probe.so is not built: run __graft_entry__.build()")
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
    """The oracle as it stands, on a random sample of outputs of each operator,
    sized from a short calibration so that each operator takes about budget_s."""
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
            "sample": "; ".join(parts) + " (random output elements, useful FLOPs pro rata, "
                      "time includes building the padded / zero-inserted tensors)"}


def bench_layer(L, steps, warmup, with_kernels=True):
    B = LayerBench(L)
    out = {"useful_gflop_per_operator": B.useful_flops / 1e9, "segments_G_Z": B.gz}
    ms_step = B.time_ms(B.step, steps, warmup)
    out["ms_per_step"] = ms_step
    out["step_tflops"] = 3 * B.useful_flops / ms_step / 1e9
    ops = {}
    for name, fn in (("conv2d_fwd", B.fwd), ("deconv2d", B.deconv), ("dilated_conv2d_wgrad", B.wgrad)):
        ms = B.time_ms(fn, steps, warmup)
        tf = B.useful_flops / ms / 1e9
        ops[name] = {"ms": ms, "useful_tflops": tf, "pct_fp32_mfma_peak": 100 * tf / PEAK_FP32_MFMA_TFLOPS}
    out["operators"] = ops
    if with_kernels:
        B.k_split(); B.k_wgrad_main()
        ker = {}
        # the step's own kernels (cfg1: one launch each for forward and input gradient, which reads the
        # filter in place; main + reduce for the filter gradient) and the stage entry points of the
        # pre-split mode (kernel split, Stage 2&3 on a split filter)
        for name, fn in (("rowrun_gemm<fwd>", B.fwd), ("rowrun_gemm<deconv>", B.deconv), ("pixel_gemm", B.k_wgrad_main),
                         ("reduce_slices", B.k_reduce), ("pack_filter<split>", B.k_split),
                         ("rowrun_gemm<deconv, presplit>", B.k_deconv_main)):
            ker[name] = B.time_ms(fn, steps, warmup)
        out["kernel_ms"] = ker
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


def warm_gpu():
    """Half a second of the cfg1 step, so that short timings that follow run at the sustained clock."""
    from paper_2306_15951_amd import synth

    B = LayerBench(synth.LAYERS["cfg1"])
    B.time_ms(B.step, 1500, 10)


def sweep(steps, warmup):
    """Useful TFLOP/s of the three operators over the SWEEP shapes."""
    import torch
    from paper_2306_15951_amd import synth

    rows = {}
    for geo in SWEEP:
        B = LayerBench(synth.Layer(*geo))
        r = {}
        for name, fn in (("conv2d_fwd", B.fwd), ("deconv2d", B.deconv), ("dilated_conv2d_wgrad", B.wgrad)):
            ms = B.time_ms(fn, steps, warmup)
            r[name] = {"ms": ms, "pct_fp32_mfma_peak": 100 * B.useful_flops / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS}
        rows[geo[0]] = {"geometry": geo[1:], "useful_gflop": B.useful_flops / 1e9, "operators": r}
        del B
        torch.cuda.empty_cache()
    return rows


def ablation(L, steps, warmup):
    """Skipping zeros against multiplying them, with the same kernels: each operator is also run in
    its textbook form on tensors with the zeros written out (padding border; stride-inserted zeros
    + rotated filter; dilated gradient), through cks_conv2d_fwd with padding 0."""
    import torch
    import torch.nn.functional as F

    B = LayerBench(L)
    cks, s, p = B.cks, L.stride, L.padding
    OH, OW = cks.cks_out_dims(L.IH, L.IW, L.FH, L.FW, s, p)
    out = {"useful_gflop": B.useful_flops / 1e9}

    def timed_pair(skip, dense):
        # alternate the two forms three times and keep each one's best: buffers run slower for their
        # first launches and the order of measurement must not decide a 5 % difference
        ts, td = [], []
        for _ in range(3):
            ts.append(B.time_ms(skip, steps, warmup))
            td.append(B.time_ms(dense, steps, warmup))
        return {"skip_ms": min(ts), "dense_ms": min(td)}

    def close(a, b):
        return float((a - b).abs().max() / max(float(b.abs().max()), 1e-30))

    # ConvV2 | padded input, padding 0
    Xp = F.pad(B.X, (0, 0, p, p, p, p)).contiguous()
    Y2 = torch.empty_like(B.Y)
    B.fwd(); cks.cks_conv2d_fwd(Xp, B.W, Y2, s, 0)
    out["conv2d_fwd"] = dict(timed_pair(B.fwd, lambda: cks.cks_conv2d_fwd(Xp, B.W, Y2, s, 0)), max_rel_diff=close(Y2, B.Y))
    # KS-deconv | zero-inserted gradient on a zero canvas, rotated filter, unit stride
    Z = torch.zeros((L.N, L.IH + L.FH - 1, L.IW + L.FW - 1, L.OC), device=B.X.device)
    o = (L.FH - 1 - p, L.FW - 1 - p)
    hs, ws = (OH - 1) * s + 1, (OW - 1) * s + 1
    ih = torch.arange(0, hs, s, device=B.X.device) + o[0]
    iw = torch.arange(0, ws, s, device=B.X.device) + o[1]
    mh, mw = (ih >= 0) & (ih < Z.shape[1]), (iw >= 0) & (iw < Z.shape[2])
    Z[:, ih[mh][:, None], iw[mw][None, :], :] = B.dY[:, mh][:, :, mw]
    Wr = B.W.flip(1, 2).permute(3, 1, 2, 0).contiguous()      # [IC, FH, FW, OC]
    dX2 = torch.empty_like(B.dX)
    B.deconv(); cks.cks_conv2d_fwd(Z, Wr, dX2, 1, 0)
    out["deconv2d"] = dict(timed_pair(B.deconv, lambda: cks.cks_conv2d_fwd(Z, Wr, dX2, 1, 0)), max_rel_diff=close(dX2, B.dX))
    # Sk-dilated | dilated gradient as the filter of a unit-stride convolution over the padded input
    # (image axis and channel axis change places: the contraction runs over n)
    D = torch.zeros((L.N, hs, ws, L.OC), device=B.X.device)
    D[:, ::s, ::s, :] = B.dY
    need_h, need_w = hs + L.FH - 1, ws + L.FW - 1                    # padded rows the FH x FW output uses
    Xq = Xp[:, :need_h, :need_w, :].permute(3, 1, 2, 0).contiguous()   # [IC, rows, cols, N]
    Dq = D.permute(3, 1, 2, 0).contiguous()                            # [OC, hs, ws, N]
    dWq = torch.empty((L.IC, L.FH, L.FW, L.OC), device=B.X.device)
    B.wgrad(); cks.cks_conv2d_fwd(Xq, Dq, dWq, 1, 0)
    out["dilated_conv2d_wgrad"] = dict(timed_pair(B.wgrad, lambda: cks.cks_conv2d_fwd(Xq, Dq, dWq, 1, 0)),
                                       max_rel_diff=close(dWq.permute(3, 1, 2, 0), B.dW))
    for v in out.values():
        if isinstance(v, dict):
            v["speedup"] = v["dense_ms"] / v["skip_ms"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200)   # the box needs some tens of milliseconds of load to reach its steady state
    ap.add_argument("--config", default="cfg1")
    ap.add_argument("--all", action="store_true", help="also time the other benchmark layers (extra JSON field)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="only: the three operators over a sweep of invented shapes")
    ap.add_argument("--ablation", action="store_true",
                    help="only: zeros skipped against zeros multiplied, same kernels, on the benchmark layers")
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
        warm_gpu()
        print(json.dumps({"mfma_probe": mfma_probe(), "unit": "TFLOP/s", "published_peak": PEAK_FP32_MFMA_TFLOPS}))
        return
    if a.sweep or a.ablation:
        warm_gpu()
    if a.sweep:
        # freshly allocated buffers run slower for their first ~60 launches: long warm-up per operator
        print(json.dumps({"sweep": sweep(max(a.steps // 2, 10), max(3 * a.warmup, 60)), "data": "synthetic, invented shapes"}))
        return
    if a.ablation:
        res = {}
        for name in ("cfg1", "cfg2", "cfg3a", "cfg3b", "cfg4a"):
            res[name] = ablation(synth.LAYERS[name], max(a.steps // 4, 10), max(2 * a.warmup, 40))
            torch.cuda.empty_cache()
        print(json.dumps({"ablation": res, "data": "synthetic"}))
        return
    L = synth.LAYERS[a.config]
    B, r = bench_layer(L, a.steps, a.warmup)

    # dominant kernel of the step = the main kernel with the longest average launch
    mains = {k: r["kernel_ms"][k] for k in ("rowrun_gemm<fwd>", "rowrun_gemm<deconv>", "pixel_gemm")}
    dom = max(mains, key=mains.get)
    achieved = B.useful_flops / mains[dom] / 1e9
    # (kernel names as the profiler prints them: the variants that load their chunks straight into LDS)
    prefix = {"rowrun_gemm<fwd>": "cks::rowrun_gemm_dma<0", "rowrun_gemm<deconv>": "cks::rowrun_gemm_dma<2",
              "pixel_gemm": "cks::pixel_gemm_dma"}[dom]
    line = {
        "metric": METRIC, "value": r["step_tflops"], "unit": "TFLOP/s", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": describe(L), "step": "conv2d_fwd + deconv2d + dilated_conv2d_wgrad",
                   "useful_gflop_per_operator": r["useful_gflop_per_operator"], "segments_G_Z": r["segments_G_Z"]},
        "pct_fp32_mfma_peak": 100 * r["step_tflops"] / PEAK_FP32_MFMA_TFLOPS,
        "operators": r["operators"], "kernel_ms": r["kernel_ms"],
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                     "traffic": measured_traffic(a.config, prefix), "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE+WRITE_SIZE)",
                     "all_main_kernels": {k: B.useful_flops / v / 1e9 for k, v in mains.items()}},
    }
    # the same rate against what the matrix cores sustain here with operands that vary (the published peak
    # assumes back-to-back issue at 2.4 GHz), and the shader clock while the dominant kernel runs
    probe = mfma_probe()
    sustained = probe["lds_fed_k_loop_varying_operands"]["tflops"]
    line["roofline"]["peak_sustained"] = {
        "what": "fp32 MFMA rate measured on this box, TFLOP/s: LDS-fed K loop of the general kernels without its global side / registers only; constant / varying operands",
        "probe": probe, "frac_of_lds_fed_varying": achieved / sustained,
        "clock_under_dominant_kernel": mfma_probe({"rowrun_gemm<fwd>": B.fwd, "rowrun_gemm<deconv>": B.deconv, "pixel_gemm": B.k_wgrad_main}[dom]),
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(L, B.host, B.useful_flops)
    if a.all:
        others = {}
        for name in synth.LAYERS:
            if name in (a.config, "cfg0"):
                continue
            del B
            torch.cuda.empty_cache()
            B, rr = bench_layer(synth.LAYERS[name], max(a.steps // 2, 10), max(a.warmup, 100))
            others[name] = rr
        line["other_configs"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
