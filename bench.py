#!/usr/bin/env python3
"""Benchmark of the Indirect Convolution hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--no-shapes] [--sweep N]

A step is one icv_conv2d_nhwc call (the Indirect GEMM, epilogue included) on the headline workload
(ResNet-style 3x3 bf16 convolution, N=32, 56x56, C=K=64).  As in the paper's protocol (section 3.1,
"Protocol") the indirection buffer and the packed filter are built once, outside the timed region; the
indirection build is timed on its own and reported under "setup".  The timed region rotates over enough
distinct input / output / indirection buffer sets to exceed the 256 MB last-level cache, so every step reads
its operands from HBM ("cold"); the same-buffers ("warm") figure is reported beside it.

Prints ONE JSON line.  metric = effective TFLOP/s = 2*N*Hout*Wout*K*R*S*C / t.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"bf16": 2500.0, "u8i8": 5000.0, "f32": 157.3}      # TFLOP/s (TOP/s), dense, MI355X public figures
HBM_PEAK_GBS = 8000.0
LLC_BYTES = 256 << 20

# HBM traffic per launch recorded from rocprofv3 --pmc runs (one for FETCH_SIZE, one for WRITE_SIZE, KiB per dispatch,
# each scaled by what the same counter reads for a 256 MiB copy; profiles/igemm_hbm_traffic.md holds the runs and the
# command).  A constant recorded then, NOT measured by this run: it is reported only while the library still picks
# the kernel it was recorded for.
FETCH_SCALE, WRITE_SCALE = 1.99975, 1.0
RECORDED_TRAFFIC = {
    # workload: (kernel, FETCH_SIZE KiB, WRITE_SIZE KiB)
    "cfg1_tiny_f32": ("generic_f32", 52.9, 2.0),
    "cfg2_3x3_c64": ("mfma_bf16_freg_w2m2", 7713.8, 25090.6),
    "cfg3a_3x3_s2": ("mfma_bf16_freg_w4m1", 15740.5, 25088.0),
    "cfg3b_3x3_d2": ("mfma_bf16_freg_w4m2", 10163.9, 32771.9),
    "cfg3c_5x5_asym": ("mfma_bf16_freg_w2m2", 6317.0, 24648.8),
    "cfg4_int8_3x3": ("mfma_i8_freg_w4m2", 6027.2, 25089.9),
    "cfg5a_1x1": ("gemm_bf16_256x64_c4x2_p8", 25305.5, 25101.9),
    "cfg5b_7x7_s2": ("mfma_bf16_lowc_64x64", 32829.0, 100363.7),
}
TRAFFIC_SOURCE = "recorded constant from profiles/igemm_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE), not measured in this run"
ALU_PEAK_F32 = 157.3          # TFLOP/s, fp32 vector ALUs: 256 CUs x 4 SIMDs x 32 lanes x 2 (FMA) x 2.4 GHz


def flops(s, Hout, Wout, c=None):
    return 2.0 * s.N * Hout * Wout * s.K * s.R * s.S * (c or s.C)


def algorithmic_bytes(s, Hout, Wout):
    """Bytes one conv launch must move: input + packed filter + output + indirection entries, each once."""
    esz = {"f32": 4, "bf16": 2, "u8i8": 1}[s.dtype]
    M, T = s.N * Hout * Wout, s.R * s.S
    return s.N * s.Hin * s.Win * s.C * esz + s.K * T * s.C * esz + M * s.K * 4 + M * T * 4


def vendor_gemm_reference(torch, n=8192, iters=10):
    """TFLOP/s of the vendor library's bf16 GEMM (torch.matmul) on an n x n x n problem, on random and on all-zero
    matrices: what a tuned, compute-bound kernel sustains on this device with and without switching activity in its
    operands.  Context for the fractions of peak, nothing the library's own path uses."""
    res = {}
    for kind in ("random", "zeros"):
        make = torch.randn if kind == "random" else torch.zeros
        a = make(n, n, device="cuda:0", dtype=torch.bfloat16)
        b = make(n, n, device="cuda:0", dtype=torch.bfloat16)
        for _ in range(3):
            c = a @ b
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                c = a @ b
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) / iters
            best = t if best is None or t < best else best
        res[f"bf16_{kind}_TFLOPs"] = 2.0 * n ** 3 / (best * 1e-3) / 1e12
        del a, b, c
    torch.cuda.empty_cache()
    res["how"] = f"torch.matmul, {n} x {n} x {n} bfloat16, best of 3 x {iters} launches"
    return res


def vendor_gemm_only_ms(torch, M, red, K, dtype, iters=20):
    """ms of the vendor library's GEMM (torch.matmul) on a patch matrix that is already in memory: [M, red] x [red, K]
    on random data -- the "GEMM-only" measurement of section 3.2 with the machine's tuned GEMM in place of this
    library's.  As many copies of the patch matrix are rotated as it takes to exceed the last-level cache."""
    dt = {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]
    esz = 2 if dtype == "bf16" else 4
    sets = max(1, min(8, -(-(320 << 20) // (M * red * esz))))
    As = [torch.randn(M, red, device="cuda:0", dtype=dt) for _ in range(sets)]
    B = torch.randn(red, K, device="cuda:0", dtype=dt)
    outs = [torch.empty(M, K, device="cuda:0", dtype=dt) for _ in range(sets)]
    for i in range(3):
        torch.matmul(As[i % sets], B, out=outs[i % sets])
    best = None
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            torch.matmul(As[i % sets], B, out=outs[i % sets])
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) / iters
        best = t if best is None or t < best else best
    del As, B, outs
    torch.cuda.empty_cache()
    return best


def roofline(s, Hout, Wout, ms, kernel, name, measured_peak=None, measured_peak_varied=None):
    """The roofline object of one shape: which of HBM time (algorithmic bytes at 8 TB/s) and arithmetic time (its
    flops at the dtype's dense peak) is the longer bounds the kernel; `achieved` is that resource's rate at the
    measured duration."""
    fl = flops(s, Hout, Wout, getattr(s, "c_logical", 0) or None)
    ab = algorithmic_bytes(s, Hout, Wout)
    tensor = kernel.startswith(("mfma_", "gemm_"))
    peak = PEAK[s.dtype] if tensor else ALU_PEAK_F32
    if ab / (HBM_PEAK_GBS * 1e9) >= fl / (peak * 1e12):
        r = {"bound": "hbm", "achieved": ab / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        r = {"bound": "mfma" if tensor else "alu", "achieved": fl / (ms * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s"}
    r["frac"] = r["achieved"] / r["peak"]
    r["algorithmic_bytes"] = ab
    r["kernel"] = kernel
    rec = RECORDED_TRAFFIC.get(name)
    if rec and rec[0] == kernel:
        r["traffic"] = int((rec[1] * FETCH_SCALE + rec[2] * WRITE_SCALE) * 1024)
        r["traffic_source"] = TRAFFIC_SOURCE
    else:
        r["traffic"] = None
        r["traffic_source"] = "none recorded for this kernel"
    r["frac_of_hbm_peak"] = ab / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    if tensor:
        r["frac_of_mfma_peak"] = fl / (ms * 1e-3) / 1e12 / PEAK[s.dtype]
        if measured_peak and measured_peak.get(s.dtype):
            r["frac_of_measured_mfma_peak"] = fl / (ms * 1e-3) / 1e12 / measured_peak[s.dtype]
        if measured_peak_varied and measured_peak_varied.get(s.dtype):
            r["frac_of_measured_mfma_peak_varied_operands"] = fl / (ms * 1e-3) / 1e12 / measured_peak_varied[s.dtype]
    return r


class Problem:
    """Device buffers of one shape, `sets` rotating copies of everything a launch touches."""

    def __init__(self, icv, torch, s, sets=1, plan=0):
        from paper_1907_02129_amd.workloads import make_tensors
        self.icv, self.torch, self.s = icv, torch, s
        x, w = make_tensors(s)
        self.x_host, self.w_host = x, w
        self.wd = icv.to_device(w)
        self.bufs = [icv.prepare(s, self.wd, plan=plan) for _ in range(sets)]
        x0 = icv.to_device(x)
        self.xs = [x0] + [x0.clone() for _ in range(sets - 1)]
        self.p = self.bufs[0].p
        self.Hout, self.Wout = self.bufs[0].Hout, self.bufs[0].Wout
        self.i = 0

    def step(self):
        b, x = self.bufs[self.i], self.xs[self.i]
        self.i = (self.i + 1) % len(self.bufs)
        self.icv.conv2d_nhwc(b.p, x, b.packed, b.indirection, b.zero_row, b.output)

    def enable_fused(self):
        """Switch step() to the fused output stage: bias + ReLU, bfloat16 (uint8 for the int8 path) output."""
        icv, torch, s = self.icv, self.torch, self.s
        quant = s.dtype == "u8i8"
        self.bias = torch.zeros(s.K, dtype=torch.int32 if quant else torch.float32, device="cuda:0")
        self.narrow = [torch.empty(b.output.shape, dtype=torch.uint8 if quant else torch.bfloat16, device="cuda:0")
                       for b in self.bufs]
        self.ep = icv.make_epilogue(self.bias, True, icv.ICV_OUT_U8 if quant else icv.ICV_OUT_BF16, 1e-4, 128)

        def step():
            b, x, o = self.bufs[self.i], self.xs[self.i], self.narrow[self.i]
            self.i = (self.i + 1) % len(self.bufs)
            icv.conv2d_nhwc_fused(b.p, x, b.packed, b.indirection, b.zero_row, self.ep, o)
        self.step = step

    def time_steps(self, steps, warmup):
        """ms per step, HIP events on the launch stream around `steps` back-to-back launches."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            self.step()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def time_quantiles(self, repeats=25, inner=20, warmup=5):
        """Median and 20 % / 80 % quantiles over `repeats` timings (the paper's protocol), ms per launch."""
        for _ in range(warmup):
            self.step()
        ts = [self.time_steps(inner, 0) for _ in range(repeats)]
        return float(np.median(ts)), float(np.quantile(ts, 0.2)), float(np.quantile(ts, 0.8))

    def time_setup(self, reps=20):
        """ms per indirection build, replayed from a HIP graph over the buffer sets (the build is a single short
        kernel: issued call by call it would measure the host's launch rate)."""
        state = {"i": 0}

        def step():
            bb = self.bufs[state["i"] % len(self.bufs)]
            state["i"] += 1
            self.icv.setup_indirection(bb.p, bb.indirection)
        return graph_time(self.torch, step, max(reps, 2 * len(self.bufs)))

    def time_ablation(self, steps=20, warmup=3, graph_steps=0):
        """im2col + GEMM through the same MFMA core: (total ms, im2col ms, gemm ms), rotating over as many
        workspace / output sets as the indirect path rotates buffer sets (the same cache regime).  With
        graph_steps, that many calls are replayed from a HIP graph instead of being issued one by one."""
        torch, icv = self.torch, self.icv
        n = len(self.bufs)
        wss = [torch.empty(icv.im2col_bytes(self.p), dtype=torch.uint8, device="cuda:0") for _ in range(n)]
        outs = [torch.empty_like(b.output) for b in self.bufs]

        def timed(fn):
            if graph_steps:
                state = {"i": 0}

                def step():
                    fn(state["i"] % n)
                    state["i"] += 1
                return graph_time(torch, step, graph_steps)
            for i in range(warmup):
                fn(i % n)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(steps):
                fn(i % n)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / steps

        bufs, xs = self.bufs, self.xs
        t_all = timed(lambda i: icv.conv2d_nhwc_im2col(bufs[i].p, xs[i], bufs[i].packed, wss[i], outs[i]))
        t_i2c = timed(lambda i: icv.im2col(bufs[i].p, xs[i], wss[i]))
        t_gemm = timed(lambda i: icv.gemm_nhwc(bufs[i].p, wss[i], bufs[i].packed, outs[i]))
        return t_all, t_i2c, t_gemm


def sets_for_cold(s, Hout, Wout):
    per_set = algorithmic_bytes(s, Hout, Wout)
    return min(32, max(2, int(np.ceil(2.5 * LLC_BYTES / per_set))))


def graph_time(torch, step, per_replay, reps=9):
    """Median ms per step of `per_replay` steps captured into one HIP graph and replayed `reps` times: what the GPU
    needs for the launches, without the host's per-call cost (some 8 us through ctypes, more than the small layers'
    kernels take)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(per_replay):
            step()
    g.replay()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) / per_replay)
    return float(np.median(ts))


def layer_sweep(icv, torch, N, dtype="bf16"):
    """The distinct convolutions of ResNet-18 and SqueezeNet 1.0 (the paper's section 3.1, "Models", Table 2) with
    synthetic data at batch N: the Indirect Convolution, the im2col + GEMM algorithm and its GEMM part alone, as in
    the paper's figures 3 and 4, and the geometric means by layer type of its Tables 3 and 4 (performance of the
    Indirect GEMM primitive relative to the GEMM primitive).  Medians of 9 replays of a HIP graph of launches
    that rotate over the buffer sets (cold where the sets exceed the last-level cache)."""
    from paper_1907_02129_amd.workloads import resnet18_layers, squeezenet10_layers, layer_type
    layers, ratios = {}, {}
    for model, fn in (("resnet18", resnet18_layers), ("squeezenet10", squeezenet10_layers)):
        for sh in fn(N):
            if dtype != "bf16":
                sh = sh.with_(dtype=dtype)
            sh = icv.stored_for_tensor_cores(sh)       # bf16: 3 -> 4 and 48 -> 64 channels; fp32: 3 -> 16; zeros in the padding
            pp = icv.make_params(sh)
            ho, wo = icv.output_size(pp)
            nsets = min(sets_for_cold(sh, ho, wo), 12)
            pr = Problem(icv, torch, sh, sets=nsets)
            per_replay = 2 * nsets if nsets >= 5 else 12
            t_default = graph_time(torch, pr.step, per_replay)
            f = flops(sh, ho, wo, sh.c_logical or None)
            kind = layer_type(sh)
            row = {"type": kind, "M": sh.N * ho * wo, "C": sh.c_logical or sh.C, "K": sh.K,
                   "kernel": icv.plan_name(pp), "ms": t_default, "TFLOPs": f / (t_default * 1e-3) / 1e12}
            # the Indirect GEMM primitive proper (rows gathered through the buffer) where the default is another
            # form of it; the ablation runs with the tile the library picks for a plain GEMM
            pr_g = Problem(icv, torch, sh, sets=nsets, plan=icv.PLAN_GATHER)
            t_gather = t_default
            if icv.plan_name(pr_g.p) != icv.plan_name(pp):
                t_gather = graph_time(torch, pr_g.step, per_replay)
                row["per_element_gather_ms"] = t_gather
            ta, ti, tg = pr_g.time_ablation(graph_steps=per_replay)
            row["gemm_only_ms"] = tg
            if kind == "1x1 stride-1":
                # no im2col in the GEMM-based algorithm here (the patch matrix is the input tensor): the paper's
                # comparison is GEMM primitive against Indirect GEMM primitive
                t_gemm_based = t_default if row["kernel"].startswith("gemm_") else tg
                t_indirect = t_gather
                cls = "1x1 stride-1"
            else:
                row["im2col_gemm_ms"] = ta
                t_gemm_based, t_indirect = ta, t_default
                cls = "1x1 stride-2" if kind == "1x1 stride-2" else "non-1x1"
            row["indirect_vs_gemm_based"] = t_gemm_based / t_indirect
            row["indirect_vs_gemm_primitive"] = (t_gemm_based if cls == "1x1 stride-1" else tg) / t_indirect
            layers[sh.name] = row
            ratios.setdefault((model, cls), []).append((row["indirect_vs_gemm_primitive"],
                                                        row["indirect_vs_gemm_based"]))
            pr = pr_g = None
            torch.cuda.empty_cache()
    geo = {}
    for (model, cls), rs in ratios.items():
        a = np.array(rs)
        g = np.exp(np.log(a).mean(axis=0))
        geo.setdefault(model, {})[cls] = {"layers": len(rs),
                                          "indirect_gemm_vs_gemm_primitive_pct": (float(g[0]) - 1) * 100,
                                          "indirect_vs_gemm_based_algorithm_pct": (float(g[1]) - 1) * 100}
    return {"N": N, "dtype": dtype, "layers": layers, "geomean_by_type": geo}


def cpu_baseline(s, x, w, min_seconds=1.0, max_passes=20):
    """The oracle as it stands, timed on this host's cores on the headline workload: whole passes of the full
    problem until `min_seconds` of wall time (times the cores used: some 10-30 s of CPU work), best pass reported."""
    import oracle

    def one_pass():
        t0 = time.perf_counter()
        if s.dtype == "u8i8":
            oracle.conv2d_u8i8(s, x, w, s.zero_point)
        else:
            oracle.conv2d(s, x, w)
        return time.perf_counter() - t0

    times = []
    while len(times) < max_passes and (not times or sum(times) < min_seconds):
        times.append(one_pass())
    dt = min(times)
    Hout, Wout = oracle.out_extent(s)
    cores = oracle.num_threads()
    # one more pass on a single thread, the setting of the paper's own measurements (section 3.1)
    oracle.set_num_threads(1)
    dt1 = one_pass()
    oracle.set_num_threads(cores)
    return {"value": flops(s, Hout, Wout) / dt / 1e12, "unit": "TFLOP/s", "cores": cores,
            "single_thread": {"value": flops(s, Hout, Wout) / dt1 / 1e12, "seconds": round(dt1, 3)},
            "kind": "oracle", "seconds": round(dt, 3), "passes": len(times),
            "cpu_seconds_total": round(sum(times) * cores, 1),
            "sample": f"{len(times)} full passes of {s.name} (fp64 7-loop direct convolution, OpenMP over n,oy), "
                      f"fastest pass reported"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-shapes", action="store_true", help="skip the per-shape table and the ablation")
    ap.add_argument("--sweep", type=int, default=0, metavar="N",
                    help="add the ResNet-18 / SqueezeNet 1.0 layer sweep at batch N (section 3.1, Table 2)")
    ap.add_argument("--sweep-dtype", default="bf16", choices=["bf16", "f32"],
                    help="tensor type of the layer sweep (f32: the paper's own precision, section 3.1)")
    ap.add_argument("--workload", default=None, help="time another shape as the headline (tuning)")
    ap.add_argument("--plan", type=int, default=0)
    ap.add_argument("--batch", type=int, default=0, help="with --workload / --traffic-probe: the shape at another batch size")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: a 256 MiB device copy (calibration) then 10 conv launches")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path shards over the batch with no "
              "exchange step; multi-GPU figures are not produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1907_02129_amd import binding as icv
    from paper_1907_02129_amd.workloads import CONFIGS, HEADLINE
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    icv.load_library()
    torch.cuda.set_device(0)

    name = args.workload or HEADLINE
    s = CONFIGS[name]
    if args.batch > 0:
        s = s.with_(N=args.batch)
        name = f"{name}@N={args.batch}"
    if args.traffic_probe:
        # FETCH_SIZE / WRITE_SIZE calibration: a plain copy of known size (reads 256 MiB, writes 256 MiB),
        # then the conv kernel on rotating buffers; the counters of both are read from the same rocprofv3 run
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        pr = Problem(icv, torch, s, sets=sets_for_cold(s, *icv.output_size(icv.make_params(s, plan=args.plan))),
                     plan=args.plan)
        for _ in range(10):
            pr.step()
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": name, "kernel": icv.plan_name(pr.p), "copy_bytes": 256 << 20}))
        return
    p0 = icv.make_params(s, plan=args.plan)
    Hout, Wout = icv.output_size(p0)
    prob = Problem(icv, torch, s, sets=sets_for_cold(s, Hout, Wout), plan=args.plan)
    fl = flops(s, Hout, Wout, getattr(s, "c_logical", 0) or None)

    # ---- the timed region: exactly --steps launches between two synchronisations
    for _ in range(args.warmup):
        prob.step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        prob.step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms = e0.elapsed_time(e1) / args.steps          # average launch duration of the conv kernel
    value = fl / (ms * 1e-3) / 1e12

    warm = Problem(icv, torch, s, sets=1, plan=args.plan)
    ms_warm = warm.time_steps(args.steps, args.warmup)
    med, q20, q80 = prob.time_quantiles()
    t_setup = prob.time_setup()
    ind_bytes = icv.indirection_bytes(prob.p)      # everything the build writes: entries, range records, 16-bit form

    # what the matrix cores of this device deliver on register operands alone, TFLOP/s (TOP/s)
    # (constant operands: the least switching activity; pseudo-random operands: what real tensors cost in clock)
    measured_peak = {d: icv.measure_mfma_peak(d, 2) / 1e12 for d in ("bf16", "u8i8")}
    measured_peak_varied = {d: icv.measure_mfma_peak(d, 2, True) / 1e12 for d in ("bf16", "u8i8")}
    roof = roofline(s, Hout, Wout, ms, icv.plan_name(prob.p), name, measured_peak, measured_peak_varied)

    out = {
        "metric": "effective TFLOP/s (2*N*Hout*Wout*K*R*S*C / t)", "value": value, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "u8i8": "u8", "f32": "f32"}[s.dtype], "data": "synthetic",
        "config": {"workload": f"{name}: N={s.N} {s.Hin}x{s.Win} C={s.C} K={s.K} {s.R}x{s.S} "
                               f"stride {s.SY} dil {s.DY} pad {s.PT},{s.PL},{s.PB},{s.PR} {s.dtype}",
                   "cache_regime": f"cold: rotation over {len(prob.bufs)} buffer sets",
                   "kernel": icv.plan_name(prob.p)},
        "roofline": roof,
        "frac_of_mfma_peak": value / PEAK[s.dtype],
        "mfma_peak_measured": {"bf16_TFLOPs": measured_peak["bf16"], "u8i8_TOPs": measured_peak["u8i8"],
                               "bf16_TFLOPs_varied_operands": measured_peak_varied["bf16"],
                               "u8i8_TOPs_varied_operands": measured_peak_varied["u8i8"],
                               "how": "icv_measure_mfma_peak: register-only MFMA loop, 2 wavefronts per SIMD on every CU; "
                                      "constant operands, and pseudo-random operands that change with every instruction"},
        "vendor_gemm_reference": vendor_gemm_reference(torch),
        "wall_ms_per_step": wall_ms,
        "warm": {"ms_per_step": ms_warm, "value": fl / (ms_warm * 1e-3) / 1e12},
        "quantiles_ms": {"median": med, "q20": q20, "q80": q80, "repeats": 25, "launches_per_repeat": 20},
        "setup": {"indirection_build_ms": t_setup, "indirection_bytes": ind_bytes,
                  "indirection_GBps": ind_bytes / (t_setup * 1e-3) / 1e9,
                  "frac_of_hbm_peak": ind_bytes / (t_setup * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }

    if not args.no_shapes:
        shapes = {}
        # the eight benchmark shapes, and the headline shape with fp32 tensors (the paper's own precision, section 3.1)
        table = dict(CONFIGS)
        table[HEADLINE + "_f32"] = CONFIGS[HEADLINE].with_(name=HEADLINE + "_f32", dtype="f32")
        for nm, sh in table.items():
            pp = icv.make_params(sh)
            ho, wo = icv.output_size(pp)
            pr = Problem(icv, torch, sh, sets=min(sets_for_cold(sh, ho, wo), 12))
            m, a, b = pr.time_quantiles(repeats=15, inner=40, warmup=3)
            f = flops(sh, ho, wo, getattr(sh, "c_logical", 0) or None)
            ab = algorithmic_bytes(sh, ho, wo)
            row = {"kernel": icv.plan_name(pp), "ms": m, "q20": a, "q80": b, "TFLOPs": f / (m * 1e-3) / 1e12,
                   "frac_of_peak": f / (m * 1e-3) / 1e12 / PEAK[sh.dtype],
                   "GBps_algorithmic": ab / (m * 1e-3) / 1e9,
                   "frac_of_hbm_peak": ab / (m * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "roofline": roofline(sh, ho, wo, m, icv.plan_name(pp), nm, measured_peak, measured_peak_varied)}
            # the same launches replayed from a HIP graph: the GPU's time without the host's per-call cost (which is
            # what "ms" shows for problems that take less than a launch through ctypes, cfg1)
            nb = len(pr.bufs)
            row["graph_replay_ms"] = graph_time(torch, pr.step, 2 * nb if nb >= 5 else 12)
            if sh.dtype != "f32" or row["kernel"].startswith("mfma_"):
                # the same launch with the fused output stage (bias + ReLU, 2- or 1-byte output elements)
                pr.enable_fused()
                row["fused_bias_relu_narrow_out_ms"] = pr.time_quantiles(repeats=9, inner=40, warmup=3)[0]
            ts = pr.time_setup(reps=10)
            ib = icv.indirection_bytes(pp)          # everything the build writes: entries, range records, 16-bit form
            row["indirection_build_ms"] = ts
            row["indirection_GBps"] = ib / (ts * 1e-3) / 1e9
            if sh.dtype != "f32":
                # the ablation and the per-element-gather variant run with the tile the library picks for them
                # (the gather plan: rows fetched per kernel element), not with the pixel-range plan's tile
                pr_abl = Problem(icv, torch, sh, sets=min(len(pr.bufs), 12), plan=icv.PLAN_GATHER)
                if icv.plan_name(pr_abl.p) != icv.plan_name(pp):
                    row["per_element_gather_kernel"] = icv.plan_name(pr_abl.p)
                    row["per_element_gather_ms"] = pr_abl.time_quantiles(repeats=9, inner=40, warmup=3)[0]
                ta, ti, tg = pr_abl.time_ablation()
                row["im2col_gemm_ms"] = ta
                row["im2col_ms"] = ti
                row["gemm_only_ms"] = tg
                row["speedup_vs_im2col_gemm"] = ta / m
            if sh.dtype in ("bf16", "f32") and nm != "cfg1_tiny_f32":
                # reference only: the vendor library's GEMM on a patch matrix that costs nothing to make
                row["vendor_gemm_only_ms"] = vendor_gemm_only_ms(torch, sh.N * ho * wo, sh.R * sh.S * sh.C, sh.K, sh.dtype)
            if sh.N > 1 and not icv.plan_name(pp).startswith("gemm_"):
                # batch-independent indirection buffer (ICV_PLAN_PER_IMAGE): one image's entries serve the whole batch
                pr_img = Problem(icv, torch, sh, sets=min(len(pr.bufs), 12), plan=icv.PLAN_PER_IMAGE)
                row["per_image_buffer"] = {
                    "kernel": icv.plan_name(pr_img.p),
                    "ms": pr_img.time_quantiles(repeats=9, inner=40, warmup=3)[0],
                    "indirection_build_ms": pr_img.time_setup(reps=10),
                    "indirection_bytes": icv.indirection_bytes(pr_img.p),
                    "whole_batch_indirection_bytes": icv.indirection_bytes(pp)}
                pr_img = None
            shapes[nm] = row
            del pr
            pr_abl = None
            torch.cuda.empty_cache()
        out["shapes"] = shapes

    if not args.no_shapes:
        # The same kernels with enough work per launch for a steady state (batch 256): what they deliver once launch,
        # start-up and the last stores are a small share of the run.
        big = {}
        for nm in ("cfg2_3x3_c64", "cfg3a_3x3_s2", "cfg3b_3x3_d2", "cfg4_int8_3x3"):
            sh = CONFIGS[nm].with_(N=256)
            pp = icv.make_params(sh)
            ho, wo = icv.output_size(pp)
            pr = Problem(icv, torch, sh, sets=2)
            m = pr.time_quantiles(repeats=7, inner=10, warmup=3)[0]
            f = flops(sh, ho, wo)
            big[nm] = {"N": 256, "kernel": icv.plan_name(pp), "ms": m, "TFLOPs": f / (m * 1e-3) / 1e12,
                       "roofline": roofline(sh, ho, wo, m, icv.plan_name(pp), nm + "@N=256", measured_peak,
                                            measured_peak_varied)}
            # Diagnostic, never a result: the same launches on activations whose bytes are all zero.  Instructions, addresses
            # and bytes moved are identical; what changes is the switching activity in the matrix cores, hence the
            # power, hence the clock the device holds.  The gap to the row above is the share of the distance to the
            # peak that is the chip's power limit on this data, not idle cycles in the kernel.
            # In between: the same tensors after a ReLU (negative values, or codes below the zero point, replaced by
            # zero) -- what every convolution of the paper's two models but the first one reads.
            for x in pr.xs:
                x.clamp_(min=128 if sh.dtype == "u8i8" else 0)
            mr = pr.time_quantiles(repeats=7, inner=10, warmup=3)[0]
            big[nm]["relu_activations_diagnostic"] = {"ms": mr, "TFLOPs": f / (mr * 1e-3) / 1e12,
                                                      "frac_of_mfma_peak": f / (mr * 1e-3) / 1e12 / PEAK[sh.dtype]}
            for x in pr.xs:
                x.zero_()
            mz = pr.time_quantiles(repeats=7, inner=10, warmup=3)[0]
            big[nm]["zero_activations_diagnostic"] = {"ms": mz, "TFLOPs": f / (mz * 1e-3) / 1e12,
                                                      "frac_of_mfma_peak": f / (mz * 1e-3) / 1e12 / PEAK[sh.dtype]}
            del pr
            torch.cuda.empty_cache()
        out["batch_256"] = big

    if args.sweep > 0:
        out["layer_sweep"] = layer_sweep(icv, torch, args.sweep, args.sweep_dtype)

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(s, prob.x_host, prob.w_host)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
