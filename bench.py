#!/usr/bin/env python3
"""Benchmark of the binarized FC / convolution hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass over the BMM sweep of the benchmark configuration (square n = 2048 ... 16384 and
the FC shapes M in {8, 128, 1024} x 4096 x 4096), every shape once with the fused threshold ->
packed bits epilogue and once with int32 output; inputs are resident in HBM before the timed
region.  `value` is the binary-op rate of that whole step (2 ops per +1/-1 multiply-accumulate).
Timed outside those K steps and reported in the same JSON line: the two BConv layer shapes, the
binarized MLP (batch 1024 and 8) and the ResNet-18-shaped forward (batch 256), plus the CPU oracle
on a bounded sample of the sweep.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published dense peaks used as roofline denominators
PEAK_FP4_MFMA_TFLOPS = 10.1e3      # 4-bit float matrix cores, TFLOP/s (2 flop per MAC)
PEAK_HBM_GBS = 8000.0
PAPER_RESNET18_IMG_S = 5.6e3       # the paper's ResNet-18 throughput on an RTX 2080 (context only)
# Memory-side bytes per launch of the dominant kernel of the default sweep, from rocprofv3 FETCH_SIZE and
# WRITE_SIZE scaled by a plain copy (profiles/bmm_sweep_dominant_kernel_hbm_traffic.md); bench.py cannot
# read hardware counters itself, so the measured figure is carried here and reported only for that kernel
# in the default configuration.
TRAFFIC_DEFAULT_SWEEP = {"mfma_fp4_bmm_xlds_wg256x256": 5.409e+08,
                         # the same kernel on K-panel operands (profiles/bmm_sweep_k_panels_kernel_stats_and_counters.md)
                         "mfma_fp4_bmm_xlds_wg256x256_kpanels": 5.411e+08}
WIDE_KERNEL = "mfma_fp4_bmm_xlds_wg256x256"


# Table 6 of the paper, BTC-FMT row (RTX 2080; trained weights, real data): context only
PAPER_TABLE6_RTX2080 = {"cifar_vgg": {"latency8_ms": 0.338, "images_per_s": 3.85e4},
                        "cifar_resnet14": {"latency8_ms": 0.724, "images_per_s": 1.71e4},
                        "alexnet": {"latency8_ms": 2.326, "images_per_s": 3.77e3},
                        "vgg16": {"latency8_ms": 7.021, "images_per_s": 1.34e3}}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--skip-extras", action="store_true", help="only the BMM sweep (for profiling runs)")
    ap.add_argument("--skip-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--path", choices=["auto", "valu", "mfma"], default="auto", help="arithmetic path (profiling runs)")
    ap.add_argument("--shapes", default="", help="comma-separated subset of the sweep, e.g. sq8192 (profiling runs)")
    ap.add_argument("--variant", choices=["both", "bits", "int32"], default="both", help="epilogues to run (profiling runs)")
    ap.add_argument("--layout", choices=["rows", "panels"], default="rows",
                    help="panels: the shapes that take the 256x256-tile kernel get both operands (and write the packed "
                         "output) in the K-panel layout of bnn.h; the default line is measured on row-major operands")
    ap.add_argument("--only", default="", help="run only these extra sections (comma-separated: bconv, bconv_sweep, general, "
                                               "layout, mlp, resnet18, table5, cfg1; or roofline alone) and print them; the BMM sweep is skipped (profiling runs)")
    ap.add_argument("--resnet-batches", default="256,8", help="batch sizes of the ResNet-18 section (profiling runs)")
    ap.add_argument("--skip-trains", action="store_true",
                    help="no per-shape launch trains after the timed steps: the run then launches each sweep kernel "
                         "exactly (steps + warmup) times per shape and epilogue (profiling runs)")
    ap.add_argument("--table5-nets", default="cifar_vgg,cifar_resnet14,alexnet,vgg16", help="networks of the table5 section (profiling runs)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="only run a plain device copy of this many MiB three times (calibrates the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2006_16578_amd as bnn
    import workloads as wl

    bnn.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def to_dev(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(dev)

    if args.calib_copy_mib > 0:
        n = args.calib_copy_mib << 20
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "device copy", "bytes_read": n, "bytes_written": n, "launches": 3}))
        return 0

    rb = tuple(int(t) for t in args.resnet_batches.split(",") if t)
    t5 = set(t for t in args.table5_nets.split(",") if t)
    if args.only == "roofline":
        print(json.dumps({"only": "roofline", "measured_ceilings": run_roofline(bnn, torch, dev)}))
        return 0
    if args.only:
        print(json.dumps({"only": args.only, **run_extras(bnn, wl, np, torch, to_dev, dev, set(args.only.split(",")), rb, t5)}))
        return 0

    # ------------------------------------------------------------------ BMM sweep, resident in HBM
    path = {"auto": bnn.PATH_AUTO, "valu": bnn.PATH_VALU, "mfma": bnn.PATH_MFMA}[args.path]
    only = [t for t in args.shapes.split(",") if t]
    do_bits, do_i32 = args.variant in ("both", "bits"), args.variant in ("both", "int32")
    def sweep(layout, steps, warmup, trains):
        """One timed run of the sweep: warmup untimed steps, then `steps` timed ones; per-shape figures and the roofline
        of the kernel variant with the most time in a step."""
        shapes = []
        for name, M, N, K, _ in wl.cfg2_shapes():
            if only and name not in only:
                continue
            case = wl.cfg2_case(name)
            A, B, tau = to_dev(case["A"]), to_dev(case["B"]), to_dev(case["tau"])
            Cb = torch.empty((M, wl.round_up(wl.nwords(N), 4)), dtype=torch.int32, device=dev)
            C = torch.empty((M, N), dtype=torch.int32, device=dev)
            sh = {"name": name, "M": M, "N": N, "K": K, "A": A, "B": B, "tau": tau, "Cb": Cb, "C": C, "panels": False,
                  "kernel": bnn.bmm_kernel_name(M, N, K, path),
                  "kernel_i32": bnn.bmm_kernel_name(M, N, K, path, int32_out=True)}
            if layout == "panels" and sh["kernel"] == WIDE_KERNEL and sh["kernel_i32"] == WIDE_KERNEL:
                sh.update({"panels": True, "A": bnn.panels_from_rows(A, K), "B": bnn.panels_from_rows(B, K),
                           "Cb": torch.empty(((N + 255) // 256, M, 8), dtype=torch.int32, device=dev),
                           "kernel": WIDE_KERNEL + "_kpanels", "kernel_i32": WIDE_KERNEL + "_kpanels"})
                del A, B
            shapes.append(sh)
        macs_step = sum((do_bits + do_i32) * float(s["M"]) * s["N"] * s["K"] for s in shapes)

        def run_bits(s):
            if s["panels"]:
                bnn.bmm_thr_panels(s["A"], s["B"], s["tau"], s["K"], out=s["Cb"])
            else:
                bnn.bmm_thr(s["A"], s["B"], s["tau"], s["K"], out=s["Cb"], path=path)

        def run_i32(s):
            if s["panels"]:
                bnn.bmm_panels(s["A"], s["B"], s["K"], out=s["C"])
            else:
                bnn.bmm(s["A"], s["B"], s["K"], out=s["C"], path=path)

        def one_step(record: bool):
            for s in shapes:
                if record:
                    e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                    e0.record()
                if do_bits:
                    run_bits(s)
                if record:
                    e1.record()
                if do_i32:
                    run_i32(s)
                if record:
                    e2.record()
                    s["ev"].append((e0, e1, e2))

        for s in shapes:
            s["ev"] = []
        for _ in range(warmup):
            one_step(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            one_step(True)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / steps
        value_tops = macs_step * 2.0 / (ms_per_step * 1e-3) / 1e12

        # Per-shape figures.  A lone launch between two events reads no less than the launch gap of the stream, and a
        # Python loop of launches no less than the host's 10 us per call, so every shape is ALSO timed as a train of
        # launches queued behind a long-running kernel (_Train): `*_ms` is the GPU time per launch inside the train,
        # `*_single_launch_ms` the in-step figure (what one isolated call costs, launch gap included).
        per_shape = []
        train = None if not trains else _Train(bnn, torch, dev)
        for s in shapes:
            thr_1 = max(float(np.mean([a.elapsed_time(b) for a, b, _ in s["ev"]])), 1e-9) if do_bits else None
            i32_1 = max(float(np.mean([b.elapsed_time(c) for _, b, c in s["ev"]])), 1e-9) if do_i32 else None
            reps = lambda one_ms: int(min(200, max(5, 2.0 / max(one_ms, 1e-3))))
            thr_ms = (thr_1 if not trains else
                      train.time(lambda: run_bits(s), reps(thr_1))) if do_bits else None
            i32_ms = (i32_1 if not trains else
                      train.time(lambda: run_i32(s), reps(i32_1))) if do_i32 else None
            ops = 2.0 * s["M"] * s["N"] * s["K"]
            kw = wl.nwords(s["K"]) * 4
            bytes_thr = s["M"] * kw + s["N"] * kw + s["M"] * wl.nwords(s["N"]) * 4 + s["N"] * 4
            bytes_i32 = s["M"] * kw + s["N"] * kw + s["M"] * s["N"] * 4
            row = {"shape": s["name"], "M": s["M"], "N": s["N"], "K": s["K"]}
            if do_bits:
                row.update({"kernel": s["kernel"], "bits_out_ms": round(thr_ms, 5), "bits_out_single_launch_ms": round(thr_1, 5),
                            "bits_out_tops": round(ops / thr_ms / 1e9, 2),
                            "bits_out_frac_fp4_mfma_peak": round(ops / thr_ms / 1e9 / PEAK_FP4_MFMA_TFLOPS, 4),
                            "bits_out_hbm_gbs": round(bytes_thr / thr_ms / 1e6, 1),
                            "bits_out_frac_hbm_peak": round(bytes_thr / thr_ms / 1e6 / PEAK_HBM_GBS, 4)})
            if do_i32:
                row.update({"int32_out_kernel": s["kernel_i32"], "int32_out_ms": round(i32_ms, 5),
                            "int32_out_single_launch_ms": round(i32_1, 5), "int32_out_tops": round(ops / i32_ms / 1e9, 2),
                            "int32_out_frac_fp4_mfma_peak": round(ops / i32_ms / 1e9 / PEAK_FP4_MFMA_TFLOPS, 4),
                            "int32_out_hbm_gbs": round(bytes_i32 / i32_ms / 1e6, 1),
                            "int32_out_frac_hbm_peak": round(bytes_i32 / i32_ms / 1e6 / PEAK_HBM_GBS, 4)})
            row["in_step_ms"] = {"bits": round(thr_1, 5) if do_bits else None, "int32": round(i32_1, 5) if do_i32 else None}
            per_shape.append(row)

        # roofline of the dominant kernel: the launches (both epilogues) of the kernel variant that
        # takes the most time in a step
        by_kernel = {}
        for s, ps in zip(shapes, per_shape):
            kw = (s["M"] + s["N"]) * wl.nwords(s["K"]) * 4
            # launch durations measured inside the timed region (events on the launch stream around every launch)
            for on, kern, ms, out_bytes in ((do_bits, s["kernel"], ps["in_step_ms"]["bits"], s["M"] * wl.nwords(s["N"]) * 4),
                                            (do_i32, s["kernel_i32"], ps["in_step_ms"]["int32"], 4 * s["M"] * s["N"])):
                if on:
                    d = by_kernel.setdefault(kern, {"ms": 0.0, "flop": 0.0, "launches": 0, "bytes": 0})
                    d["ms"] += ms
                    d["flop"] += 2.0 * s["M"] * s["N"] * s["K"]
                    d["launches"] += 1
                    d["bytes"] += kw + out_bytes
        dom = max(by_kernel, key=lambda k: by_kernel[k]["ms"])
        dk = by_kernel[dom]
        achieved = dk["flop"] / (dk["ms"] * 1e-3) / 1e12
        probe_buf = torch.empty(4 << 20, dtype=torch.uint8, device=dev)
        measured_peak = bnn.probe_pipeline("mfma_fp4", probe_buf, iters=4000)[0] / 1e12
        measured_loop = bnn.probe_pipeline("mfma_fp4_expand", probe_buf, iters=4000)[0] / 1e12
        del probe_buf
        roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 1), "peak": PEAK_FP4_MFMA_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP4_MFMA_TFLOPS, 4),
                    "measured_peak": round(measured_peak, 1), "frac_of_measured_peak": round(achieved / measured_peak, 4),
                    "measured_expand_plus_mfma_loop": round(measured_loop, 1),
                    "frac_of_measured_loop": round(achieved / measured_loop, 4),
                    "traffic": (TRAFFIC_DEFAULT_SWEEP.get(dom) if (args.path == "auto" and not only and args.variant == "both")
                                else None),   # keyed by kernel AND layout (the panel runs carry the _kpanels name)
                    "algorithmic_bytes_per_launch": round(dk["bytes"] / max(dk["launches"], 1)),
                    "avg_launch_ms": round(dk["ms"] / dk["launches"], 5), "launches_per_step": dk["launches"],
                    "flop_per_launch": dk["flop"] / dk["launches"],
                    "note": "peak: published fp4 (E2M1) dense matrix-core rate; measured_peak: the same MFMA alone, register-"
                            "resident, in this run; measured_expand_plus_mfma_loop: the kernel's inner loop without memory "
                            "(bnn_probe_pipeline); 1 MAC on +1/-1 = 2 flop = 2 binary ops"}

        return value_tops, ms_per_step, per_shape, roofline

    value_tops, ms_per_step, per_shape, roofline = sweep(args.layout, args.steps, args.warmup, not args.skip_trains)

    extras = {}
    if args.layout == "rows" and not args.skip_extras and args.path == "auto":
        # the same sweep once more with the large squares in the K-panel layout (Sec. 5.1: the paper reports its
        # products on its own fixed-stride format beside the general one); not the `value` of this line
        v2, ms2, ps2, rf2 = sweep("panels", args.steps, args.warmup, False)
        conv = []
        for n in (4096, 16384):
            X = torch.randint(-2**31, 2**31 - 1, (n, n // 32), dtype=torch.int32, device=dev)
            Xp = bnn.panels_from_rows(X, n)
            t_to = _time_gpu(torch, lambda: bnn.panels_from_rows(X, n), 10)
            t_back = _time_gpu(torch, lambda: bnn.rows_from_panels(Xp, n), 10)
            conv.append({"rows": n, "K": n, "panels_from_rows_ms": round(t_to, 5), "rows_from_panels_ms": round(t_back, 5)})
            del X, Xp
        extras["bmm_sweep_k_panels"] = {
            "value": round(v2, 2), "unit": "binary TOPS", "ms_per_step": round(ms2, 4), "roofline": rf2,
            "shapes_in_panels": [r for r in ps2 if r.get("kernel", r.get("int32_out_kernel", "")).endswith("_kpanels")],
            "conversion": conv,
            "note": "operands resident in HBM in the K-panel layout (bnn_panels_from_rows, done once and not timed, as "
                    "for weights and for activations produced by bnn_bmm_thr_panels); the other shapes row-major as above"}
    if not args.skip_extras:
        extras.update(run_extras(bnn, wl, np, torch, to_dev, dev, None, rb, t5))
    cpu = None
    if not args.skip_cpu:
        cpu = cpu_baseline(wl, np)
        extras["cpu_oracle_per_shape"] = cpu_oracle_detail(wl, np)

    line = {
        "metric": "binary TOPS for BMM/BConv (fraction of roofline); BNN ResNet-18 images/s",
        "value": round(value_tops, 2), "unit": "binary TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u1 (+1/-1 bits as fp4 E2M1 on the matrix cores, fp32/int32 accumulate)", "data": "synthetic",
        "config": {"workload": "BMM sweep (config 2): square n in {2048,4096,8192,16384} + FC M in {8,128,1024} x "
                               "K=4096 x N=4096; each shape with fused threshold->bits and with int32 output; "
                               "uniform random bits, seeded", "path": args.path,
                   "shapes": args.shapes or "all", "variant": args.variant,
                   "layout": "row-major packed words" if args.layout == "rows" else
                             "K panels of 256 bits for the shapes of the 256x256-tile kernel, row-major for the others"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "bmm_shapes": per_shape,
    }
    line.update(extras)
    print(json.dumps(line))
    return 0


def run_roofline(bnn, torch, dev):
    """The measured ceilings of this chip for every pipeline the library uses or decided against (bnn_probe_pipeline)."""
    small = torch.empty(4 << 20, dtype=torch.uint8, device=dev)
    big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)       # well beyond the 256 MB last-level cache
    out = {}
    for name, buf, unit, scale, pub in (
            ("mfma_fp4", small, "PFLOP/s", 1e15, 10.1), ("mfma_fp4_expand", small, "PFLOP/s", 1e15, None),
            ("mfma_i8", small, "POP/s", 1e15, 5.0), ("mfma_bf16", small, "PFLOP/s", 1e15, 2.5),
            ("valu_xor_popc", small, "binary POP/s", 1e15, 1.26), ("lds_read", small, "TB/s", 1e12, None),
            ("hbm_read", big, "TB/s", 1e12, 8.0), ("hbm_write", big, "TB/s", 1e12, 8.0), ("hbm_copy", big, "TB/s", 1e12, 8.0)):
        rate, sec = bnn.probe_pipeline(name, buf, iters=4000)
        out[name] = {"measured": round(rate / scale, 3), "unit": unit, "launch_ms": round(sec * 1e3, 4)}
        if pub is not None:
            out[name]["published_or_derived_peak"] = pub
            out[name]["frac"] = round(rate / scale / pub, 3)
    out["notes"] = ("mfma_fp4_expand = 8 MFMAs + 6 word expansions per K-step of a 4x2 wave tile, no memory traffic; "
                    "valu_xor_popc peak derived: 256 CUs x 64 lanes x 2.4 GHz x 32 bits / 2 instructions x 2 ops; "
                    "hbm_copy counts bytes read + written")
    return out


def _time_gpu(torch, fn, iters, warmup=3):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


class _Train:
    """Device time per launch of a small kernel.  Launching from Python costs about 10 us per call, more than such
    a kernel runs, so a plain loop measures the host.  Here a long-running kernel is enqueued first; while it
    keeps the GPU busy the host enqueues `n` launches of `fn` behind it, and the events on either side of the
    train then bracket GPU time only (kernel time plus the command processor's gap between dependent launches)."""

    def __init__(self, bnn, torch, dev):
        self.bnn, self.torch = bnn, torch
        self.buf = torch.empty(4 << 20, dtype=torch.uint8, device=dev)
        self.iters = 4000
        rate, sec = bnn.probe_pipeline("mfma_i8", self.buf, iters=self.iters, reps=1)
        self.iters = max(1000, int(self.iters * 4e-3 / sec))          # a blocker of about 4 ms

    def time(self, fn, n=100):
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            self.bnn.probe_pipeline_enqueue("mfma_i8", self.buf, self.iters)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / n
            best = ms if best is None else min(best, ms)
        return best


def _time_graph(torch, fn, iters):
    """The same call captured once into a HIP graph and replayed: per-layer launch cost without the host."""
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    torch.cuda.synchronize()
    return _time_gpu(torch, g.replay, iters)


def run_extras(bnn, wl, np, torch, to_dev, dev, only=None, resnet_batches=(256, 8), table5_nets=None):
    out = {}

    def want(section):
        return only is None or section in only

    # ---- config 1 (BMM 1024^3): latency-bound; one isolated launch and a train of 100
    if want("cfg1"):
        case = wl.cfg1()
        A, B, tau = to_dev(case["A"]), to_dev(case["B"]), to_dev(case["tau"])
        C = torch.empty((1024, 1024), dtype=torch.int32, device=dev)
        Cb = torch.empty((1024, 32), dtype=torch.int32, device=dev)
        ops = 2.0 * 1024 ** 3
        r = {"kernel": bnn.bmm_kernel_name(1024, 1024, 1024), "int32_out_kernel": bnn.bmm_kernel_name(1024, 1024, 1024, int32_out=True)}
        for key, fn, nbytes in (("int32_out", lambda: bnn.bmm(A, B, 1024, out=C), 2 * 131072 + 4 * 1024 * 1024),
                                ("bits_out", lambda: bnn.bmm_thr(A, B, tau, 1024, out=Cb), 3 * 131072)):
            single = float(np.median([_time_gpu(torch, fn, 1, warmup=1) for _ in range(20)]))
            train = _Train(bnn, torch, dev).time(fn, 100)
            r[key] = {"single_launch_ms": round(single, 5), "train_of_100_ms_per_launch": round(train, 5),
                      "note": "train: 100 launches queued behind a long-running kernel, GPU time per launch",
                      "tops_in_train": round(ops / train / 1e9, 1),
                      "frac_fp4_mfma_peak_in_train": round(ops / train / 1e9 / PEAK_FP4_MFMA_TFLOPS, 4),
                      "hbm_gbs_in_train": round(nbytes / train / 1e6, 1),
                      "frac_hbm_peak_in_train": round(nbytes / train / 1e6 / PEAK_HBM_GBS, 4)}
        out["bmm_1024_config1"] = r
        del A, B, C, Cb
    # ---- single BConv layers (config 4)
    if want("bconv"):
        convs = []
        for name, case in (("conv_56x56_c128_o128_s1", wl.cfg4a()), ("conv_56x56_c64_o128_s2", wl.cfg4b())):
            x, f, tau = to_dev(case["x"]), to_dev(case["filt"]), to_dev(case["tau"])
            N, H, W, C, O, k, st, pad = (case[q] for q in ("N", "H", "W", "C", "O", "k", "stride", "pad"))
            P, Q = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
            bits = torch.empty((N, P, Q, wl.nwords(O)), dtype=torch.int32, device=dev)
            y = torch.empty((N, P, Q, O), dtype=torch.int32, device=dev)
            ops = 2.0 * N * P * Q * O * k * k * C
            tr = _Train(bnn, torch, dev)
            t_b = tr.time(lambda: bnn.bconv_thr(x, f, tau, C, st, pad, bnn.PAD_MINUS_ONE, out=bits), 50)
            t_i = tr.time(lambda: bnn.bconv(x, f, C, st, pad, bnn.PAD_MINUS_ONE, out=y), 50)
            convs.append({"shape": name, "kernel": bnn.bconv_kernel_name(N, H, W, C, O, k, st, pad),
                          "bits_out_ms": round(t_b, 5), "bits_out_tops": round(ops / t_b / 1e9, 2),
                          "bits_out_frac_fp4_mfma_peak": round(ops / t_b / 1e9 / PEAK_FP4_MFMA_TFLOPS, 4),
                          "int32_out_ms": round(t_i, 5), "int32_out_tops": round(ops / t_i / 1e9, 2),
                          "bits_out_hbm_gbs": round((x.numel() + bits.numel() + f.numel()) * 4 / t_b / 1e6, 1),
                          "bits_out_frac_hbm_peak": round((x.numel() + bits.numel() + f.numel()) * 4 / t_b / 1e6 / PEAK_HBM_GBS, 4),
                          "int32_out_hbm_gbs": round((y.numel() * 4 + x.numel() * 4) / t_i / 1e6, 1),
                          "int32_out_frac_hbm_peak": round((y.numel() * 4 + x.numel() * 4) / t_i / 1e6 / PEAK_HBM_GBS, 4)})
            del x, f, bits, y
        out["bconv_shapes"] = convs
    # ---- the paper's BConv sweep (Sec. 7.3): batch 16, 64x64 input, 3x3, stride 1, C = O
    if want("bconv_sweep"):
        sweep = []
        for ch in (128, 256, 512, 640, 1024, 2048):
            case = wl.bconv_case(6, 16, 64, 64, ch, ch, 3, 1, 1, index0=ch % 97)
            x, f, tau = to_dev(case["x"]), to_dev(case["filt"]), to_dev(case["tau"])
            bits = torch.empty((16, 64, 64, wl.nwords(ch)), dtype=torch.int32, device=dev)
            ops = 2.0 * 16 * 64 * 64 * ch * 9 * ch
            t_b = _time_gpu(torch, lambda: bnn.bconv_thr(x, f, tau, ch, 1, 1, bnn.PAD_MINUS_ONE, out=bits), 10)
            sweep.append({"C=O": ch, "kernel": bnn.bconv_kernel_name(16, 64, 64, ch, ch, 3, 1, 1), "bits_out_ms": round(t_b, 5),
                          "bits_out_tops": round(ops / t_b / 1e9, 1),
                          "bits_out_frac_fp4_mfma_peak": round(ops / t_b / 1e9 / PEAK_FP4_MFMA_TFLOPS, 4)})
            del x, f, bits
        out["bconv_sweep_batch16_64x64_3x3"] = sweep
    # ---- "general" forms (Sec. 7.2 / 7.3): real-valued operands binarized on the way in, fp32 result
    if want("general"):
        gen = []
        for n in (2048, 4096, 8192):
            A = torch.randn((n, n), dtype=torch.float32, device=dev)
            B = torch.randn((n, n), dtype=torch.float32, device=dev)
            C = torch.empty((n, n), dtype=torch.float32, device=dev)
            ws = torch.empty(2 * n * n // 8 + 1024, dtype=torch.uint8, device=dev)
            t = _time_gpu(torch, lambda: bnn.bmm_general_f32(A, B, out=C, workspace=ws), 10)
            tp = _time_gpu(torch, lambda: bnn.sign_pack_f32(A), 10)
            gen.append({"shape": "bmm_sq%d" % n, "ms": round(t, 5), "tops": round(2.0 * n ** 3 / t / 1e9, 1),
                        "binarize_one_operand_ms": round(tp, 5),
                        "hbm_gbs": round((3 * n * n * 4 + 4 * n * n / 8) / t / 1e6, 1)})
            del A, B, C, ws
        for ch in (128, 512):
            x = torch.randn((16, 64, 64, ch), dtype=torch.float32, device=dev)
            f = torch.randn((ch, 3, 3, ch), dtype=torch.float32, device=dev)
            o = torch.empty((16, 64, 64, ch), dtype=torch.float32, device=dev)
            ws = torch.empty((x.numel() + f.numel()) // 8 + 1024, dtype=torch.uint8, device=dev)
            t = _time_gpu(torch, lambda: bnn.bconv_general_f32(x, f, 1, 1, out=o, workspace=ws), 10)
            gen.append({"shape": "bconv_batch16_64x64_3x3_c%d" % ch, "ms": round(t, 5),
                        "tops": round(2.0 * 16 * 64 * 64 * ch * 9 * ch / t / 1e9, 1)})
            del x, f, o, ws
        out["general_f32_in_f32_out"] = gen
    # ---- layout study (Sec. 5.1 / 4.1 redone for this chip): weights pre-tiled in MFMA fragment order against plain
    if want("layout"):
        # rows on the shapes that read operands straight from L2, and the fragment-load latency against the row stride
        # (GPU time per launch in a train behind a long-running kernel: the small shapes run shorter than a host launch)
        lay = {"fc_shapes": [], "fragment_load_ticks_vs_row_stride_bytes": {}}
        train = _Train(bnn, torch, dev)
        for (M, N, K) in ((8, 4096, 4096), (128, 4096, 4096), (1024, 1024, 1024), (1024, 4096, 4096), (4096, 4096, 4096),
                          (8192, 8192, 8192)):
            case = wl.bmm_case(2, M, N, K, index0=900 + M % 7)
            A, B, tau = to_dev(case["A"]), to_dev(case["B"]), to_dev(case["tau"])
            Bt = bnn.tile_b(B, K)
            Ap, Bp = bnn.panels_from_rows(A, K), bnn.panels_from_rows(B, K)
            o = torch.empty((M, wl.round_up(wl.nwords(N), 4)), dtype=torch.int32, device=dev)
            op = torch.empty(((N + 255) // 256, M, 8), dtype=torch.int32, device=dev)
            n = 100 if M * N <= (1 << 22) else 20
            t_rows = train.time(lambda: bnn.bmm_thr(A, B, tau, K, out=o), n)
            t_tile = train.time(lambda: bnn.bmm_thr_tiled(A, Bt, tau, N, K, out=o), n)
            t_pan = train.time(lambda: bnn.bmm_thr_panels(Ap, Bp, tau, K, out=op), n)
            lay["fc_shapes"].append({"M": M, "N": N, "K": K, "rows_kernel": bnn.bmm_kernel_name(M, N, K),
                                     "rows_ms": round(t_rows, 5), "pretiled_direct_ms": round(t_tile, 5),
                                     "k_panels_wg256x256_ms": round(t_pan, 5),
                                     "rows_tops": round(2.0 * M * N * K / t_rows / 1e9, 1),
                                     "pretiled_tops": round(2.0 * M * N * K / t_tile / 1e9, 1),
                                     "k_panels_tops": round(2.0 * M * N * K / t_pan / 1e9, 1)})
            del A, B, Bt, Ap, Bp, o, op
        del train
        for stride in (32, 48, 64, 96, 128, 256, 512, 1024, 2048, 2064, 4096):
            lay["fragment_load_ticks_vs_row_stride_bytes"][str(stride)] = {
                "dependent": round(bnn.probe_load_stride(stride, iters=8192, dependent=True), 1),
                "eight_in_flight": round(bnn.probe_load_stride(stride, iters=8192, dependent=False), 1),
                "dependent_16KiB_footprint": round(bnn.probe_load_stride(stride, iters=8192, dependent=True, footprint_bytes=16384), 1)}
        out["layout_study"] = lay
    # ---- binarized MLP (config 3)
    if want("mlp"):
        params = wl.mlp_params()
        net = bnn.Net()
        net.input_u8(784, 127)
        for l in range(4):
            net.add_fc(to_dev(params["W"][l]), to_dev(params["thr"][l]) if l < 3 else None, params["K"][l])
        mlp = {}
        for batch in (32768, 1024, 8):
            imgs = to_dev(wl.mlp_images(batch))
            o = torch.empty((batch, 10), dtype=torch.int32, device=dev)
            t = _time_gpu(torch, lambda: net.forward(imgs, out=o), 50)
            # one cooperative launch for the whole network (Sec. 6.2), with and without its device-wide barriers
            # (without: results undefined, timing only -- the way the paper's Table 10 prices synchronisation)
            tp = _time_gpu(torch, lambda: net.forward_persistent(imgs, out=o), 50)
            tn = _time_gpu(torch, lambda: net.forward_persistent(imgs, out=o, no_sync=True), 50)
            net.forward(imgs, out=o)
            mlp["batch%d" % batch] = {"ms": round(min(t, tp), 5), "images_per_s": round(batch / min(t, tp) * 1e3, 1),
                                      "per_layer_launches_ms": round(t, 5), "persistent_kernel_ms": round(tp, 5),
                                      "persistent_without_barriers_ms": round(tn, 5),
                                      "barrier_share_of_persistent": round(max(tp - tn, 0.0) / tp, 3)}
            if batch == 8:
                tg = _time_graph(torch, lambda: net.forward(imgs, out=o), 50)
                mlp["batch8"]["hip_graph_replay_ms"] = round(tg, 5)
            del imgs, o
        mlp["paper_rtx2080_btc_fmt_context_only"] = {"latency8_ms": 0.055, "images_per_s_batch1024": 5.48e6,
                                                     "images_per_s_batch32k": 7.62e6, "sync_share": 0.0826}
        out["mlp_784_1024x3_10"] = mlp
    # ---- ResNet-18-shaped forward (config 5), batch 256
    if want("resnet18"):
        p = wl.resnet18_params()
        rnet = bnn.Net()
        rnet.input_conv_f32(to_dev(p["stem_w"]), to_dev(p["stem_thr"]), 224, 224, 4, 3)
        for blk in p["blocks"]:
            rnet.add_block(to_dev(blk["W1"]), to_dev(blk["thr1"]), to_dev(blk["W2"]), to_dev(blk["thr2"]),
                           to_dev(blk["Wd"]) if "Wd" in blk else None, blk["cin"], blk["cout"], blk["stride"])
        rnet.add_head_f32(to_dev(p["fc_w"]))
        res = {}
        for batch in resnet_batches:
            x = to_dev(wl.resnet18_input(batch))
            o = torch.empty((batch, 1000), dtype=torch.float32, device=dev)
            t = _time_gpu(torch, lambda: rnet.forward(x, out=o), 10 if batch == 256 else 30)
            res["batch%d" % batch] = {"ms": round(t, 4), "images_per_s": round(batch / t * 1e3, 1)}
            if batch == 8:
                tg = _time_graph(torch, lambda: rnet.forward(x, out=o), 30)
                res["batch8"]["hip_graph_replay_ms"] = round(tg, 4)
                # Sec. 6.2 / Table 10 for a residual network: all 16 block convolutions as ONE persistent kernel
                # (stem and head stay ordinary launches), against one launch per layer; the same kernel with its
                # barriers switched off prices the synchronisation (results undefined, timing only)
                pers = {}
                for cap in (32, 64, 128, 256):
                    tp = _time_gpu(torch, lambda: rnet.forward_persistent(x, out=o, grid_cap=cap), 30)
                    tn = _time_gpu(torch, lambda: rnet.forward_persistent(x, out=o, grid_cap=cap, no_sync=True), 30)
                    pers["grid_%d" % cap] = {"ms": round(tp, 4), "without_barriers_ms": round(tn, 4),
                                             "barrier_share": round(max(tp - tn, 0.0) / tp, 3)}
                res["batch8"]["persistent_blocks_kernel"] = pers
            if batch == 256:
                xs, w, th = x, to_dev(p["stem_w"]), to_dev(p["stem_thr"])
                ts = _time_gpu(torch, lambda: bnn.conv_f32_split_thr(xs, w, th, 4, 3, products=6), 5)
                ts9 = _time_gpu(torch, lambda: bnn.conv_f32_split_thr(xs, w, th, 4, 3, products=9), 5)
                tsf = _time_gpu(torch, lambda: bnn.conv_f32_thr(xs, w, th, 4, 3), 5)
                res["batch256"]["stem_fp32_ms"] = round(ts, 4)                    # as the forward runs it: bf16 x 3 split, six term products
                res["batch256"]["stem_all_nine_products_ms"] = round(ts9, 4)     # every term product: exact products
                res["batch256"]["stem_on_fp32_mfma_ms"] = round(tsf, 4)           # the same layer on the fp32 matrix cores
                res["batch256"]["binarized_layers_tops"] = round(2 * 1.70e9 * batch / max(t - ts, 1e-6) / 1e9, 1)
            del x
        res["paper_rtx2080_images_per_s_context_only"] = PAPER_RESNET18_IMG_S
        out["resnet18_224"] = res
        del rnet
    # ---- the other network shapes of the paper's Table 5: 8-image latency and throughput at the paper's batch sizes
    if want("table5"):
        t5 = {}
        for name, big in (("cifar_vgg", 1024), ("cifar_resnet14", 1024), ("alexnet", 512), ("vgg16", 512)):
            if table5_nets is not None and name not in table5_nets:
                continue
            spec = wl.cnn_layers(name)
            net5 = bnn.Net.from_layers(spec["layers"], spec["in_hw"], device=dev)
            r = {}
            for batch in (big, 8):
                x = to_dev(wl.cnn_input(name, batch))
                persistent_ok = batch == 8 and name in ("cifar_vgg", "cifar_resnet14")
                o = torch.empty((batch, spec["classes"]), dtype=torch.int32, device=dev)
                t = _time_gpu(torch, lambda: net5.forward(x, out=o), 5 if batch == big else 20)
                r["batch%d" % batch] = {"ms": round(t, 4), "images_per_s": round(batch / t * 1e3, 1)}
                if persistent_ok:       # runs of layers between pools as persistent kernels (Sec. 6.2), as for ResNet-18
                    tp = _time_gpu(torch, lambda: net5.forward_persistent(x, out=o), 20)
                    tn = _time_gpu(torch, lambda: net5.forward_persistent(x, out=o, no_sync=True), 20)
                    r["batch8"]["persistent_runs_ms"] = round(tp, 4)
                    r["batch8"]["persistent_without_barriers_ms"] = round(tn, 4)
                    r["batch8"]["barrier_share_of_persistent"] = round(max(tp - tn, 0.0) / tp, 3)
                if batch == big:
                    # the first layer alone: binarized weights on the bf16 matrix cores (what the network uses, Sec. 6.1),
                    # and the same shape with real-valued weights on the fp32 matrix cores
                    L0 = spec["layers"][0]
                    wb, t0 = to_dev(L0["W"]), to_dev(L0["thr"])
                    O0, k0 = L0["W"].shape[0], L0["W"].shape[1]
                    wf = torch.randn((O0, k0, k0, L0["C"]), dtype=torch.float32, device=dev) * 0.05
                    tb = _time_gpu(torch, lambda: bnn.bwn_conv_thr(x, wb, t0, L0["C"], L0["stride"], L0["pad"]), 5)
                    tf = _time_gpu(torch, lambda: bnn.conv_f32_thr(x, wf, t0, L0["stride"], L0["pad"]), 3)
                    hw0 = (spec["in_hw"] + 2 * L0["pad"] - k0) // L0["stride"] + 1
                    flop = 2.0 * batch * hw0 * hw0 * O0 * k0 * k0 * L0["C"]
                    r["batch%d" % batch]["first_layer_bwn_ms"] = round(tb, 4)
                    r["batch%d" % batch]["first_layer_bwn_tflops"] = round(flop / tb / 1e9, 1)
                    r["batch%d" % batch]["first_layer_bwn_hbm_gbs"] = round(
                        (x.numel() * 4 + batch * hw0 * hw0 * O0 / 8) / tb / 1e6, 1)
                    r["batch%d" % batch]["same_shape_fp32_weights_ms"] = round(tf, 4)
                del x, o
            r["paper_rtx2080_btc_fmt_context_only"] = PAPER_TABLE6_RTX2080[name]
            t5[name] = r
            del net5
        out["table5_networks"] = t5
    return out


def cpu_baseline(wl, np):
    """The CPU oracle (tier 0: naive +1/-1 int8 loops, OpenMP over rows) timed on a bounded sample
    of the same sweep: the first 768 rows of A of every shape (all rows where M < 768)."""
    import oracle as orc
    orc.build()
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    macs = 0.0
    secs = 0.0
    for name, M, N, K, _ in wl.cfg2_shapes():
        case = wl.cfg2_case(name)
        rows = min(M, 768)
        t0 = time.perf_counter()
        orc.bmm_rows(case["A"], case["B"], K, 0, rows)
        secs += time.perf_counter() - t0
        macs += float(rows) * N * K
    return {"value": round(2.0 * macs / secs / 1e12, 5), "unit": "binary TOPS", "cores": cores, "kind": "oracle",
            "seconds": round(secs, 2),
            "sample": "tier-0 oracle (unpacked int8 +1/-1, naive loops, includes unpacking B) on the first 768 rows of A "
                      "of every sweep shape (all rows where M < 768), int32 output"}


def cpu_oracle_detail(wl, np):
    """The CPU oracle per shape, next to the GPU figures (a baseline, never the target): the packed tier-1 oracle
    (uint64 xor + popcount, plain C, OpenMP over rows) in full on every sweep shape; the naive tier-0 oracle
    (+1/-1 as int8) in full where that takes seconds, else on a slab of rows / images scaled linearly and labelled
    extrapolated; config 1 also on a single thread."""
    import ctypes

    import oracle as orc
    from oracle import nets
    orc.build()
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    gomp = ctypes.CDLL("libgomp.so.1")

    def timed(fn):
        t0 = time.perf_counter()
        fn()
        return time.perf_counter() - t0

    out = {"cores": cores, "bmm": [], "note": "seconds on the host CPU; tops = binary TOPS = 2 x bit-MAC/s / 1e12"}
    for name, M, N, K, _ in [("cfg1_sq1024", 1024, 1024, 1024, 0)] + wl.cfg2_shapes():
        case = wl.cfg1() if name == "cfg1_sq1024" else wl.cfg2_case(name)
        macs = float(M) * N * K
        row = {"shape": name}
        rows1 = M if macs <= 6e11 else M // 8                 # tier 1 in full up to n = 8192
        t1 = timed(lambda: orc.bmm(case["A"][:rows1], case["B"], K, tier=1)) * M / rows1
        row["tier1_packed_s"] = round(t1, 4)
        row["tier1_tops"] = round(2 * macs / t1 / 1e12, 4)
        row["tier1_sample"] = "full" if rows1 == M else "first %d rows of A, extrapolated" % rows1
        rows = M if macs <= 8e10 else 64                      # tier 0 in full up to n = 4096
        t0 = timed(lambda: orc.bmm_rows(case["A"], case["B"], K, 0, rows))
        row["tier0_naive_s"] = round(t0 * M / rows, 4)
        row["tier0_tops"] = round(2 * macs / (t0 * M / rows) / 1e12, 5)
        row["tier0_sample"] = "full" if rows == M else "first %d rows of A, extrapolated" % rows
        if name == "cfg1_sq1024":
            gomp.omp_set_num_threads(1)
            t0s = timed(lambda: orc.bmm_rows(case["A"], case["B"], K, 0, M))
            t1s = timed(lambda: orc.bmm(case["A"], case["B"], K, tier=1))
            gomp.omp_set_num_threads(cores)
            row["tier0_naive_single_thread_s"] = round(t0s, 4)
            row["tier1_packed_single_thread_s"] = round(t1s, 4)
        out["bmm"].append(row)
    convs = []
    for name, case in (("conv_56x56_c128_o128_s1", wl.cfg4a()), ("conv_56x56_c64_o128_s2", wl.cfg4b())):
        N, H, W, C, O, k, st, pad = (case[q] for q in ("N", "H", "W", "C", "O", "k", "stride", "pad"))
        P, Q = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
        macs = float(N) * P * Q * O * k * k * C
        t1 = timed(lambda: orc.bconv(case["x"], case["filt"], C, st, pad, orc.PAD_MINUS_ONE, tier=1))
        t0 = timed(lambda: orc.bconv_images(case["x"], case["filt"], C, st, pad, orc.PAD_MINUS_ONE, 0, 2))
        convs.append({"shape": name, "tier1_packed_s": round(t1, 4), "tier1_tops": round(2 * macs / t1 / 1e12, 4),
                      "tier0_naive_s": round(t0 * N / 2, 3), "tier0_tops": round(2 * macs / (t0 * N / 2) / 1e12, 5),
                      "tier0_sample": "2 of %d images, extrapolated" % N})
    out["bconv"] = convs
    p = wl.resnet18_params()
    x2 = wl.resnet18_input(2)
    t0 = timed(lambda: nets.resnet18_forward(x2, p, tier=0))
    t1 = timed(lambda: nets.resnet18_forward(x2, p, tier=1))
    out["resnet18_224"] = {"tier0_naive_images_per_s": round(2 / t0, 3), "tier1_packed_images_per_s": round(2 / t1, 3),
                           "sample": "whole forward (fp32 stem and head in double) on 2 images"}
    params = wl.mlp_params()
    imgs = wl.mlp_images(1024)
    t0 = timed(lambda: nets.mlp_forward(imgs, params))
    out["mlp_784_1024x3_10"] = {"tier0_naive_images_per_s": round(1024 / t0, 1), "sample": "batch 1024, full"}
    return out


if __name__ == "__main__":
    sys.exit(main())
