#!/usr/bin/env python3
"""Benchmark of the conv2d hot path on one MI355X.

A step is one pass of the whole path over one batch: for every layer of the
workload, conv2d_fwd (with fused bias), then conv2d_bwd_data and
conv2d_bwd_weight (with the bias gradient).  Each layer is an independent
synthetic layer at its stated input shape (seeded device-resident tensors), as
in the per-layer convolution timings the paper discusses (Sec. 3.4, Sec. 4.1).

Prints ONE JSON line on stdout.  `value` is direct-equivalent TFLOP/s
(2*N*K*P*Q*C*R*S per pass, three passes per layer) over the timed steps with all
inputs already resident in HBM.  `roofline` covers the kernel family with the
largest share of the step; `cpu_baseline` is the CPU oracle timed on a bounded
sample of the same workload.  Per-layer detail goes to stderr with --detail.
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

PEAK_MFMA_FP32_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0

# kernels whose roofline is HBM bandwidth over their minimal bytes (streaming and transform
# kernels); every other main kernel is a dense contraction on fp32 MFMA
HBM_BOUND_KERNELS = {"pw_stream_kernel", "pw_wgrad_kernel", "bwd_data_smallc_kernel", "wino4_input_kernel",
                     "wino4_output_kernel", "wino4_wg_input_kernel", "wino4_wg_dy_kernel", "fft_filter_kernel",
                     "fft_wg_output_kernel"}

# main kernel of a call by (resolved algorithm, pass), for the call-level cross-check of the
# roofline block (3x3 layers with even maps; other shapes take sibling kernels)
CALL_KERNEL = {(3, "fwd"): "wino4_gemm_kernel", (3, "bwd_data"): "wino4_gemm_kernel", (3, "bwd_weight"): "wino4_gemm_kernel",
               (2, "fwd"): "wino_pair_kernel", (2, "bwd_data"): "wino_pair_kernel", (2, "bwd_weight"): "wino_wgrad_vec_kernel"}

WORKLOADS = {"tiny": 0, "alexnet": 1, "vgg16": 2, "inception": 3, "overfeat": 4, "apply": -1}


def layer_flops(L, P, Q):
    """Direct-equivalent flops of one pass over one layer."""
    return 2.0 * L.N * L.K * P * Q * L.C * L.R * L.S


def executed_flops(L, P, Q, op, algo):
    """MFMA flops the chosen algorithm itself has to execute for one pass: the
    direct count for the implicit GEMM; for Winograd F(2x2,3x3) the 16 GEMMs,
    2*16*K*C per 2x2 tile (tiles of the pass's output: y for fwd/bwd_weight, dx for
    bwd_data)."""
    if algo == 4:
        # product of spectra: one complex K x C x N product (8 real flops per term) per kept frequency
        return 8.0 * 544 * L.K * L.C * L.N
    if algo == 3:
        # F(4x4,3x3): 36 GEMMs, 2*36*K*C per 4x4 tile of the pass's output
        th, tw = (-(-L.H // 4), -(-L.W // 4)) if op == "bwd_data" else (-(-P // 4), -(-Q // 4))
        return 72.0 * L.N * th * tw * L.K * L.C * (-(-L.R // 3) * -(-L.S // 3))
    if algo != 2:
        return layer_flops(L, P, Q)
    if L.stride > 1:
        # strided layer as a stride-1 3x3 layer over stride^2 * C channels (padded to the
        # kernels' channel granularity) on a (P+2) x (Q+2) map
        cq = L.stride * L.stride * L.C
        cq = -(-cq // 32) * 32 if op == "bwd_weight" else -(-cq // 8) * 8
        th, tw = (-(-(P + 2) // 2), -(-(Q + 2) // 2)) if op == "bwd_data" else (-(-P // 2), -(-Q // 2))
        return 32.0 * L.N * th * tw * L.K * cq
    th, tw = (-(-L.H // 2), -(-L.W // 2)) if op == "bwd_data" else (-(-P // 2), -(-Q // 2))
    nsub = -(-L.R // 3) * -(-L.S // 3)        # 3x3 sub-filters of a larger filter
    c = -(-L.C // 8) * 8 if op == "fwd" else L.C      # forward reduces over whole 8-channel chunks
    return 32.0 * L.N * th * tw * L.K * c * nsub


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="vgg16", choices=sorted(WORKLOADS))
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--algo", type=int, default=0,
                    help="0 auto, 1 implicit GEMM, 2 Winograd F(2x2,3x3) fused, 3 Winograd F(4x4,3x3) unfused, 4 product of spectra; "
                         "calls the algorithm cannot serve use auto")
    ap.add_argument("--detail", action="store_true", help="per-layer table on stderr")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (the same calls, in the same order) into a HIP graph after the warm-up and "
                         "time K replays of it instead of K sequences of stream launches; the per-layer and per-kernel "
                         "figures then come from K further eager steps")
    ap.add_argument("--no-calib", action="store_true", help="skip the MFMA / copy probes (roofline.measured_peak)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="run the library's probe_copy_kernel once over this many MiB before the warm-up (a kernel "
                         "of known traffic for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters, see "
                         "paper_1606_04884_amd/profsum.py)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path would shard by data parallelism over the batch)", file=sys.stderr)
        return 2

    import torch
    from paper_1606_04884_amd import binding as B
    from paper_1606_04884_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "apply":
        return bench_apply(args, dev)
    cfg = WORKLOADS[args.workload]
    layers = synth.config_layers(cfg, args.batch or None)

    # ---- device-resident synthetic tensors (seeded) ----
    gen = torch.Generator(device=dev)
    recs = []
    ws_need = 256
    for li, L in enumerate(layers):
        geom = L.desc()
        P, Q = B.conv2d_output_dims(geom)
        gen.manual_seed(synth.layer_seed(cfg, li, 0))
        x = torch.randn((L.N, L.C, L.H, L.W), device=dev, generator=gen)
        w = torch.randn((L.K, L.C, L.R, L.S), device=dev, generator=gen) * (2.0 / (L.C * L.R * L.S)) ** 0.5
        b = (torch.rand((L.K,), device=dev, generator=gen) - 0.5) * 0.2
        dy = torch.randn((L.N, L.K, P, Q), device=dev, generator=gen)
        rec = dict(L=L, geom=B.make_desc(geom), P=P, Q=Q, x=x, w=w, b=b, dy=dy,
                   y=torch.empty_like(dy), dx=torch.empty_like(x), dw=torch.empty_like(w),
                   db=torch.empty_like(b), flops=layer_flops(L, P, Q))
        rec["algo"] = {}
        rec["req"] = {}          # the algo argument of the call: --algo where it applies, else AUTO
        rec["xflops"] = {}
        for name, op in (("fwd", B.OP_FWD), ("bwd_data", B.OP_BWD_DATA), ("bwd_weight", B.OP_BWD_WEIGHT)):
            req = args.algo if args.algo and B.conv2d_workspace_bytes(rec["geom"], op, args.algo) else 0
            al = req if req else B.conv2d_pick_algo(rec["geom"], op)
            rec["req"][name] = req
            rec["algo"][name] = al
            rec["xflops"][name] = executed_flops(L, P, Q, name, al)
            ws_need = max(ws_need, B.conv2d_workspace_bytes(rec["geom"], op, req))
        recs.append(rec)
    ws = B.alloc_workspace(ws_need, dev)
    stream = torch.cuda.current_stream()
    launch_on = [stream]     # the stream the step's calls are given (the capturing stream while a graph is recorded)

    ev = []          # (op, layer index, start event, end event) for timed steps

    def step(record: bool):
        stream = launch_on[0]
        for li, r in enumerate(recs):
            if record:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
            B.conv2d_fwd(r["geom"], r["x"], r["w"], r["b"], r["y"], ws=ws, algo=r["req"]["fwd"], stream=stream)
            if record:
                e1.record(stream)
                ev.append(("fwd", li, e0, e1))
        for li in range(len(recs) - 1, -1, -1):
            r = recs[li]
            if record:
                e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                e0.record(stream)
            B.conv2d_bwd_data(r["geom"], r["dy"], r["w"], r["dx"], ws=ws, algo=r["req"]["bwd_data"], stream=stream)
            if record:
                e1.record(stream)
            B.conv2d_bwd_weight(r["geom"], r["x"], r["dy"], r["dw"], r["db"], ws=ws, algo=r["req"]["bwd_weight"],
                                stream=stream)
            if record:
                e2.record(stream)
                ev.append(("bwd_data", li, e0, e1))
                ev.append(("bwd_weight", li, e1, e2))

    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib * (1 << 18), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        B.conv2d_probe_copy(src, dst, stream=stream)
        torch.cuda.synchronize()
        del src, dst
    calib = None if args.no_calib else calibrate(dev, stream)
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            launch_on[0] = torch.cuda.current_stream()
            step(False)
        launch_on[0] = stream
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):      # per-layer events: eager steps outside the timed region
            step(True)
        torch.cuda.synchronize()
    else:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(True)
        torch.cuda.synchronize()
        t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    # the same K steps once more with the library's per-kernel events on (two events per
    # main-kernel launch: they cost a few percent of the step, so they stay out of `value`)
    B.conv2d_profile_begin(args.steps * (16 * len(recs) + 16))
    tp0 = time.perf_counter()
    for _ in range(args.steps):
        step(False)
    torch.cuda.synchronize()
    ms_per_step_profiled = (time.perf_counter() - tp0) * 1e3 / args.steps
    nrec = B.conv2d_profile_end()
    total_flops = 3.0 * sum(r["flops"] for r in recs)
    tflops = total_flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-op / per-layer durations from the events of the timed region ----
    per = {}
    for op, li, e0, e1 in ev:
        per.setdefault((op, li), []).append(e0.elapsed_time(e1))
    op_ms = {"fwd": 0.0, "bwd_data": 0.0, "bwd_weight": 0.0}
    xflops_step = 0.0
    for (op, li), ts in per.items():
        op_ms[op] += sum(ts)
        xflops_step += recs[li]["xflops"][op]

    # ---- per-kernel durations: the library's own events around every main-kernel launch
    # of the timed region, on the launch stream (conv2d_profile_*), with the algorithmic
    # flops / minimal bytes each launch stated ----
    kern = {}
    for i in range(nrec):
        kid, fl, by, ms = B.conv2d_profile_record(i)
        k = kern.setdefault(B.conv2d_profile_kernel_name(kid), dict(ms=[], flops=0.0, bytes=0.0))
        k["ms"].append(ms)
        k["flops"] += fl
        k["bytes"] += by

    def kernel_line(name, k):
        tot = sum(k["ms"])
        # (the taps forms serve both first layers, bound by their output, and small 5x5 banks,
        # bound by the matrix pipe: by their arithmetic intensity against the ridge)
        hbm = name in HBM_BOUND_KERNELS or ("TAPS" in name and k["flops"] / max(k["bytes"], 1.0)
                                            < PEAK_MFMA_FP32_TFLOPS * 1e3 / PEAK_HBM_GBS)
        if hbm:
            ach, peak, unit = k["bytes"] / (tot * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        else:
            ach, peak, unit = k["flops"] / (tot * 1e-3) / 1e12, PEAK_MFMA_FP32_TFLOPS, "TFLOP/s"
        return {"bound": "hbm" if hbm else "mfma", "kernel": name, "achieved": round(ach, 3), "peak": peak,
                "unit": unit, "frac": round(ach / peak, 4), "avg_launch_ms": round(tot / len(k["ms"]), 4),
                "launches": len(k["ms"]), "ms_per_step": round(tot / args.steps, 3)}

    if args.detail:
        print("%-12s %-10s %-5s %9s %9s %9s %10s %8s %10s" % ("layer", "op", "algo", "ms(avg)", "ms(med)", "ms(min)",
                                                            "TF/s(dir)", "%peak", "TF/s(exec)"), file=sys.stderr)
        for li, r in enumerate(recs):
            for op in ("fwd", "bwd_data", "bwd_weight"):
                ts = sorted(per[(op, li)])
                ms = sum(ts) / len(ts)
                med = ts[len(ts) // 2] if len(ts) % 2 else 0.5 * (ts[len(ts) // 2 - 1] + ts[len(ts) // 2])
                tf = r["flops"] / (ms * 1e-3) / 1e12
                xtf = r["xflops"][op] / (ms * 1e-3) / 1e12
                print("%-12s %-10s %-5s %9.3f %9.3f %9.3f %10.2f %8.1f %10.2f" % (
                    r["L"].name, op, {2: "wino", 3: "wino4", 4: "fft"}.get(r["algo"][op], "igemm"), ms, med, ts[0], tf,
                    100 * tf / PEAK_MFMA_FP32_TFLOPS, xtf), file=sys.stderr)
        for op in op_ms:
            print("total %-10s %9.3f ms/step" % (op, op_ms[op] / args.steps), file=sys.stderr)
        for name, k in sorted(kern.items(), key=lambda kv: -sum(kv[1]["ms"])):
            kl = kernel_line(name, k)
            print("kernel %-24s %8.3f ms/step %5d launches  %9.1f %s = %.3f of %s peak" % (
                name, kl["ms_per_step"], kl["launches"], kl["achieved"], kl["unit"], kl["frac"], kl["bound"]),
                file=sys.stderr)
        print("wall %.3f ms/step, %.2f TFLOP/s direct-equivalent (%.1f%% of fp32 MFMA peak); executed %.2f TFLOP/s" % (
            ms_per_step, tflops, 100 * tflops / PEAK_MFMA_FP32_TFLOPS, xflops_step / (ms_per_step * 1e-3) / 1e12),
            file=sys.stderr)
        # training skips the input gradient of the first layer: the same totals without it
        first_bd = sum(per[("bwd_data", 0)]) / args.steps
        ev_ms = sum(op_ms.values()) / args.steps
        fl_wo = total_flops - recs[0]["flops"]
        print("without first-layer bwd_data: %.3f ms/step (event sum), %.2f TFLOP/s direct-equivalent" % (
            ev_ms - first_bd, fl_wo / ((ev_ms - first_bd) * 1e-3) / 1e12), file=sys.stderr)
        if args.workload == "vgg16":
            chained_forward(recs, ws, stream, args.algo)
        if args.workload == "inception":
            grouped_1x1(recs, per, ws, stream)

    # roofline of the dominant kernel: the one with the largest summed duration in the
    # timed region; the next ones follow in "others"
    ranked = sorted(kern.items(), key=lambda kv: -sum(kv[1]["ms"]))
    roofline = kernel_line(*ranked[0])
    roofline["traffic"] = None
    # HBM traffic of that kernel per launch as rocprofv3 counted it in an earlier profiling
    # run of this command (the summary is committed; null if none has been taken)
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % args.workload)
    if os.path.exists(tpath):
        try:
            with open(tpath) as fh:
                tr = json.load(fh)
            if roofline["kernel"] in tr.get("bytes_per_launch", {}):
                roofline["traffic"] = tr["bytes_per_launch"][roofline["kernel"]]
                roofline["traffic_source"] = "profiles/traffic_%s.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, %s)" % (
                    args.workload, tr.get("date", "undated"))
        except (OSError, ValueError):
            pass
    if calib:
        roofline["measured_peak"] = calib
        ref = calib["hbm_copy_GBps"] if roofline["bound"] == "hbm" else calib["mfma_f32_TFLOPs"]
        roofline["frac_of_measured_peak"] = round(roofline["achieved"] / ref, 4)
    roofline["others"] = [kernel_line(n, k) for n, k in ranked[1:4]]
    roofline["measured_in"] = ("%d further steps of the same loop right after the timed region, HIP events of the library "
                               "around every main-kernel launch on the launch stream (%.3f ms/step with them on)"
                               % (args.steps, ms_per_step_profiled))
    # cross-check from the timed region itself: the calls this kernel serves, events around the calls
    fam_ms = fam_x = 0.0
    fam_calls = 0
    for (op, li), ts in per.items():
        if CALL_KERNEL.get((recs[li]["algo"][op], op)) == roofline["kernel"]:
            fam_ms += sum(ts)
            fam_x += recs[li]["xflops"][op] * len(ts)
            fam_calls += len(ts)
    if fam_calls:
        roofline["timed_region_calls"] = {"calls": fam_calls, "avg_call_ms": round(fam_ms / fam_calls, 4),
                                          "executed_tflops": round(fam_x / (fam_ms * 1e-3) / 1e12, 3),
                                          "note": "whole calls (main kernel + its transform / reduction kernels)"}

    out = {
        "metric": "fp32 conv TFLOP/s fwd+bwd, direct-equivalent flops (%s conv stack)" % args.workload,
        "value": round(tflops, 3), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "pct_mfma_peak_direct_equivalent": round(100 * tflops / PEAK_MFMA_FP32_TFLOPS, 2),
        "executed_tflops_step": round(xflops_step / (ms_per_step * 1e-3) / 1e12, 3),
        "executed_frac_step": round(xflops_step / (ms_per_step * 1e-3) / 1e12 / PEAK_MFMA_FP32_TFLOPS, 4),
        "config": {"workload": "%s conv stack, N=%d, %d layers, fwd+bwd_data+bwd_weight, fp32 NCHW"
                   % (args.workload, layers[0].N, len(layers)), "algo": args.algo,
                   "launch": "one HIP graph replay per step" if args.graph else "stream launches"},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, layers)
    print(json.dumps(out))
    return 0


def calibrate(dev, stream):
    """What this chip sustains, outside the timed region: a pure v_mfma_f32_32x32x2_f32 loop
    and a 16-byte-vector copy / fill of 1 GiB (the library's probe kernels), best of three."""
    import torch
    from paper_1606_04884_amd import binding as B
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    sink = torch.zeros(4, device=dev)
    n = 1 << 28
    src, dst = torch.ones(n, device=dev), torch.empty(n, device=dev)

    def best(fn, reps=3):
        fn()
        ts = []
        for _ in range(reps):
            e0.record(stream)
            fn()
            e1.record(stream)
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return min(ts) * 1e-3

    flops = [0.0]

    def mfma():
        flops[0] = B.conv2d_probe_mfma_f32(sink, 4000, stream=stream)

    t_m = best(mfma)
    t_c = best(lambda: B.conv2d_probe_copy(src, dst, stream=stream))
    t_f = best(lambda: B.conv2d_probe_copy(None, dst, stream=stream))
    return {"mfma_f32_TFLOPs": round(flops[0] / t_m / 1e12, 2), "hbm_copy_GBps": round(8.0 * n / t_c / 1e9, 1),
            "hbm_fill_GBps": round(4.0 * n / t_f / 1e9, 1),
            "how": "library probes: 512x4 waves of v_mfma_f32_32x32x2_f32 only (%.0f ms); float4 copy and fill of 1 GiB"
                   % (t_m * 1e3)}


def bench_apply(args, dev):
    """The per-element experiment of Sec. 3.3: bandwidth of one per-element kernel
    launch (y = a*x + b, 8 bytes per element) against the number of floats per
    launch.  The curve goes to stderr; the JSON line is the point at 1e7 floats,
    the size the paper singles out.  Each size rotates over enough distinct buffers
    (> 512 MB in total for the large sizes) that repeats are not served from cache."""
    import numpy as np
    import torch
    from paper_1606_04884_amd import binding as B
    import oracle
    stream = torch.cuda.current_stream()
    sizes = [10 ** 3, 10 ** 4, 10 ** 5, 10 ** 6, 10 ** 7, 10 ** 8]
    pool = torch.randn(1 << 28, device=dev)              # 1 GiB of input
    outp = torch.empty(1 << 28, device=dev)
    curve = {}
    for n in sizes:
        nbuf = max(1, min(64, (1 << 28) // ((n + 1023) // 1024 * 1024)))
        pitch = (1 << 28) // nbuf // 1024 * 1024
        reps = max(args.steps * 4, min(2000, (1 << 27) // n + 1))
        for i in range(args.warmup + 2):
            o = (i % nbuf) * pitch
            B.apply_mul_add(pool[o:o + n], outp[o:o + n], 1.5, 0.25, stream=stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(reps):
            o = (i % nbuf) * pitch
            B.apply_mul_add(pool[o:o + n], outp[o:o + n], 1.5, 0.25, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        curve[n] = (us, 8.0 * n / (us * 1e-6) / 1e9)
        print("apply n=%-10d %10.2f us/launch %10.1f GB/s" % (n, us, curve[n][1]), file=sys.stderr)
    n0 = 10 ** 7
    us, gbs = curve[n0]
    out = {
        "metric": "per-element kernel bandwidth at 1e7 floats per launch (y = a*x + b, 8 B/element)",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us * 1e-3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "per-element mul+add, 1e7 floats per launch, back-to-back launches on one stream",
                   "curve_GBps": {str(k): round(v[1], 1) for k, v in curve.items()},
                   "curve_us_per_launch": {str(k): round(v[0], 2) for k, v in curve.items()}},
        "roofline": {"bound": "hbm", "kernel": "apply_mul_add_vec_kernel", "achieved": round(gbs, 1),
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None},
    }
    if not args.no_cpu_baseline:
        x = np.random.default_rng(1).standard_normal(n0).astype(np.float32)
        t0 = time.perf_counter()
        k = 0
        while time.perf_counter() - t0 < 5.0:
            oracle.apply_mul_add(x, 1.5, 0.25)
            k += 1
        sec = (time.perf_counter() - t0) / k
        out["cpu_baseline"] = {"value": round(8.0 * n0 / sec / 1e9, 2), "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": "the numpy oracle on 1e7 floats, %d repetitions" % k}
    print(json.dumps(out))
    return 0


def chained_forward(recs, ws, stream, algo):
    """VGG-16 forward as a chain (outside the timed region): each layer's output,
    max-pooled 2x2/stride 2 after every block (support code, a plain tensor
    reduction), is the next layer's input.  Shows that the per-layer calls compose;
    parity of the chain is covered by tests/test_gpu_chain.py."""
    import torch
    from paper_1606_04884_amd import binding as B
    pool_after = {"conv1_2", "conv2_2", "conv3_3", "conv4_3"}
    outs = [torch.empty_like(r["dy"]) for r in recs]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ms = []
    for _ in range(3):
        x = recs[0]["x"]
        e0.record(stream)
        for r, y in zip(recs, outs):
            B.conv2d_fwd(r["geom"], x, r["w"], r["b"], y, ws=ws, algo=algo, stream=stream)
            x = y
            if r["L"].name in pool_after:
                L = r["L"]
                x = y.view(L.N, L.K, r["P"] // 2, 2, r["Q"] // 2, 2).amax(dim=(3, 5))
        e1.record(stream)
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
    print("chained forward (13 conv calls + 4 max-pool reductions): %.3f ms (best of 3)" % min(ms),
          file=sys.stderr)
    # the same chain with the rectifier after every convolution: as a separate in-place
    # tensor operation (one more read and write of every y) and fused into the epilogue
    res = {}
    for mode in ("separate", "fused"):
        ms = []
        for _ in range(3):
            x = recs[0]["x"]
            e0.record(stream)
            for r, y in zip(recs, outs):
                if mode == "fused":
                    B.conv2d_fwd_relu(r["geom"], x, r["w"], r["b"], y, ws=ws, algo=algo, stream=stream)
                else:
                    B.conv2d_fwd(r["geom"], x, r["w"], r["b"], y, ws=ws, algo=algo, stream=stream)
                    y.clamp_(min=0.0)
                x = y
                if r["L"].name in pool_after:
                    L = r["L"]
                    x = y.view(L.N, L.K, r["P"] // 2, 2, r["Q"] // 2, 2).amax(dim=(3, 5))
            e1.record(stream)
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        res[mode] = min(ms)
    # ... and with the four poolings fused as well (conv2d_fwd_relu_pool2: the unpooled maps
    # of conv1_2, conv2_2, conv3_3 and conv4_3 are never written)
    pooled = {r["L"].name: torch.empty((r["L"].N, r["L"].K, r["P"] // 2, r["Q"] // 2), device=outs[0].device)
              for r in recs if r["L"].name in pool_after}
    ms = []
    for _ in range(3):
        x = recs[0]["x"]
        e0.record(stream)
        for r, y in zip(recs, outs):
            if r["L"].name in pool_after:
                x_next = pooled[r["L"].name]
                B.conv2d_fwd_relu_pool2(r["geom"], x, r["w"], r["b"], x_next, ws=ws, stream=stream)
                x = x_next
            else:
                B.conv2d_fwd_relu(r["geom"], x, r["w"], r["b"], y, ws=ws, algo=algo, stream=stream)
                x = y
        e1.record(stream)
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
    res["pool"] = min(ms)
    print("chained forward with ReLU after every layer: %.3f ms as 13 separate in-place passes, "
          "%.3f ms fused into the convolutions' epilogues (conv2d_fwd_relu), %.3f ms with the four "
          "poolings fused too (conv2d_fwd_relu_pool2)" % (res["separate"], res["fused"], res["pool"]),
          file=sys.stderr)


def grouped_1x1(recs, per, ws, stream):
    """The inception module's three 1x1 convolutions of the block input (1x1,
    3x3_reduce, 5x5_reduce) as ONE call that reads the input once, against the sum
    of the three separate forward calls of the timed region (outside it)."""
    import torch
    from paper_1606_04884_amd import binding as B
    idx = [i for i, r in enumerate(recs) if r["L"].name in ("1x1", "3x3_reduce", "5x5_reduce")]
    if len(idx) != 3:
        return
    L0 = recs[idx[0]]["L"]
    geom = (L0.N, L0.C, L0.H, L0.W, sum(recs[i]["L"].K for i in idx), 1, 1, 1, 1, 0, 0)
    x = recs[idx[0]]["x"]
    wl = [recs[i]["w"] for i in idx]
    bl = [recs[i]["b"] for i in idx]
    yl = [recs[i]["y"] for i in idx]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ms = []
    for _ in range(5):
        e0.record(stream)
        B.conv2d_fwd_1x1_group(geom, x, wl, bl, yl, ws=ws, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
    sep = sum(sum(per[("fwd", i)]) / len(per[("fwd", i)]) for i in idx)
    byt = 4.0 * (x.numel() + sum(y.numel() for y in yl))
    print("grouped 1x1 forward (K = %s in one call): %.3f ms (best of 5) = %.2f TB/s over x + y once; "
          "three separate calls: %.3f ms" % ("+".join(str(recs[i]["L"].K) for i in idx), min(ms),
                                             byt / (min(ms) * 1e-3) / 1e12, sep), file=sys.stderr)


def cpu_baseline(cfg, layers):
    """The oracle as it stands, timed on the host cores on a bounded sample: the
    same stack at batch 1 (every layer, all three passes)."""
    import numpy as np
    import oracle
    from paper_1606_04884_amd import synth

    nb = 8
    flops = 0.0
    sec = 0.0
    for li, L in enumerate(layers):
        Ls = L.with_batch(nb)
        geom = Ls.desc()
        P, Q = oracle.output_dims(geom)
        t = synth.layer_tensors(max(cfg, 1), li, Ls, (P, Q))
        t0 = time.perf_counter()
        oracle.fwd(geom, t["x"], t["w"], t["b"])
        oracle.bwd_data(geom, t["dy"], t["w"])
        oracle.bwd_weight(geom, t["x"], t["dy"])
        sec += time.perf_counter() - t0
        flops += 3.0 * 2.0 * nb * L.K * P * Q * L.C * L.R * L.S
    return {"value": round(flops / sec / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(sec, 2),
            "sample": "same stack at batch %d of %d: all %d layers, fwd+bwd_data+bwd_weight"
                      % (nb, layers[0].N, len(layers))}


if __name__ == "__main__":
    sys.exit(main())
