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

WORKLOADS = {"tiny": 0, "alexnet": 1, "vgg16": 2, "inception": 3, "overfeat": 4}


def layer_flops(L, P, Q):
    return 2.0 * L.N * L.K * P * Q * L.C * L.R * L.S


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="vgg16", choices=sorted(WORKLOADS))
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--algo", type=int, default=0, help="0 auto, 1 implicit GEMM, 2 Winograd")
    ap.add_argument("--detail", action="store_true", help="per-layer table on stderr")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path shards by data parallelism over the batch, see DESIGN.md)", file=sys.stderr)
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
        for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
            ws_need = max(ws_need, B.conv2d_workspace_bytes(rec["geom"], op, args.algo))
        recs.append(rec)
    ws = B.alloc_workspace(ws_need, dev)
    stream = torch.cuda.current_stream()

    ev = []          # (op, layer index, start event, end event) for timed steps

    def step(record: bool):
        for li, r in enumerate(recs):
            if record:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
            B.conv2d_fwd(r["geom"], r["x"], r["w"], r["b"], r["y"], ws=ws, algo=args.algo, stream=stream)
            if record:
                e1.record(stream)
                ev.append(("fwd", li, e0, e1))
        for li in range(len(recs) - 1, -1, -1):
            r = recs[li]
            if record:
                e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                e0.record(stream)
            B.conv2d_bwd_data(r["geom"], r["dy"], r["w"], r["dx"], ws=ws, algo=args.algo, stream=stream)
            if record:
                e1.record(stream)
            B.conv2d_bwd_weight(r["geom"], r["x"], r["dy"], r["dw"], r["db"], ws=ws, algo=args.algo,
                                stream=stream)
            if record:
                e2.record(stream)
                ev.append(("bwd_data", li, e0, e1))
                ev.append(("bwd_weight", li, e1, e2))

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    total_flops = 3.0 * sum(r["flops"] for r in recs)
    tflops = total_flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-op / per-layer durations from the events of the timed region ----
    per = {}
    for op, li, e0, e1 in ev:
        per.setdefault((op, li), []).append(e0.elapsed_time(e1))
    fam_ms = {"fwd": 0.0, "bwd_data": 0.0, "bwd_weight": 0.0}
    fam_flops = {"fwd": 0.0, "bwd_data": 0.0, "bwd_weight": 0.0}
    fam_calls = {"fwd": 0, "bwd_data": 0, "bwd_weight": 0}
    for (op, li), ts in per.items():
        fam_ms[op] += sum(ts)
        fam_flops[op] += recs[li]["flops"] * len(ts)
        fam_calls[op] += len(ts)
    if args.detail:
        print("%-12s %-10s %9s %9s %8s" % ("layer", "op", "ms(avg)", "TFLOP/s", "%peak"), file=sys.stderr)
        for li, r in enumerate(recs):
            for op in ("fwd", "bwd_data", "bwd_weight"):
                ts = per[(op, li)]
                ms = sum(ts) / len(ts)
                tf = r["flops"] / (ms * 1e-3) / 1e12
                print("%-12s %-10s %9.3f %9.2f %8.1f" % (r["L"].name, op, ms, tf,
                                                         100 * tf / PEAK_MFMA_FP32_TFLOPS), file=sys.stderr)
        for op in fam_ms:
            print("total %-10s %9.3f ms/step" % (op, fam_ms[op] / args.steps), file=sys.stderr)
        print("wall %.3f ms/step, %.2f TFLOP/s (%.1f%% of fp32 MFMA peak)" % (
            ms_per_step, tflops, 100 * tflops / PEAK_MFMA_FP32_TFLOPS), file=sys.stderr)

    # dominant kernel family: the gather kernel serves fwd and bwd_data calls
    gather_ms = fam_ms["fwd"] + fam_ms["bwd_data"]
    if gather_ms >= fam_ms["bwd_weight"]:
        kname, k_ms = "gemmconv_kernel (fwd + bwd_data calls)", gather_ms
        k_flops = fam_flops["fwd"] + fam_flops["bwd_data"]
        k_calls = fam_calls["fwd"] + fam_calls["bwd_data"]
    else:
        kname, k_ms, k_flops = "wgrad_kernel (bwd_weight calls)", fam_ms["bwd_weight"], fam_flops["bwd_weight"]
        k_calls = fam_calls["bwd_weight"]
    achieved = k_flops / (k_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": kname, "achieved": round(achieved, 3),
                "peak": PEAK_MFMA_FP32_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_MFMA_FP32_TFLOPS, 4), "traffic": None,
                "avg_launch_ms": round(k_ms / k_calls, 4), "launches": k_calls}

    out = {
        "metric": "fp32 conv TFLOP/s fwd+bwd (%s conv stack)" % args.workload,
        "value": round(tflops, 3), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "pct_mfma_peak": round(100 * tflops / PEAK_MFMA_FP32_TFLOPS, 2),
        "config": {"workload": "%s conv stack, N=%d, %d layers, fwd+bwd_data+bwd_weight, fp32 NCHW"
                   % (args.workload, layers[0].N, len(layers)), "algo": args.algo},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, layers)
    print(json.dumps(out))
    return 0


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
