#!/usr/bin/env python3
"""Benchmark of the fused forward convolution (conv + bias + ReLU) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5b] [--no-layers] [--no-cpu]
                    [--fusion-sweep] [--calibration-copy]

A step is one cvx_conv_fwd_fused call on one batch of synthetic input already resident in HBM.
Steps rotate over enough disjoint (x, y) buffer sets that the working set exceeds the 256 MiB
Infinity Cache, so the figures are HBM figures.  The K timed steps are recorded once into HIP
graphs (so the Python call overhead is not what is measured) and replayed between two HIP events
on the launch stream, inside a wall-clock bracket with device synchronisation on both sides.
The same steps are also timed once as plain calls through the C ABI (no graph): `eager_us_per_step`.

Prints ONE JSON line.  The headline workload is the largest single-GPU layer of the benchmark
set (c5b: 29.6 GFLOP, 65 MB); `layers` carries the same measurement for all seven layers.
`roofline` prices the kernel against the MI355X peak for its bound; `cpu_baseline` is the fp64 CPU
oracle timed on this host in the same run (a reported baseline, not a target); `parity` is the
check of the warm-up output and of an output of the timed replay against that oracle.  If a
parity check fails the line carries "value": null and the exit status is 1.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_MFMA_16BIT_TFLOPS = 2516.6      # dense bf16 / fp16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
ROTATE_BYTES = 1 << 30               # rotate buffer sets over at least this much memory
RESULTS_DIR = os.path.join(ROOT, "gpurun_out")   # where the per-layer tables are written as JSON
GRAPH_CHUNK = 250
LAYERS = ["c1", "c2", "c3a", "c3b", "c4", "c5a", "c5b", "c2f32"]   # the seven benchmark layers, and c2 in fp32
HEADLINE = "c5b"

# Which roofline binds each layer (arithmetic intensity against the ridge point of 2516.6 TFLOP/s over
# 8 TB/s = 315 FLOP/byte): the two 1x1 layers and the stem are HBM-bound, the 3x3 layers MFMA-bound.
BOUND = {"c1": "alu", "c2": "mfma", "c3a": "hbm", "c3b": "hbm", "c4": "hbm", "c5a": "mfma", "c5b": "mfma", "c2f32": "mfma"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_workload(name, steps: int, warmup: int, check: bool, unfused: bool = False, eager: bool = False):
    """Time one workload (a name from workloads.WORKLOADS, or a ConvWorkload).  `unfused` runs the
    same operator as three launches -- convolution, bias add, ReLU -- the unfused route of Sec. V."""
    import torch
    import workloads as wl
    from paper_1910_00078_amd import cvx
    from parity import to_device, to_host_f64, tolerance_ok, DT_CODE

    w = wl.WORKLOADS[name] if isinstance(name, str) else name
    name = w.name
    x, wt, b = wl.make_inputs(w)
    stream = torch.cuda.current_stream()
    plan = cvx.ConvPlan(DT_CODE[w.dtype], (w.N, w.C, w.H, w.W), (w.K, w.C // w.groups, w.R, w.S),
                        w.pad, w.stride, w.dil, w.groups, stream=stream.cuda_stream)
    dw, db = to_device(wt, w.dtype), to_device(b, w.dtype)
    x0 = to_device(x, w.dtype)
    set_bytes = w.elem_bytes * (w.N * w.C * w.H * w.W + w.N * w.K * w.Ho * w.Wo)
    nsets = min(64, max(2, -(-ROTATE_BYTES // set_bytes)))
    xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
    # every output starts as NaN: an element the kernel never writes fails the parity check
    ys = [torch.full(plan.y_shape, float("nan"), dtype=x0.dtype, device="cuda") for _ in range(nsets)]

    def step(i):
        j = i % nsets
        if unfused:
            plan.run_plain(xs[j].data_ptr(), dw.data_ptr(), ys[j].data_ptr())
            cvx.cvx_bias_add(plan.h, plan.bd, db.data_ptr(), plan.yd, ys[j].data_ptr())
            cvx.cvx_activation_fwd(plan.h, cvx.CVX_ACT_RELU, 0.0, plan.yd, ys[j].data_ptr())
        else:
            plan.run(xs[j].data_ptr(), dw.data_ptr(), db.data_ptr(), ys[j].data_ptr(), cvx.CVX_ACT_RELU, 0.0)

    for i in range(max(warmup, 1)):
        step(i)
    torch.cuda.synchronize()
    kernel = plan.last_kernel()

    parity = None
    ref = None
    cpu = None
    if check:
        from oracle import conv_oracle
        X, Wt, B = wl.to_f64(x, w.dtype), wl.to_f64(wt, w.dtype), wl.to_f64(b, w.dtype)
        t0 = time.perf_counter()
        ref = conv_oracle.conv_fwd(X, Wt, B, pad=w.pad, stride=w.stride, dil=w.dil, groups=w.groups, act=1)
        dt = time.perf_counter() - t0
        cpu = {"value": w.flops / dt / 1e12, "unit": "TFLOP/s", "cores": conv_oracle.threads(), "kind": "oracle",
               "sample": "the whole %s workload once (%.2f GFLOP in %.2f s, fp64)" % (name, w.flops / 1e9, dt)}
        ok, msg = tolerance_ok(to_host_f64(ys[0], w.dtype), ref, w.dtype)
        parity = {"ok": bool(ok), "detail": msg}
        log("[bench] parity %s (warm-up output): %s" % (name, msg))

    eager_ms = None
    if eager:
        # the same steps as plain calls through the C ABI: what a caller without graphs pays per call
        n = min(steps, 500)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        eager_ms = e0.elapsed_time(e1) / n

    # record the timed steps into graphs: chunks of GRAPH_CHUNK launches, replayed
    chunk = min(steps, GRAPH_CHUNK)
    reps, rem = divmod(steps, chunk)
    side = torch.cuda.Stream()
    graphs = []
    for gi, n in enumerate([chunk] + ([rem] if rem else [])):
        gph = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            plan.set_stream(side.cuda_stream)
            with torch.cuda.graph(gph, stream=side):
                for i in range(n):
                    step(gi * chunk + i)
        graphs.append(gph)
    plan.set_stream(stream.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    graphs[0].replay()                      # one untimed replay (graph upload)
    torch.cuda.synchronize()
    if check:
        # the timed replays must write every output again: poison one buffer the replay covers
        ys[(chunk - 1) % nsets].fill_(float("nan"))

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(reps):
        graphs[0].replay()
    if rem:
        graphs[1].replay()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    if check:
        ok, msg = tolerance_ok(to_host_f64(ys[(chunk - 1) % nsets], w.dtype), ref, w.dtype)
        log("[bench] parity %s (output of the timed replay): %s" % (name, msg))
        parity = {"ok": bool(parity["ok"] and ok), "detail": parity["detail"], "replay_detail": msg}
    plan.close()
    return {"workload": w, "kernel": kernel, "wall_ms_per_step": wall_ms / steps, "event_ms_per_step": ev_ms / steps,
            "eager_ms_per_step": eager_ms, "nsets": nsets, "parity": parity, "cpu": cpu}


def measured_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 counter runs (profiles/pmc_traffic.json,
    written by profile_summary.py); None if the layer has no entry.  It is a figure of the commit the
    profiles were taken at, not of this run."""
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    if os.path.exists(tpath):
        return json.load(open(tpath)).get(name)
    return None


def roofline(w, name, ms_kernel):
    bound = BOUND[name]
    traffic = measured_traffic(name)
    src = "profiles/pmc_traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a 256 MiB copy)" if traffic else None
    if bound == "hbm":
        ach = w.algorithmic_bytes / (ms_kernel * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                "traffic": traffic, "traffic_source": src}
    ach = w.flops / (ms_kernel * 1e-3) / 1e12
    # a contraction is priced against the matrix peak of its own data type (fp32: 157.3, as the vector pipe)
    peak = PEAK_MFMA_16BIT_TFLOPS if bound == "mfma" and w.dtype != "f32" else PEAK_FP32_TFLOPS
    return {"bound": bound, "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak, "traffic": traffic,
            "traffic_source": src}


def fusion_sweep(steps: int):
    """Fused conv+bias+ReLU (one launch) against conv, bias add, ReLU (three launches, two extra
    passes over the output) on the benchmark layers and on a sweep of the filter count K for a 3x3
    and a 1x1 layer: the experiment of Fig. 6a of the paper."""
    import dataclasses
    import workloads as wl
    cases = [wl.WORKLOADS[n] for n in ("c2", "c3a", "c3b", "c4", "c5a", "c5b")]
    for k in (16, 32, 64, 128, 256, 512):
        cases.append(dataclasses.replace(wl.WORKLOADS["c2"], name="3x3_c64_56x56_k%d" % k, K=k))
    for k in (16, 64, 256, 1024):
        cases.append(dataclasses.replace(wl.WORKLOADS["c3a"], name="1x1_c256_56x56_k%d" % k, K=k, N=16))
    rows = []
    for w in cases:
        f = time_workload(w, steps, 3, check=False)
        u = time_workload(w, steps, 3, check=False, unfused=True)
        row = {"case": w.name, "K": w.K, "kernel": f["kernel"], "fused_us": f["event_ms_per_step"] * 1e3,
               "unfused_us": u["event_ms_per_step"] * 1e3,
               "speedup": u["event_ms_per_step"] / f["event_ms_per_step"]}
        rows.append(row)
        log("[fusion] %-24s K=%-5d %-28s fused %8.2f us   conv+bias+relu %8.2f us   x%.2f"
            % (row["case"], row["K"], row["kernel"], row["fused_us"], row["unfused_us"], row["speedup"]))
    os.makedirs(RESULTS_DIR, exist_ok=True)
    json.dump(rows, open(os.path.join(RESULTS_DIR, "fusion_sweep.json"), "w"), indent=1)
    return rows


def layer_row(name, rr):
    w = rr["workload"]
    ms = rr["event_ms_per_step"]
    rf = roofline(w, name, ms)
    return {"workload": name, "kernel": rr["kernel"], "us": ms * 1e3,
            "eager_us": None if rr["eager_ms_per_step"] is None else rr["eager_ms_per_step"] * 1e3,
            "tflops": w.flops / (ms * 1e-3) / 1e12, "gbs": w.algorithmic_bytes / (ms * 1e-3) / 1e9,
            "bound": rf["bound"], "frac": rf["frac"], "traffic": rf["traffic"],
            "parity_ok": None if rr["parity"] is None else rr["parity"]["ok"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-layers", action="store_true", help="time only the headline workload (no `layers` table)")
    ap.add_argument("--all", action="store_true", help="accepted for compatibility: the table of all layers is the default")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle (no parity check, no cpu_baseline)")
    ap.add_argument("--fusion-sweep", action="store_true",
                    help="also time fused against unfused (conv, bias add, ReLU as three launches) on every layer and "
                         "over a sweep of K; table to stderr and fusion_sweep.json in the results directory")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first run one plain 256 MiB device copy (a kernel of known traffic, to scale rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (forward convolution shards over the batch with no "
              "communication: each GPU would take a slice of the images and a copy of the filters); --gpus %d is not available" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    check = not args.no_cpu
    r = time_workload(args.workload, args.steps, args.warmup, check=check, eager=True)
    w = r["workload"]
    ms = r["event_ms_per_step"]
    all_ok = r["parity"] is None or r["parity"]["ok"]
    out = {
        "metric": "conv-fwd TFLOP/s (fused bias+ReLU, bf16) and % of MFMA/HBM roofline",
        "value": w.flops / (r["wall_ms_per_step"] * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["wall_ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "f16": "f16", "f32": "f32"}[w.dtype],
        "data": "synthetic",
        "config": {"workload": "%s: %s NCHW %dx%dx%dx%d -> K=%d, %dx%d filter, pad %d, stride %d, bias+ReLU"
                               % (args.workload, w.dtype, w.N, w.C, w.H, w.W, w.K, w.R, w.S, w.pad[0], w.stride[0]),
                   "kernel": r["kernel"], "buffer_sets": r["nsets"],
                   "gflop_per_step": w.flops / 1e9, "algorithmic_mb_per_step": w.algorithmic_bytes / 1e6},
        "roofline": roofline(w, args.workload, ms),
        "cpu_baseline": r["cpu"],
        "parity": r["parity"],
        "event_ms_per_step": ms,
        "eager_us_per_step": None if r["eager_ms_per_step"] is None else r["eager_ms_per_step"] * 1e3,
    }

    if not args.no_layers:
        rows = []
        for name in LAYERS:
            if name == args.workload:
                rr = r
            else:
                steps = 300 if name in ("c3a", "c3b", "c4") else 500
                rr = time_workload(name, steps, 5, check=check, eager=True)
            row = layer_row(name, rr)
            rows.append(row)
            all_ok = all_ok and row["parity_ok"] is not False
            log("[bench] %-4s %-28s %9.2f us (eager %s)  %8.1f TFLOP/s  %8.1f GB/s  %s frac %.3f  parity %s"
                % (name, row["kernel"], row["us"], "-" if row["eager_us"] is None else "%.2f us" % row["eager_us"],
                   row["tflops"], row["gbs"], row["bound"], row["frac"], row["parity_ok"]))
        os.makedirs(RESULTS_DIR, exist_ok=True)
        json.dump(rows, open(os.path.join(RESULTS_DIR, "bench_all.json"), "w"), indent=1)
        out["layers"] = rows

    if args.fusion_sweep:
        out["fusion_sweep"] = fusion_sweep(200)

    if not all_ok:
        out["value"] = None            # a wrong kernel produces no throughput figure
    print(json.dumps(out), flush=True)
    sys.exit(0 if all_ok else 1)


if __name__ == "__main__":
    main()
