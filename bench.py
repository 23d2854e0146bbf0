#!/usr/bin/env python3
"""Throughput of the TS + TAB-Q hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
compress (threshold splitting, width selection, scan, quantize + pack, CSR emission)
followed by decompress (unpack, dequantize, outlier scatter).  Inputs are resident
in HBM before the timed region; the step rotates over several buffer sets so that
the 256 MB last-level cache does not serve the input.

Prints ONE JSON line: metric, value, unit, ms_per_step, config, plus the objects `roofline` (the dominant
kernel against the HBM peak, per-kernel times) and `cpu_baseline` (the CPU checker timed on a sample).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published peak

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, scaled by
# what the same counters read for a plain 128 MiB copy (profiles/C4_*_hbm_traffic.txt);
# keyed by (workload, pipeline, eps) -> kernel -> bytes.  None where no such run was made.
TRAFFIC = {
    ("C4", "staged", 0.05): {"k_row_stats": 134.3e6 + 0.6e6, "k_pack": 136.6e6 + 62.7e6,
                             "k_unpack": 67.1e6 + 134.2e6, "k_scan": 0.2e6},
    ("C4", "fused", 0.05): {"k_fused": 135.2e6 + 64.1e6, "k_unpack": 67.1e6 + 134.2e6},
}


# VALU instructions per launch (wave level) from a rocprofv3 --pmc SQ_INSTS_VALU run of this command
# (profiles/C4_fused_valu_counts.txt), and the issue peak they are priced against: 256 CUs x 4 SIMDs x 16 lanes
# x 2.4 GHz = 39.3e12 lane-operations per second (packed fp32 is not used, so every VALU instruction occupies
# its SIMD for four cycles per wave of 64).
VALU_INSTS = {("C4", "fused", 0.05): {"k_fused": 23.6e6, "k_unpack": 7.75e6}}
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5", "KV7", "KV13"])
    ap.add_argument("--eps", type=float, default=0.05, help="error budget, relative to the row RMS")
    ap.add_argument("--pipeline", default="auto", choices=["auto", "staged", "fused"])
    ap.add_argument("--nbuf", type=int, default=0,
                    help="buffer sets rotated through (default 4; 1 for C5 and the KV workloads, whose "
                         "single set is beyond the last-level cache already)")
    ap.add_argument("--graph", action="store_true", help="replay the timed steps as one HIP graph")
    ap.add_argument("--bits", default="", help="allowed widths, e.g. 2,4,8 (default: the workload's set)")
    ap.add_argument("--tau", type=float, default=0.0, help="outlier threshold (default: the workload's)")
    ap.add_argument("--c5-seqs", type=int, default=32)
    ap.add_argument("--c5-workers", type=int, default=8,
                    help="processes that generate C5 (use 1 under a profiler: its preloaded tool does not survive a fork)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=0, help="0 = sized for about 10-30 s")
    return ap.parse_args()


def make_input(args):
    from paper_2511_04002_amd import synth
    w = synth.WORKLOADS[args.workload]
    if args.workload in synth.KV_WORKLOADS:
        x = synth.make_kv(args.workload)          # a list of tensors: the batch form of the calls
    elif args.workload == "C5":
        x = synth.make_c5(seqs=args.c5_seqs, workers=args.c5_workers)
    elif args.workload == "C3":
        x = synth.make_c3(0)
    else:
        x = synth.make(args.workload)
    return w, x


def cpu_baseline(x, w, tau, bit_set, eps, rows):
    """The oracle as it stands, on a bounded sample of the same workload."""
    from oracle import tsq_oracle as O
    O.build()
    dt = O.F16 if w.dtype == "f16" else O.BF16
    threads = min(O.max_threads(), os.cpu_count() or 1, 16)
    rows = min(rows, x.shape[0])
    xs = x[:rows]
    gb = xs.size * 2 / 1e9
    # repeat the sample until about 15 core-seconds of work have been done; report the best pass
    best, passes, spent = None, 0, 0.0
    while passes < 1 or (spent * threads < 15.0 and passes < 50):
        t0 = time.perf_counter()
        c = O.compress(xs, dt, tau, bit_set, eps, O.BUDGET_REL_RMS, nthreads=threads)
        t1 = time.perf_counter()
        O.decompress(c, nthreads=threads)
        t2 = time.perf_counter()
        passes += 1
        spent += t2 - t0
        if best is None or t2 - t0 < best[0]:
            best = (t2 - t0, t1 - t0, t2 - t1)
    return {"value": gb / best[0], "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "first %d of the first %d rows of %s, best of %d passes (%.1f s in all): compress %.3f s + "
                      "decompress %.3f s, %d threads" % (rows, x.shape[0], w.name, passes, spent, best[1], best[2],
                                                          threads)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no cross-GPU step (rows are independent); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    w, x = make_input(args)               # host only, before anything touches the GPU (it may fork)
    parts = x if isinstance(x, list) else None       # KV workloads: separate tensors, batch calls
    if parts is not None:
        x = np.concatenate(parts[:2])                 # what the CPU baseline samples from
    import torch
    from paper_2511_04002_amd import tsq

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    tsq.lib()
    torch.cuda.set_device(0)
    T, H = (len(parts) * parts[0].shape[0], parts[0].shape[1]) if parts else x.shape
    pipe = "fused" if args.pipeline == "auto" else args.pipeline     # what "auto" resolves to
    bit_set = tuple(int(b) for b in args.bits.split(",")) if args.bits else tuple(w.bit_set)
    tau = args.tau if args.tau > 0 else w.tau
    plan = tsq.Plan(T, H, w.dtype, tau, bit_set, args.eps, mode="rel_rms", pipeline=pipe,
                    max_outliers=max(1, (T * H) // 8))
    nbuf = max(1, args.nbuf or (1 if parts or w.name == "C5" else 4))
    if parts:
        x0 = [torch.from_numpy(p.view(np.int16)).cuda() for p in parts]
        xs = [x0] + [[t.clone() for t in x0] for _ in range(nbuf - 1)]
        outs = [[torch.empty_like(t) for t in x0] for _ in range(nbuf)]
        tin = [plan.pointer_table(v) for v in xs]
        tout = [plan.pointer_table(v) for v in outs]
    else:
        x0 = torch.from_numpy(x.view(np.int16)).cuda()
        xs = [x0] + [x0.clone() for _ in range(nbuf - 1)]
        outs = [plan.new_output() for _ in range(nbuf)]
    blobs = [plan.new_blob() for _ in range(nbuf)]
    ws = plan.new_workspace()

    def step(i, ev=None):
        k = i % nbuf
        if ev:
            ev[0].record()
        if parts:
            plan.compress_batch(xs[k], blobs[k], ws, table=tin[k])
        else:
            plan.compress(xs[k], blobs[k], ws)
        if ev:
            ev[1].record()
        if parts:
            plan.decompress_batch(blobs[k], outs[k], table=tout[k])
        else:
            plan.decompress(blobs[k], outs[k])
        if ev:
            ev[2].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    info = plan.info(blobs[0])
    assert info.status == 0

    # the timed region: exactly K steps between two events on the stream (nothing else is enqueued
    # in between); with --graph the K steps are captured once and replayed as one HIP graph
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    graph = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for i in range(args.steps):
                    step(args.warmup + i)
        torch.cuda.current_stream().wait_stream(side)
        graph.replay()                     # one untimed replay
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    if graph is not None:
        graph.replay()
    else:
        for i in range(args.steps):
            step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    assert plan.info(blobs[0]).status == 0

    # compress / decompress split of the same steps (events between the two calls: not the headline)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(args.warmup + i, evs[i])
    torch.cuda.synchronize()
    ms_c = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    ms_d = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps

    n = T * H
    rho = info.nnz / n
    bbar = 8.0 * info.payload_bytes / n
    side = info.payload_bytes + 4 * info.nnz + 21 * T      # payload + CSR + per-token metadata
    alg_c = 2 * n + side                                   # compress: read input, write the blob
    alg_d = side + 2 * n                                   # decompress: read the blob, write output

    # per-kernel durations of the same steps, HIP events around every launch inside the library
    # (tsq_compress_timed) and around the one decompress kernel
    names = ["k_fused"] if pipe == "fused" else ["k_row_stats", "k_scan", "k_pack"]
    acc = [0.0] * len(names)
    if parts:
        assert pipe == "fused", "the batch form is timed per call: with one kernel per call that is per kernel"
        acc = [ms_c * args.steps]
    for i in range(0 if parts else args.steps):
        k = (args.warmup + i) % nbuf
        ms = tsq.tsq_compress_timed(plan.handle, xs[k].data_ptr(), blobs[k].data_ptr(), ws.data_ptr(),
                                    plan._stream())
        for j in range(len(names)):
            acc[j] += ms[j]
        plan.decompress(blobs[k], outs[k])
    torch.cuda.synchronize()
    # algorithmic bytes of each kernel: what it must read and write once
    kalg = {"k_fused": alg_c, "k_row_stats": 2 * n + 9 * T, "k_scan": 29 * T, "k_pack": alg_c,
            "k_unpack": alg_d}
    kern = {nm: {"ms": acc[j] / args.steps, "alg_bytes": kalg[nm]} for j, nm in enumerate(names)}
    kern["k_unpack"] = {"ms": ms_d, "alg_bytes": alg_d}
    for v in kern.values():
        v["GBps"] = v["alg_bytes"] / v["ms"] / 1e6
    dom = max(kern, key=lambda nm: kern[nm]["ms"])
    achieved = kern[dom]["GBps"]
    pair_gbps = (alg_c + alg_d) / (ms_c + ms_d) / 1e6
    traffic = TRAFFIC.get((w.name, pipe, args.eps), {}).get(dom)
    insts = VALU_INSTS.get((w.name, pipe, args.eps), {}).get(dom)
    valu = None
    if insts:
        ops = insts * 64.0 / (kern[dom]["ms"] * 1e-3)
        valu = {"wave_instructions": insts, "achieved_lane_ops_per_s": ops, "peak_lane_ops_per_s": VALU_PEAK_LANE_OPS,
                "frac": ops / VALU_PEAK_LANE_OPS}

    res = {
        "metric": "compress+decompress GB/s of split-point activations",
        "value": 2.0 * n / ms_per_step / 1e6,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": ("%s %dx%d %s" % (w.name, T, H, w.dtype)) +
                               (" as %d tensors of %d rows" % (len(parts), parts[0].shape[0]) if parts else ""),
                   "tau": tau,
                   "bit_set": list(bit_set), "budget": "%.3g x row RMS" % args.eps,
                   "pipeline": pipe, "launch": "hip graph" if args.graph else "stream", "buffer_sets": nbuf, "mean_width": round(bbar, 3),
                   "outlier_fraction": round(rho, 6), "width_hist": list(info.width_hist),
                   "compression_ratio": round(2.0 * n / info.compressed_bytes, 3)},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "compress_ms": ms_c, "decompress_ms": ms_d,
                     "pair_achieved": pair_gbps, "pair_frac": pair_gbps / HBM_PEAK_GBS,
                     "valu_issue": valu, "kernels": kern},
        "host_wall_ms_per_step": wall * 1e3 / args.steps,
    }
    if not args.no_cpu_baseline:
        rows = args.cpu_sample_rows or max(64, min(T, int(2.5e8 // H)))
        res["cpu_baseline"] = cpu_baseline(x, w, tau, bit_set, args.eps, rows)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
