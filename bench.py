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
# the issue peak that VALU instruction counts are priced against: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz =
# 39.3e12 lane-operations per second (one VALU instruction occupies its SIMD for four cycles per wave of 64)
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9


def kernels_sha():
    """Fingerprint of the kernel sources: counter figures from a profile are used only for the sources they
    were taken from."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2511_04002_amd", "csrc", "*"))):
        if f.endswith((".hip", ".hpp", ".cpp", ".h")):
            h.update(open(f, "rb").read())
    return h.hexdigest()[:12]


def profile_records():
    """Counter figures per launch from the rocprofv3 summaries under profiles/: lines of the form
    `bench-record: workload=C4 pipeline=fused eps=0.05 kernel=k_fused hbm_bytes=1.99e8 valu_wave_insts=2.3e7
    kernels_sha=...` that each summary ends with.  -> {(workload, pipeline, eps, kernel): {...}}"""
    import glob
    out = {}
    for f in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(f):
            if not line.startswith("bench-record:"):
                continue
            kv = dict(item.split("=", 1) for item in line.split()[1:])
            key = (kv.get("workload"), kv.get("pipeline"), float(kv.get("eps", "nan")), kv.get("kernel"))
            out.setdefault(key, {"source": os.path.basename(f)}).update(
                {k: (float(v) if k in ("hbm_bytes", "valu_wave_insts") else v) for k, v in kv.items()
                 if k in ("hbm_bytes", "valu_wave_insts", "kernels_sha")})
    return out


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (the card needs a few milliseconds of work before its clocks settle: with 5 warm-up steps the same
    # kernels read about 10 % slower)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5", "KV7", "KV13"])
    ap.add_argument("--eps", type=float, default=0.05, help="error budget, relative to the row RMS")
    ap.add_argument("--pipeline", default="auto", choices=["auto", "staged", "fused"])
    ap.add_argument("--nbuf", type=int, default=0,
                    help="buffer sets rotated through (default 4; 1 for C5 and the KV workloads, whose "
                         "single set is beyond the last-level cache already)")
    ap.add_argument("--launch", default="auto", choices=["auto", "stream", "graph", "two-streams"],
                    help="how the timed steps that give the headline are enqueued (the line reports all three either "
                         "way): one by one on one stream; replayed from a HIP graph; compress calls on one stream and "
                         "decompress calls on a second one, each decompress behind its compress by an event, so that "
                         "a step's decompress overlaps the next step's compress.  auto: the faster of stream and "
                         "two-streams")
    ap.add_argument("--graph", action="store_true", help="the same as --launch graph")
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


def oracle_check(x, w, tau, bit_set, eps, sec, rows=64):
    """The first `rows` tokens of the benchmarked blob against the oracle, bit for bit (a token's width,
    scale, codes and outliers do not depend on the tokens behind it; its offsets are those of the prefix)."""
    import numpy as np
    from oracle import tsq_oracle as O
    O.build()
    dt = O.F16 if w.dtype == "f16" else O.BF16
    rows = min(rows, x.shape[0])
    c = O.compress(x[:rows], dt, tau, bit_set, eps, O.BUDGET_REL_RMS, nthreads=1)
    ok = (np.array_equal(sec["bits"][:rows], c.bits) and
          np.array_equal(sec["scale"][:rows].view(np.uint32), c.scale.view(np.uint32)) and
          np.array_equal(sec["pay_off"][: rows + 1], c.pay_off) and np.array_equal(sec["row_ptr"][: rows + 1], c.row_ptr) and
          np.array_equal(sec["payload"][: c.payload_bytes], c.payload) and
          np.array_equal(sec["out_col"][: c.nnz], c.out_col) and np.array_equal(sec["out_val"][: c.nnz], c.out_val))
    return {"rows": rows, "bit_exact": bool(ok)}


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


def copy_ceilings(tsq, torch, srcs, dsts, nbytes, stream, reps=40):
    """What kernels that only move bytes reach on this card in this run: a plain copy (nbytes read + nbytes
    written) and a read-only pass, over the rotating buffer sets.  -> GB/s of bytes moved."""
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for timed in (False, True):
        if timed:
            ev[0].record()
        for i in range(reps):
            tsq.tsq_measure_copy(dsts[i % len(dsts)].data_ptr(), srcs[i % len(srcs)].data_ptr(), nbytes, stream)
        if timed:
            ev[1].record()
        for i in range(reps):
            tsq.tsq_measure_read(srcs[i % len(srcs)].data_ptr(), nbytes, sink.data_ptr(), stream)
        if timed:
            ev[2].record()
    torch.cuda.synchronize()
    ms_copy, ms_read = ev[0].elapsed_time(ev[1]) / reps, ev[1].elapsed_time(ev[2]) / reps
    return {"copy_GBps": 2.0 * nbytes / ms_copy / 1e6, "read_GBps": nbytes / ms_read / 1e6,
            "copy_ms": ms_copy, "read_ms": ms_read, "bytes": nbytes,
            "what": "tsq_measure_copy / tsq_measure_read over %d buffer sets, %d launches each" % (len(srcs), reps)}


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
    nblob = max(nbuf, 2)                   # (two streams: a blob is read while the next one is written)
    blobs = [plan.new_blob() for _ in range(nblob)]
    ws = plan.new_workspace()

    def compress(k, kb):
        if parts:
            plan.compress_batch(xs[k], blobs[kb], ws, table=tin[k])
        else:
            plan.compress(xs[k], blobs[kb], ws)

    def decompress(k, kb):
        if parts:
            plan.decompress_batch(blobs[kb], outs[k], table=tout[k])
        else:
            plan.decompress(blobs[kb], outs[k])

    def step(i, ev=None):
        k = i % nbuf
        if ev:
            ev[0].record()
        compress(k, k)
        if ev:
            ev[1].record()
        decompress(k, k)
        if ev:
            ev[2].record()

    # The same steps on two streams: every compress call on the current stream, every decompress call on a second
    # one, behind its compress call by an event; a blob is written again only when the decompress call that read it
    # has finished (another event).  Step i's decompress then overlaps step i+1's compress; every step still does
    # all of its work, in order.  (All compress calls share a stream, so no two single-pass kernels meet.)
    second = torch.cuda.Stream()
    written = [torch.cuda.Event() for _ in range(nblob)]
    read = [torch.cuda.Event() for _ in range(nblob)]

    def steps_on_two_streams(first, count):
        main_stream = torch.cuda.current_stream()
        for i in range(first, first + count):
            k, kb = i % nbuf, i % nblob
            if i - first >= nblob:
                main_stream.wait_event(read[kb])
            compress(k, kb)
            written[kb].record(main_stream)
            with torch.cuda.stream(second):
                second.wait_event(written[kb])
                decompress(k, kb)
                read[kb].record(second)
        main_stream.wait_stream(second)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    info = plan.info(blobs[0])
    assert info.status == 0
    # parity in the run that is timed: the head of the blob against the oracle
    parity = None
    if not args.no_cpu_baseline:
        parity = oracle_check(x, w, tau, bit_set, args.eps, plan.sections(blobs[0]))
        assert parity["bit_exact"], "the benchmarked blob differs from the oracle's"
        for i in range(args.warmup):              # the check idled the card: warm up again
            step(i)
        torch.cuda.synchronize()

    def timed_region(graph, two_streams=False):
        """Exactly K steps between two events on the stream (nothing else is enqueued in between; with two
        streams the second event waits for the second stream's last call)."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        if graph is not None:
            for _ in range(args.steps // graph_steps):
                graph.replay()
        elif two_streams:
            steps_on_two_streams(args.warmup, args.steps)
        else:
            for i in range(args.steps):
                step(args.warmup + i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps, (time.perf_counter() - t0) * 1e3 / args.steps

    # both launch modes: the steps enqueued one by one, and replayed from a HIP graph that holds a block of
    # them (K is a multiple of the block); the headline is the one asked for.  The stream pass comes first:
    # once a graph has been captured and instantiated in the process, the same kernels enqueued on a stream
    # take about 1.3 us longer each on this stack (measured: 84.4 -> 87.1 us per step), as they do in the graph
    ms_stream, wall_stream = timed_region(None)
    assert plan.info(blobs[0]).status == 0
    # compress / decompress split of the same steps (events between the two calls: not the headline)
    n_split = min(args.steps, 200)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_split)]
    for i in range(n_split):
        step(args.warmup + i, evs[i])
    torch.cuda.synchronize()
    ms_c = sum(e[0].elapsed_time(e[1]) for e in evs) / n_split
    ms_d = sum(e[1].elapsed_time(e[2]) for e in evs) / n_split

    n = T * H
    rho = info.nnz / n
    bbar = 8.0 * info.payload_bytes / n
    side = info.payload_bytes + 4 * info.nnz + 21 * T      # payload + CSR + per-token metadata
    alg_c = 2 * n + side                                   # compress: read input, write the blob
    alg_d = side + 2 * n                                   # decompress: read the blob, write output

    # per-kernel durations.  Single pass: compress is one kernel and decompress is one kernel, so each is timed
    # as a run of back-to-back launches over the rotating buffers between two events (an event pair around every
    # single launch reads 2-4 us more than the kernel lasts).  Staged pipeline: HIP events around every launch
    # inside the library (tsq_compress_timed).
    names = ["k_fused"] if pipe == "fused" else ["k_row_stats", "k_scan", "k_pack"]
    acc = [0.0] * len(names)

    def run_of(call):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for i in range(min(50, n_split)):
            call((args.warmup + i) % nbuf)
        ev[0].record()
        for i in range(n_split):
            call((args.warmup + i) % nbuf)
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / n_split

    if parts:
        ms_kc = run_of(lambda k: plan.compress_batch(xs[k], blobs[k], ws, table=tin[k]))
        ms_kd = run_of(lambda k: plan.decompress_batch(blobs[k], outs[k], table=tout[k]))
    else:
        ms_kc = run_of(lambda k: plan.compress(xs[k], blobs[k], ws))
        ms_kd = run_of(lambda k: plan.decompress(blobs[k], outs[k]))
    if pipe == "fused":
        acc = [ms_kc * n_split]
    else:
        assert not parts, "the staged pipeline is timed per kernel on single tensors"
        for i in range(n_split):
            k = (args.warmup + i) % nbuf
            ms = tsq.tsq_compress_timed(plan.handle, xs[k].data_ptr(), blobs[k].data_ptr(), ws.data_ptr(),
                                        plan._stream())
            for j in range(len(names)):
                acc[j] += ms[j]
        torch.cuda.synchronize()
    # algorithmic bytes of each kernel: what it must read and write once
    kalg = {"k_fused": alg_c, "k_row_stats": 2 * n + 9 * T, "k_scan": 29 * T, "k_pack": alg_c,
            "k_unpack": alg_d}
    kern = {nm: {"ms": acc[j] / n_split, "alg_bytes": kalg[nm]} for j, nm in enumerate(names)}
    # decompress in its place behind compress (it then finds most of the blob in the memory-side cache; a run of
    # decompress calls alone reads about 3 us longer, reported as ms_alone)
    kern["k_unpack"] = {"ms": ms_d, "alg_bytes": alg_d, "ms_alone": ms_kd}
    for v in kern.values():
        v["GBps"] = v["alg_bytes"] / v["ms"] / 1e6
    dom = max(kern, key=lambda nm: kern[nm]["ms"])
    achieved = kern[dom]["GBps"]
    pair_split_gbps = (alg_c + alg_d) / (ms_c + ms_d) / 1e6
    # counter figures: from the committed rocprofv3 summaries, and only while the kernels are the ones profiled
    rec = profile_records().get((w.name, pipe, args.eps, dom))
    sha = kernels_sha()
    traffic, valu = None, None
    if rec and rec.get("kernels_sha") == sha:
        traffic = rec.get("hbm_bytes")
        insts = rec.get("valu_wave_insts")
        if insts:
            ops = insts * 64.0 / (kern[dom]["ms"] * 1e-3)
            valu = {"wave_instructions": insts, "achieved_lane_ops_per_s": ops, "peak_lane_ops_per_s": VALU_PEAK_LANE_OPS,
                    "frac": ops / VALU_PEAK_LANE_OPS, "source": "profiles/" + rec["source"]}
    # what kernels that only move bytes reach here, over the same buffers
    if parts:
        ceil = copy_ceilings(tsq, torch, xs[0], outs[0], parts[0].size * 2, plan._stream(), reps=2 * len(parts))
    else:
        ceil = copy_ceilings(tsq, torch, xs, outs, 2 * n, plan._stream())
    # the two-stream pass: warm-up steps of its own, then K steps; its outputs must be those of the steps on one stream.
    # (It comes after the per-call timings: once a second stream has been used, an event pair around a single
    # call reads about 2 us more.)
    # (Left out when one stream or the graph is asked for by name: a kernel trace of such a run then holds no
    # kernels that ran side by side.)
    ms_two, wall_two, two_streams_failed = None, None, False
    if not args.graph and args.launch in ("auto", "two-streams"):
        step(0)                            # (the copy kernels above wrote to the outputs)
        torch.cuda.synchronize()
        if parts:
            want_out = [t.clone() for t in outs[0]]
            for t in outs[0]:
                t.zero_()
        else:
            want_out = outs[0].clone()
            outs[0].zero_()
        steps_on_two_streams(0, args.warmup)
        ms_two, wall_two = timed_region(None, two_streams=True)
        if all(plan.info(b, check=False).status == 0 for b in blobs):
            same = all(torch.equal(a, b) for a, b in zip(want_out, outs[0])) if parts else torch.equal(want_out, outs[0])
            assert same, "the steps on two streams restored something else than the steps on one"
        else:
            # a compress call gave up (a bounded wait of the single-pass kernel expired while another kernel held
            # the device): this pass does not count, and the workspace starts afresh for what follows
            two_streams_failed = True
            ms_two, wall_two = None, None
            ws = plan.new_workspace()
            for i in range(nblob):
                step(i)
            torch.cuda.synchronize()
            assert plan.info(blobs[0]).status == 0
        del want_out

    # the graph pass, last (see above)
    graph_steps = max(d for d in range(1, min(args.steps, 100) + 1) if args.steps % d == 0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(graph_steps):
                step(args.warmup + i)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(max(1, args.warmup // graph_steps)):
        graph.replay()                     # untimed
    ms_graph, wall_graph = timed_region(graph)
    launch = "graph" if args.graph else args.launch
    if launch == "auto" or (launch == "two-streams" and ms_two is None):
        launch = "two-streams" if ms_two is not None and ms_two < ms_stream else "stream"
    ms_per_step, wall = {"stream": (ms_stream, wall_stream), "graph": (ms_graph, wall_graph),
                         "two-streams": (ms_two, wall_two)}[launch]
    launch_name = {"stream": "stream", "graph": "hip graph",
                   "two-streams": "two streams: compress calls on one, decompress calls on the other, each behind its "
                                  "compress call by an event"}[launch]
    assert plan.info(blobs[0]).status == 0
    pair_gbps = (alg_c + alg_d) / ms_per_step / 1e6
    copy_pair_ms = (alg_c + alg_d) / (ceil["copy_GBps"] * 1e6)      # the pair's bytes at the copy kernel's rate

    res = {
        "metric": "compress+decompress GB/s of split-point activations",
        "value": 2.0 * n / ms_per_step / 1e6,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype,              # the tensors' storage type; the arithmetic is in "arith"
        "arith": "f32 products rounded to integer codes, integer sums, f64 budget test",
        "data": "synthetic",
        "config": {"workload": ("%s %dx%d %s" % (w.name, T, H, w.dtype)) +
                               (" as %d tensors of %d rows" % (len(parts), parts[0].shape[0]) if parts else ""),
                   "tau": tau,
                   "bit_set": list(bit_set), "budget": "%.3g x row RMS" % args.eps,
                   "pipeline": pipe, "launch": launch_name, "buffer_sets": nbuf, "mean_width": round(bbar, 3),
                   "outlier_fraction": round(rho, 6), "width_hist": list(info.width_hist),
                   "compression_ratio": round(2.0 * n / info.compressed_bytes, 3)},
        "launch_modes": {"stream_ms_per_step": ms_stream, "hip_graph_ms_per_step": ms_graph,
                         "two_streams_ms_per_step": ms_two, "graph_holds_steps": graph_steps,
                         "pair_frac": {"stream": (alg_c + alg_d) / ms_stream / 1e6 / HBM_PEAK_GBS,
                                       "hip_graph": (alg_c + alg_d) / ms_graph / 1e6 / HBM_PEAK_GBS,
                                       "two_streams": (alg_c + alg_d) / ms_two / 1e6 / HBM_PEAK_GBS if ms_two else None},
                         "two_streams_gave_up": two_streams_failed, "headline": launch},
        # the bar: algorithmic bytes of compress + decompress over the timed step, against the 8 TB/s peak
        "target": {"quantity": "roofline.pair_frac", "bar": 0.6, "met": pair_gbps / HBM_PEAK_GBS >= 0.6},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "frac_is": "algorithmic bytes of the dominant kernel / its duration (a run of back-to-back launches "
                                "between two HIP events) / peak",
                     "pair_achieved": pair_gbps, "pair_frac": pair_gbps / HBM_PEAK_GBS,
                     "pair_frac_is": "algorithmic bytes of compress + decompress / ms_per_step / peak",
                     "compress_ms": ms_c, "decompress_ms": ms_d,
                     "pair_frac_split": pair_split_gbps / HBM_PEAK_GBS,
                     "pair_frac_split_is": "the same over compress_ms + decompress_ms, each call between events of its own",
                     "copy_ceiling": ceil,
                     "pair_vs_copy": copy_pair_ms / ms_per_step,
                     "pair_vs_copy_is": "time a plain copy kernel needs for the pair's algorithmic bytes / ms_per_step",
                     "valu_issue": valu, "kernels_sha": sha, "kernels": kern},
        "parity_check": parity,
        "host_wall_ms_per_step": wall,
    }
    if not args.no_cpu_baseline:
        rows = args.cpu_sample_rows or max(64, min(T, int(2.5e8 // H)))
        res["cpu_baseline"] = cpu_baseline(x, w, tau, bit_set, args.eps, rows)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
