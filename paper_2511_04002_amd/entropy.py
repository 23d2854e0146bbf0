"""Achievable-entropy report for a workload: how far below the packed size an entropy coder
placed after TAB-Q (Sec. II-C.2, last paragraph) could go.

    python -m paper_2511_04002_amd.entropy --workload C4 [--eps 0.05]

Compresses the workload on the GPU, counts the codes of every token with tsq_code_histogram, and
prints one JSON line: bits per element as packed (the mean width), with an ideal coder that has
one frequency table per token, and with one table per width class; the side costs of those
tables are listed next to them (a table entry taken as 2 bytes).  Also the duration of the
histogram kernel and the HBM rate it corresponds to (payload read + table written).
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def shannon_bits(counts: np.ndarray) -> float:
    """Bits an ideal coder needs for the symbols counted in `counts` (the report's own figure, from the
    library's entropy routine; no kernel and no test depends on it)."""
    from scipy.stats import entropy
    total = float(np.asarray(counts, np.float64).sum())
    return total * float(entropy(np.asarray(counts, np.float64).ravel(), base=2)) if total > 0 else 0.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "KV7", "KV13"],
                    help="KV7 / KV13: the cache of the batch form (one blob for all the per-layer key and value tensors)")
    ap.add_argument("--eps", type=float, default=0.05)
    ap.add_argument("--steps", type=int, default=20)
    args = ap.parse_args()
    from . import synth
    w = synth.WORKLOADS[args.workload]
    kv = args.workload.startswith("KV")
    parts = synth.make_kv(args.workload) if kv else None
    x = None if kv else (synth.make_c3(0) if args.workload == "C3" else synth.make(args.workload))
    import torch
    from . import tsq
    tsq.lib()
    T, H = (len(parts) * parts[0].shape[0], parts[0].shape[1]) if kv else x.shape
    plan = tsq.Plan(T, H, w.dtype, w.tau, w.bit_set, args.eps, max_outliers=max(1, T * H // 8))
    if kv:
        tensors = [torch.from_numpy(t.view(np.int16)).cuda() for t in parts]
        blob, _table = plan.compress_batch(tensors)
        torch.cuda.synchronize()
    else:
        blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    info = plan.info(blob)
    hist = plan.code_histogram(blob)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        plan.code_histogram(blob, hist)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    h = hist.cpu().numpy().view(np.uint32)
    bits = plan.sections(blob)["bits"]
    n = float(T) * H
    per_token = sum(shannon_bits(h[t]) for t in range(T))
    widths = sorted(set(bits.tolist()))
    pooled = sum(shannon_bits(h[bits == b].sum(axis=0, dtype=np.uint64)) for b in widths)
    table_per_token = float(sum(16.0 * (1 << int(b)) for b in bits))        # 2-byte entries
    table_per_width = float(sum(16.0 * (1 << int(b)) for b in widths))
    moved = info.payload_bytes + 1024.0 * T
    # the coder itself: encode (counts, tables, streams) and decode, timed the same way
    eblob, ews = plan.new_entropy_blob(), plan.new_entropy_workspace()
    plan.entropy_encode(blob, eblob, ews)
    einfo = tsq.tsq_entropy_info(plan.handle, eblob.data_ptr(), plan._stream())
    back = blob.clone()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record()
    for _ in range(args.steps):
        plan.entropy_encode(blob, eblob, ews)
    ev[1].record()
    for _ in range(args.steps):
        plan.entropy_decode(eblob, back)
    ev[2].record()
    torch.cuda.synchronize()
    assert torch.equal(back, blob)
    ms_enc, ms_dec = ev[0].elapsed_time(ev[1]) / args.steps, ev[1].elapsed_time(ev[2]) / args.steps
    print(json.dumps({
        "workload": "%s %dx%d %s" % (w.name, T, H, w.dtype), "budget": "%.3g x row RMS" % args.eps,
        "bits_per_element": {
            "packed": 8.0 * info.payload_bytes / n,
            "ideal_one_table_per_token": per_token / n,
            "ideal_one_table_per_token_with_tables": (per_token + table_per_token) / n,
            "ideal_one_table_per_width": pooled / n,
            "ideal_one_table_per_width_with_tables": (pooled + table_per_width) / n},
        "width_hist": list(info.width_hist),
        "k_code_hist": {"ms": ms, "bytes": moved, "GBps": moved / ms / 1e6, "frac_of_8TBps": moved / ms / 1e6 / 8000.0},
        "rans": {"stream_bytes": einfo.stream_bytes, "coded_bytes": einfo.coded_bytes, "payload_bytes": info.payload_bytes,
                 "bits_per_element": 8.0 * einfo.coded_bytes / n, "encode_ms": ms_enc, "decode_ms": ms_dec,
                 "encode_GBps_of_payload": info.payload_bytes / ms_enc / 1e6,
                 "decode_GBps_of_payload": info.payload_bytes / ms_dec / 1e6},
    }))


if __name__ == "__main__":
    main()
