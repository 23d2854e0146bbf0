"""Algorithm 2 (early exit under a delay constraint, Sec. II-D.2) driven by sizes measured on the GPU.

    python -m paper_2511_04002_amd.early_exit [--tokens 512] [--layers 20]

The hidden state of `tokens` tokens at the split layer and the KV cache of the `layers` layers
below it (synthetic, 7B-shaped: HD = 4096, fp16) are compressed with tsq_compress /
tsq_compress_batch; their compressed sizes, token by token for the hidden state, feed
tsq_early_exit_decide together with the link of the paper's evaluation (W = 10 MHz, SNR 10,
outage 0.001) at the rate tsq_link_best_rate finds.  The local computation latency L_c(w) is a
stand-in (the paper profiles it on its edge device): c0 + c1 * w.  One JSON line per deadline.
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def prefix_bits(sections, tokens: int):
    """Compressed size in bits of the first k tokens of a blob, k = 0 .. tokens: header, per-token
    width and scale, the two offset tables, payload and CSR entries."""
    k = np.arange(tokens + 1, dtype=np.uint64)
    pay, nnz = sections["pay_off"][: tokens + 1], sections["row_ptr"][: tokens + 1]
    return (np.uint64(8) * (np.uint64(128) + np.uint64(5) * k + np.uint64(16) * (k + np.uint64(1)) + pay +
                            np.uint64(4) * nnz)).tolist()


def measure(tokens: int, layers: int, eps: float = 0.05):
    """-> (raw_bits, compressed_bits_with_kv, hidden_prefix_bits) from GPU compress calls."""
    import torch
    from . import synth, tsq
    w2, wk = synth.WORKLOADS["C2"], synth.WORKLOADS["KV7"]
    H = w2.hidden
    hid = synth.make_c2(tokens=tokens)
    plan = tsq.Plan(tokens, H, w2.dtype, w2.tau, w2.bit_set, eps, max_outliers=tokens * H // 8)
    blob = plan.compress(torch.from_numpy(hid.view(np.int16)).cuda())
    info = plan.info(blob)
    pre = prefix_bits(plan.sections(blob), tokens)
    assert pre[-1] == 8 * info.compressed_bytes
    kv = [torch.from_numpy(p.view(np.int16)).cuda() for p in synth.make_kv("KV7", layers=layers, rows=tokens)]
    plan_kv = tsq.Plan(2 * layers * tokens, H, wk.dtype, wk.tau, wk.bit_set, eps,
                       max_outliers=2 * layers * tokens * H // 8)
    blob_kv, _ = plan_kv.compress_batch(kv)
    info_kv = plan_kv.info(blob_kv)
    raw = 16.0 * (tokens * H + 2 * layers * tokens * H)           # Eq. (if_total), I_kv = 1, 16-bit activations
    return raw, 8.0 * (info.compressed_bytes + info_kv.compressed_bytes), pre


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=512)
    ap.add_argument("--layers", type=int, default=20)
    ap.add_argument("--c0", type=float, default=0.05, help="L_c(w) = c0 + c1 * w, seconds")
    ap.add_argument("--c1", type=float, default=0.002)
    args = ap.parse_args()
    from . import tsq
    raw, with_kv, pre = measure(args.tokens, args.layers)
    link = tsq.tsq_link(10e6, 10.0, 1e-3)
    rate = tsq.tsq_link_best_rate(link, 1e5, 1e8, 2000)
    lc = [args.c0 + args.c1 * k if k else 0.0 for k in range(args.tokens + 1)]
    names = {0: "continue", 1: "compressed", 2: "without_kv", 3: "fewer_tokens"}
    print(json.dumps({"rate_bits_per_s": rate, "outage_probability": tsq.tsq_link_outage_probability(link, rate),
                      "raw_bits": raw, "compressed_bits_with_kv": with_kv, "compressed_bits_hidden": pre[-1]}))
    for D in (1e4, 1e3, 300.0, 100.0, 30.0, 10.0, 3.0, 1.0, 0.3):
        d = tsq.tsq_early_exit_decide(link, rate, D, lc, raw, with_kv, pre)
        print(json.dumps({"deadline_s": D, "action": names[d.action], "with_kv": d.with_kv, "tokens": d.tokens,
                          "latency_s": d.latency}))


if __name__ == "__main__":
    main()
