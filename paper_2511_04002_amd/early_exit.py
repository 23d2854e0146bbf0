"""Algorithm 2 (early exit under a delay constraint, Sec. II-D.2) driven by sizes measured on the GPU.

    python -m paper_2511_04002_amd.early_exit [--tokens 512] [--layers 20]
    python -m paper_2511_04002_amd.early_exit --walk --tokens 32 --layers 8     (both loops of Algorithm 2)

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


def measure(tokens: int, layers: int, eps: float = 0.05, entropy: bool = False):
    """-> (raw_bits, compressed_bits_with_kv, hidden_prefix_bits) from GPU compress calls.  entropy: the codes
    travel through the rANS stage (tsq_entropy_encode; sizes from tsq_entropy_prefix_bytes)."""
    import torch
    from . import synth, tsq
    w2, wk = synth.WORKLOADS["C2"], synth.WORKLOADS["KV7"]
    H = w2.hidden
    hid = synth.make_c2(tokens=tokens)
    plan = tsq.Plan(tokens, H, w2.dtype, w2.tau, w2.bit_set, eps, max_outliers=tokens * H // 8)
    blob = plan.compress(torch.from_numpy(hid.view(np.int16)).cuda())
    info = plan.info(blob)
    if entropy:
        eblob = plan.entropy_encode(blob)
        pre = [8 * v for v in plan.entropy_prefix_bytes(blob, eblob)]
        einfo = tsq.tsq_entropy_info(plan.handle, eblob.data_ptr(), plan._stream())
        hidden_bytes = info.compressed_bytes - info.payload_bytes + einfo.coded_bytes
    else:
        pre = [8 * v for v in plan.prefix_bytes(blob)]      # bits, k = 0 .. tokens (tsq_prefix_bytes)
        hidden_bytes = info.compressed_bytes
    assert pre[-1] == 8 * hidden_bytes
    kv = [torch.from_numpy(p.view(np.int16)).cuda() for p in synth.make_kv("KV7", layers=layers, rows=tokens)]
    plan_kv = tsq.Plan(2 * layers * tokens, H, wk.dtype, wk.tau, wk.bit_set, eps,
                       max_outliers=2 * layers * tokens * H // 8)
    blob_kv, _ = plan_kv.compress_batch(kv)
    info_kv = plan_kv.info(blob_kv)
    kv_bytes = info_kv.compressed_bytes
    if entropy:
        eblob_kv = plan_kv.entropy_encode(blob_kv)
        kv_bytes += tsq.tsq_entropy_info(plan_kv.handle, eblob_kv.data_ptr(), plan_kv._stream()).coded_bytes - info_kv.payload_bytes
    raw = 16.0 * (tokens * H + 2 * layers * tokens * H)           # Eq. (if_total), I_kv = 1, 16-bit activations
    return raw, 8.0 * (hidden_bytes + kv_bytes), pre


class StepSizes:
    """Sizes for Algorithm 2's walk, measured on the GPU when the walk asks for them: the hidden state of w
    tokens at the split layer and the KV cache of the `layer` layers below it, compressed with tsq_compress /
    tsq_compress_batch (one plan per shape, kept)."""

    def __init__(self, max_tokens: int, layers: int, eps: float = 0.05, entropy: bool = False):
        import torch
        from . import synth, tsq
        self.tsq, self.torch, self.entropy = tsq, torch, entropy
        self.w2, self.wk, self.eps = synth.WORKLOADS["C2"], synth.WORKLOADS["KV7"], eps
        self.H = self.w2.hidden
        self.hid = torch.from_numpy(synth.make_c2(tokens=max_tokens).view(np.int16)).cuda()
        self.kv = [torch.from_numpy(p.view(np.int16)).cuda()
                   for p in synth.make_kv("KV7", layers=layers, rows=max_tokens)]       # K_1, V_1, K_2, ...
        self.cache = {}
        self.compress_calls = 0

    def hidden_prefix_bits(self, w: int):
        key = ("h", w)
        if key not in self.cache:
            plan = self.tsq.Plan(w, self.H, self.w2.dtype, self.w2.tau, self.w2.bit_set, self.eps,
                                 max_outliers=max(1, w * self.H // 8))
            blob = plan.compress(self.hid[:w].contiguous())
            self.compress_calls += 1
            if self.entropy:
                self.cache[key] = [8 * v for v in plan.entropy_prefix_bytes(blob, plan.entropy_encode(blob))]
            else:
                self.cache[key] = [8 * v for v in plan.prefix_bytes(blob)]
        return self.cache[key]

    def kv_bits(self, w: int, layer: int) -> float:
        key = ("kv", w, layer)
        if key not in self.cache:
            plan = self.tsq.Plan(2 * layer * w, self.H, self.wk.dtype, self.wk.tau, self.wk.bit_set, self.eps,
                                 max_outliers=max(1, 2 * layer * w * self.H // 8))
            blob, _ = plan.compress_batch([t[:w].contiguous() for t in self.kv[: 2 * layer]])
            self.compress_calls += 1
            info = plan.info(blob)
            nbytes = info.compressed_bytes
            if self.entropy:
                eblob = plan.entropy_encode(blob)
                nbytes += self.tsq.tsq_entropy_info(plan.handle, eblob.data_ptr(), plan._stream()).coded_bytes - info.payload_bytes
            self.cache[key] = 8.0 * nbytes
        return self.cache[key]

    def bits(self, w, layer, with_kv, compressed, keep):
        if not compressed:                                    # Eq. (if_total), 16-bit activations
            return 16.0 * (keep * self.H + (2 * layer * w * self.H if with_kv else 0))
        return float(self.hidden_prefix_bits(w)[keep]) + (self.kv_bits(w, layer) if with_kv else 0.0)


def walk(max_tokens: int, layers: int, c0: float, c1: float, deadlines, entropy: bool = False):
    """Algorithm 2 with both loops (tsq_early_exit_walk); sizes are measured at the step that needs them."""
    from . import tsq
    sizes = StepSizes(max_tokens, layers, entropy=entropy)
    link = tsq.tsq_link(10e6, 10.0, 1e-3)
    rate = tsq.tsq_link_best_rate(link, 1e5, 1e8, 2000)
    names = {1: "compressed", 3: "fewer_tokens", 4: "completed"}
    for D in deadlines:
        r = tsq.tsq_early_exit_walk(link, rate, D, max_tokens, layers, lambda w, layer: (c0 + c1 * w) * layer / layers if w else 0.0,
                                    sizes.bits)
        print(json.dumps({"deadline_s": D, "action": names[r.action], "with_kv": r.with_kv, "tokens": r.tokens,
                          "layer": r.layer, "sent_tokens": r.sent_tokens, "steps": r.steps, "latency_s": r.latency,
                          "compress_calls_so_far": sizes.compress_calls}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=512)
    ap.add_argument("--layers", type=int, default=20)
    ap.add_argument("--c0", type=float, default=0.05, help="L_c(w) = c0 + c1 * w, seconds")
    ap.add_argument("--c1", type=float, default=0.002)
    ap.add_argument("--entropy", action="store_true",
                    help="the codes travel through the rANS stage (sizes from tsq_entropy_prefix_bytes)")
    ap.add_argument("--walk", action="store_true",
                    help="run Algorithm 2's loops over w = 1..tokens and layer = 1..layers, measuring sizes at each exit")
    args = ap.parse_args()
    if args.walk:
        walk(args.tokens, args.layers, args.c0, args.c1, (10.0, 1.0, 0.3, 0.1, 0.03, 0.01, 0.003), entropy=args.entropy)
        return
    from . import tsq
    raw, with_kv, pre = measure(args.tokens, args.layers, entropy=args.entropy)
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
