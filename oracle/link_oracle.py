"""The link model and the early-exit ladder of Sec. II-D.2, written out in plain Python floats.

TEST INFRASTRUCTURE ONLY (see tsq_oracle.py).

  outage_probability   P_o(R) = 1 - exp(-(2^(R/W) - 1) / gamma)                 (below Eq. (comm_latency))
  latency              L_eps(D_tx; R) = D_tx / R * ceil(ln eps / ln P_o(R))      (Eq. (comm_latency))
  best_rate            Eq. (epsilon_rstar) by one-dimensional search on a uniform grid.  Reading: the
                       text defines g(R) = ln(1/P_o(R)) / R and takes its minimiser, but that g falls
                       monotonically to 0 as P_o -> 1 (its minimiser is the rate at which every
                       transmission fails).  What Eq. (comm_latency) makes small, ceiling aside, is
                       D_tx ln(1/eps) / (R ln(1/P_o(R))), so the rate sought maximises
                       R ln(1/P_o(R)); that is what is searched for here.
  early_exit           Algorithm 2 for one (w, layer): as it is -> compressed -> without the KV cache
                       -> fewer tokens, total latency L_c(w) + L_eps (Eq. (total))
  early_exit_walk      Algorithm 2 with its two loops (for w = 1 .. W-bar, for layer = 1 .. L), in the
                       printed order of steps.  Readings: (a) when dropping the KV cache brings the
                       latency under the deadline the printed steps do not return, so the walk goes on
                       with I_kv = 0 from there; (b) "w <- w - 1" stops at zero tokens; (c) L_c of a
                       shortened output is that of the tokens kept (as in early_exit above).
"""
from __future__ import annotations

import math


def outage_probability(W: float, gamma: float, rate: float) -> float:
    return 1.0 - math.exp(-(2.0 ** (rate / W) - 1.0) / gamma)


def transmissions(W: float, gamma: float, eps: float, rate: float) -> float:
    po = outage_probability(W, gamma, rate)
    if po >= 1.0:
        return math.inf
    if po <= 0.0:
        return 1.0
    return max(1.0, math.ceil(math.log(eps) / math.log(po)))


def latency(W: float, gamma: float, eps: float, bits: float, rate: float) -> float:
    if bits <= 0:
        return 0.0
    return bits / rate * transmissions(W, gamma, eps, rate)


def goodput_exponent(W: float, gamma: float, rate: float) -> float:
    """R * ln(1 / P_o(R)): the larger, the shorter the worst-case delay."""
    return rate * math.log(1.0 / outage_probability(W, gamma, rate))


def best_rate(W: float, gamma: float, lo: float, hi: float, steps: int) -> float:
    rates = [lo + (hi - lo) * (i / steps) for i in range(steps + 1)]
    vals = [goodput_exponent(W, gamma, r) for r in rates]
    return rates[vals.index(max(vals))]


CONTINUE, COMPRESSED, WITHOUT_KV, FEWER_TOKENS = 0, 1, 2, 3


def early_exit(W, gamma, eps, rate, deadline, compute_latency, raw_bits, compressed_bits_with_kv,
               hidden_prefix_bits):
    """-> (action, with_kv, tokens, latency)."""
    w = len(compute_latency) - 1
    lat = compute_latency[w] + latency(W, gamma, eps, raw_bits, rate)
    if lat <= deadline:
        return CONTINUE, 1, w, lat
    lat = compute_latency[w] + latency(W, gamma, eps, compressed_bits_with_kv, rate)
    if lat <= deadline:
        return COMPRESSED, 1, w, lat
    lat = compute_latency[w] + latency(W, gamma, eps, hidden_prefix_bits[w], rate)
    if lat <= deadline:
        return WITHOUT_KV, 0, w, lat
    while lat > deadline and w > 0:
        w -= 1
        lat = compute_latency[w] + latency(W, gamma, eps, hidden_prefix_bits[w], rate)
    return FEWER_TOKENS, 0, w, lat


COMPLETED = 4


def early_exit_walk(W, gamma, eps, rate, deadline, max_tokens, layers, compute_latency, bits):
    """compute_latency(w, layer) -> seconds; bits(w, layer, with_kv, compressed, keep) -> size in bits of
    what is sent after w tokens at `layer`: raw (compressed = 0) or through TS + TAB-Q with only the first
    `keep` tokens of the hidden state.  -> (action, with_kv, tokens, layer, kept, latency)."""
    ikv = 1
    for w in range(1, max_tokens + 1):
        for layer in range(1, layers + 1):
            lat = compute_latency(w, layer) + latency(W, gamma, eps, bits(w, layer, ikv, 0, w), rate)
            if lat > deadline:
                lat = compute_latency(w, layer) + latency(W, gamma, eps, bits(w, layer, ikv, 1, w), rate)
                if lat <= deadline:
                    return COMPRESSED, ikv, w, layer, w, lat
                ikv = 0
                lat = compute_latency(w, layer) + latency(W, gamma, eps, bits(w, layer, 0, 1, w), rate)
                if lat > deadline:
                    keep = w
                    while lat > deadline and keep > 0:
                        keep -= 1
                        lat = compute_latency(keep, layer) + latency(W, gamma, eps, bits(w, layer, 0, 1, keep), rate)
                    return FEWER_TOKENS, 0, w, layer, keep, lat
    w, layer = max_tokens, layers
    lat = compute_latency(w, layer) + latency(W, gamma, eps, bits(w, layer, ikv, 1, w), rate)
    return COMPLETED, ikv, w, layer, w, lat
