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
