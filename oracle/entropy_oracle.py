"""Symbol statistics of a compressed tensor, and what an ideal entropy coder would make of them.

TEST INFRASTRUCTURE ONLY (like tsq_oracle.py, which this module builds on): tests and the
measurement scripts' baseline legs may import it; the product package must not.

The paper hands the codes that TAB-Q produces to an rANS coder (Sec. II-C.2, last paragraph).
What such a coder can reach is fixed by the symbol counts:
  - code_histogram: per token, how often each b_t-bit code (sign bit on top of the magnitude,
    the field of the payload) occurs -- the definition written out: unpack the token's fields,
    count them with numpy.bincount;
  - entropy_bits: Shannon's bound  sum_c n_c * log2(N / n_c)  in bits for one table of counts
    (fp64), the size below which no coder that knows only this table can go.
"""
from __future__ import annotations

import numpy as np

from . import tsq_oracle as O


def token_codes(c: "O.Compressed", t: int) -> np.ndarray:
    """The H codes of token t as stored: (neg << (b-1)) | m."""
    b = int(c.bits[t])
    lo, hi = int(c.pay_off[t]), int(c.pay_off[t + 1])
    m, neg = O.unpack_row(c.payload[lo:hi], c.hidden, b)
    return (neg.astype(np.uint32) << np.uint32(b - 1)) | m.astype(np.uint32)


def code_histogram(c: "O.Compressed") -> np.ndarray:
    """-> u32 [T, 256]; row t counts the codes of token t, entries >= 2^b_t are 0."""
    out = np.zeros((c.tokens, 256), np.uint32)
    for t in range(c.tokens):
        out[t] = np.bincount(token_codes(c, t), minlength=256)
    return out


def entropy_bits(counts: np.ndarray) -> float:
    """Shannon bound in bits for coding sum(counts) symbols drawn with these counts."""
    n = np.asarray(counts, np.float64).ravel()
    n = n[n > 0]
    N = n.sum()
    return float((n * np.log2(N / n)).sum()) if N > 0 else 0.0


def report(hist: np.ndarray, bits: np.ndarray, hidden: int) -> dict:
    """Bits per element: as packed (mean width), with one ideal table per token, with one ideal
    table per width class shared by all tokens of that width."""
    T = hist.shape[0]
    per_token = sum(entropy_bits(hist[t]) for t in range(T))
    pooled = 0.0
    for b in np.unique(bits):
        pooled += entropy_bits(hist[bits == b].sum(axis=0, dtype=np.uint64))
    n = float(T) * hidden
    return {"packed": float(bits.astype(np.float64).mean()), "per_token_table": per_token / n,
            "per_width_table": pooled / n}
