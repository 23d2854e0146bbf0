"""Other readings of the paper's quantizer, side by side with the one the library implements.

TEST INFRASTRUCTURE ONLY (see tsq_oracle.py).  Nothing here is a product path: the module
exists to put numbers on how much three readings of Sec. II-C.2 matter.

  literal_break   Algorithm 1 as printed returns the quantization at the width whose distortion
                  EXCEEDED the budget; the library returns the last width that passed.
  with_minimum    Eq. (Proposed) as printed takes the step from T_max - T_min and carries a zero
                  point; the library pins T_min to 0 (magnitudes of T_below contain zeros wherever
                  an element was split off, and otherwise come within a fraction of a step of 0).
  whole_tensor    Algorithm 1 as printed runs over all n = W x HD elements at once (one absmax,
                  one width); the library works token by token, as the section title says.

Every variant reuses the row primitives of the C file (tsqo_ts_row, tsqo_aiq_row,
tsqo_select_row) for the arithmetic they share with the baseline, so that a difference in the
numbers below is a difference of the reading and of nothing else.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import tsq_oracle as O


@dataclass
class Outcome:
    bits: np.ndarray        # width per token
    recon: np.ndarray       # f32 [T, H]: reconstruction of T_below (outlier slots 0), before the 16-bit store
    inl: np.ndarray         # f32 [T, H]: |T_below| with signs, what recon approximates

    def mean_width(self) -> float:
        return float(self.bits.astype(np.float64).mean())

    def rel_rmse(self) -> float:
        d = self.recon.astype(np.float64) - self.inl.astype(np.float64)
        return float(np.sqrt((d * d).sum() / max((self.inl.astype(np.float64) ** 2).sum(), 1e-300)))


def _widths(bit_set):
    return sorted({int(b) for b in bit_set}, reverse=True)


def _split(x, dtype, tau):
    T, H = x.shape
    a = np.zeros((T, H), np.float32)
    amax = np.zeros(T, np.float32)
    for t in range(T):
        _, a[t], _, amax[t] = O.ts_row(x[t], dtype, tau)
    v = O.widen(x, dtype) if T * H <= 1 << 16 else _widen_fast(x, dtype)
    sign = np.where(np.signbit(v), np.float32(-1), np.float32(1))
    return a, amax, sign


def _widen_fast(x, dtype):
    if dtype == O.F16:
        return x.view(np.float16).astype(np.float32)
    return (x.astype(np.uint32) << 16).view(np.float32)


def _dequant(a_row, amax, b):
    m, _, s = O.aiq_row(a_row, amax, b)
    return m.astype(np.float32) * np.float32(s)


def baseline(x, dtype, tau, bit_set, budget, mode) -> Outcome:
    a, amax, sign = _split(x, dtype, tau)
    T = x.shape[0]
    bits = np.zeros(T, np.uint8)
    rec = np.zeros_like(a)
    for t in range(T):
        info = O.select_row(a[t], amax[t], bit_set, budget, mode)
        bits[t] = info["bits"]
        rec[t] = _dequant(a[t], amax[t], int(bits[t]))
    return Outcome(bits, rec * sign, a * sign)


def literal_break(x, dtype, tau, bit_set, budget, mode) -> Outcome:
    """The width at which the test first fails (the smallest allowed width if it never fails).  Derived
    here from the default descent's record (how many candidates it evaluated); the C file's own switch
    (TSQO_RETURN_AS_PRINTED) must give the same widths, which tests check."""
    a, amax, sign = _split(x, dtype, tau)
    W = _widths(bit_set)
    T = x.shape[0]
    bits = np.zeros(T, np.uint8)
    rec = np.zeros_like(a)
    for t in range(T):
        info = O.select_row(a[t], amax[t], bit_set, budget, mode)
        n, sel = int(info["n_eval"]), int(info["bits"])
        # candidates 1..n were evaluated; the descent stopped at n iff candidate n is not the selected width
        stopped = n >= 1 and W[n] != sel
        bits[t] = W[n] if stopped else W[-1]
        rec[t] = _dequant(a[t], amax[t], int(bits[t]))
    return Outcome(bits, rec * sign, a * sign)


def with_minimum(x, dtype, tau, bit_set, budget, mode) -> Outcome:
    """Same widths as the baseline; step (T_max - T_min) / Q with zero point z = rint(T_min / s),
    codes rint(a / s) - z clamped to [0, Q], reconstruction (code + z) * s."""
    a, amax, sign = _split(x, dtype, tau)
    T = x.shape[0]
    bits = np.zeros(T, np.uint8)
    rec = np.zeros_like(a)
    for t in range(T):
        info = O.select_row(a[t], amax[t], bit_set, budget, mode)
        b = int(info["bits"])
        bits[t] = b
        Q = np.float32((1 << (b - 1)) - 1)
        amin = np.float32(a[t].min())
        span = np.float32(amax[t] - amin)
        if not span > 0:
            rec[t] = a[t]                               # constant magnitudes: nothing to quantize
            continue
        s = np.float32(span / Q)
        z = np.rint(np.float32(amin / s))
        q = np.clip(np.rint((a[t] / s).astype(np.float32)) - z, 0, Q)
        rec[t] = ((q + z) * s).astype(np.float32)
    return Outcome(bits, rec * sign, a * sign)


def whole_tensor(x, dtype, tau, bit_set, budget, mode) -> Outcome:
    """One absmax and one width for all T x H elements."""
    a, _, sign = _split(x, dtype, tau)
    T, H = a.shape
    flat = np.ascontiguousarray(a.reshape(-1))
    amax = np.float32(flat.max())
    info = O.select_row(flat, amax, bit_set, budget, mode)
    b = int(info["bits"])
    rec = _dequant(flat, amax, b).reshape(T, H)
    return Outcome(np.full(T, b, np.uint8), rec * sign, a * sign)


VARIANTS = {"library": baseline, "literal_break": literal_break, "with_minimum": with_minimum,
            "whole_tensor": whole_tensor}


def table(x, dtype, tau, bit_set, budget, mode=O.BUDGET_REL_RMS) -> dict:
    return {k: {"mean_width": o.mean_width(), "rel_rmse": o.rel_rmse()}
            for k, o in ((k, f(x, dtype, tau, bit_set, budget, mode)) for k, f in VARIANTS.items())}


if __name__ == "__main__":
    # python -m oracle.variants : the table quoted in the design notes
    import json
    from paper_2511_04002_amd import synth
    O.build()
    cases = [("C1", synth.make_c1(), O.F16), ("C2 (256 tokens)", synth.make_c2(tokens=256), O.F16),
             ("C4 (128 tokens)", synth.make_c4(tokens=128), O.BF16)]
    for name, x, dt in cases:
        w = synth.WORKLOADS[name.split()[0]]
        for eps in (0.05, 0.2):
            print(name, "eps", eps, json.dumps(table(x, dt, w.tau, w.bit_set, eps)))
