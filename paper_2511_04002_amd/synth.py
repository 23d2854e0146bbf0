"""Seeded synthetic split-point activations.

This module only draws numbers: it holds none of the method's arithmetic and is
the one piece of code that both the GPU tests and the CPU checker feed from, so
that both sides see identical bytes.  The tensors stand in for hidden states at
the split layer of the models the paper evaluates (Sec. III, evaluation setup);
real activations are not needed and not used.

Every recipe draws in float64 with numpy's PCG64 generator, in the order the
code states, then casts once to the 16-bit storage type (fp16 through numpy,
bf16 by round-to-nearest-even on the fp32 bit pattern).  Arrays are returned as
raw uint16 bit patterns, shape [tokens, hidden], row-major.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    tokens: int            # rows per call
    hidden: int
    dtype: str             # "f16" | "bf16"
    tau: float
    bit_set: Tuple[int, ...]
    budget: float = 0.05   # epsilon, relative to the row RMS
    mode: str = "rel_rms"
    steps: int = 1         # independent calls per run (decode regime)
    note: str = ""


WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", 128, 768, "f16", 6.0, (2, 4, 8),
                   note="tiny: N(0,1), channels 17 and 401 x50"),
    "C2": Workload("C2", 2048, 4096, "f16", 8.0, (2, 3, 4, 6, 8),
                   note="7B-shaped prefill: per-token lognormal scale, 6 outlier channels, 0.01% spikes"),
    "C3": Workload("C3", 512, 5120, "f16", 8.0, (2, 4, 8), steps=64,
                   note="13B-shaped decode: 512 sequences x 1 token per step, 8 outlier channels"),
    "C4": Workload("C4", 8192, 8192, "bf16", 10.0, (2, 3, 4, 5, 6, 8),
                   note="70B-shaped prefill: Student-t(5) x per-token lognormal(0,0.7), 12 outlier channels"),
    "C5": Workload("C5", 131072, 8192, "bf16", 8.0, (2, 4, 8),
                   note="stress: 32 sequences x 4096 tokens, Student-t(3), 16 channels, 1% unstructured outliers"),
}

# KV-cache workloads (Sec. II-B, Eq. (bkv_lth_stage)): the key and value tensors of every layer for
# w cached tokens, each [w x HD]; `tokens` counts the rows of all of them.  Shapes of the two models
# the paper evaluates (Llama-2 7B: 32 layers, HD 4096; 13B: 40 layers, HD 5120), w = 1024.
KV_WORKLOADS: Dict[str, Tuple[int, int]] = {"KV7": (32, 1024), "KV13": (40, 1024)}   # layers, w
WORKLOADS["KV7"] = Workload("KV7", 2 * 32 * 1024, 4096, "f16", 8.0, (2, 3, 4, 6, 8),
                            note="KV cache, 7B-shaped: 64 tensors [1024 x 4096]")
WORKLOADS["KV13"] = Workload("KV13", 2 * 40 * 1024, 5120, "f16", 8.0, (2, 3, 4, 6, 8),
                             note="KV cache, 13B-shaped: 80 tensors [1024 x 5120]")

# C5 is swept over these thresholds and bit sets
C5_TAUS = (4.0, 8.0, 16.0)
C5_BIT_SETS = ((2, 4, 8), (2, 3, 4, 5, 6, 7, 8))
C5_SEQ_TOKENS = 4096
C5_SEQS = 32


def to_f16_bits(x64: np.ndarray) -> np.ndarray:
    return x64.astype(np.float16).view(np.uint16)


def to_bf16_bits(x64: np.ndarray) -> np.ndarray:
    u = x64.astype(np.float32).view(np.uint32)
    # finite inputs only: round to nearest, ties to the even 16-bit pattern
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def _cast(x64: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f16":
        return to_f16_bits(x64)
    if dtype == "bf16":
        return to_bf16_bits(x64)
    raise ValueError(dtype)


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


def make_c1() -> np.ndarray:
    w = WORKLOADS["C1"]
    g = np.random.Generator(np.random.PCG64(0))
    x = g.standard_normal((w.tokens, w.hidden))
    x[:, 17] *= 50.0
    x[:, 401] *= 50.0
    return _cast(x, w.dtype)


def make_c2(tokens: Optional[int] = None) -> np.ndarray:
    w = WORKLOADS["C2"]
    T = tokens or w.tokens
    g = np.random.Generator(np.random.PCG64(1))
    x = g.standard_normal((T, w.hidden))
    x *= g.lognormal(0.0, 0.5, size=(T, 1))
    ch = g.choice(w.hidden, 6, replace=False)
    x[:, ch] *= g.uniform(20.0, 100.0, size=6)
    k = int(round(1e-4 * T * w.hidden))
    pos = g.choice(T * w.hidden, k, replace=False)
    mag = g.uniform(30.0, 80.0, size=k)
    sgn = g.integers(0, 2, size=k) * 2.0 - 1.0
    x.reshape(-1)[pos] = mag * sgn
    return _cast(x, w.dtype)


def c3_channels() -> Tuple[np.ndarray, np.ndarray]:
    w = WORKLOADS["C3"]
    g = _rng(2)
    ch = g.choice(w.hidden, 8, replace=False)
    sc = g.uniform(20.0, 80.0, size=8)
    return ch, sc


def make_c3(step: int, tokens: Optional[int] = None) -> np.ndarray:
    w = WORKLOADS["C3"]
    T = tokens or w.tokens
    ch, sc = c3_channels()
    g = _rng(2, step)
    x = g.standard_normal((T, w.hidden))
    x[:, ch] *= sc
    return _cast(x, w.dtype)


def make_c4(tokens: Optional[int] = None) -> np.ndarray:
    """Rows are drawn in blocks of 1024 tokens, each from its own stream, so that
    a row subset (a prefix of whole blocks) equals the same rows of the full tensor."""
    w = WORKLOADS["C4"]
    T = tokens or w.tokens
    g0 = _rng(3)
    ch = g0.choice(w.hidden, 12, replace=False)
    sc = g0.uniform(30.0, 150.0, size=12)
    out = np.empty((T, w.hidden), np.uint16)
    blk = 1024
    for i, r0 in enumerate(range(0, T, blk)):
        n = min(blk, T - r0)
        g = _rng(3, i)
        x = g.standard_t(5.0, size=(n, w.hidden))
        x *= g.lognormal(0.0, 0.7, size=(n, 1))
        x[:, ch] *= sc
        out[r0:r0 + n] = _cast(x, w.dtype)
    return out


def c5_channels() -> Tuple[np.ndarray, np.ndarray]:
    w = WORKLOADS["C5"]
    g = _rng(4)
    ch = g.choice(w.hidden, 16, replace=False)
    sc = g.uniform(30.0, 150.0, size=16)
    return ch, sc


def make_c5_seq(seq: int, tokens: int = C5_SEQ_TOKENS) -> np.ndarray:
    """One of the 32 sequences of the stress workload (4096 tokens x 8192)."""
    w = WORKLOADS["C5"]
    ch, sc = c5_channels()
    g = _rng(4, seq)
    x = g.standard_t(3.0, size=(tokens, w.hidden))
    x[:, ch] *= sc
    n = tokens * w.hidden
    k = int(round(0.01 * n))
    pos = g.choice(n, k, replace=False)
    mag = g.uniform(20.0, 200.0, size=k)
    sgn = g.integers(0, 2, size=k) * 2.0 - 1.0
    x.reshape(-1)[pos] = mag * sgn
    return _cast(x, w.dtype)


def make_c5(seqs: int = C5_SEQS, workers: int = 8) -> np.ndarray:
    """The stress tensor (seqs x 4096 rows).  Sequences are independent streams,
    drawn in a small process pool to keep generation to seconds."""
    w = WORKLOADS["C5"]
    out = np.empty((seqs * C5_SEQ_TOKENS, w.hidden), np.uint16)
    if workers <= 1 or seqs <= 1:
        for s in range(seqs):
            out[s * C5_SEQ_TOKENS:(s + 1) * C5_SEQ_TOKENS] = make_c5_seq(s)
        return out
    import multiprocessing as mp
    with mp.get_context("fork").Pool(min(workers, seqs)) as pool:
        for s, blk in enumerate(pool.imap(make_c5_seq, range(seqs))):
            out[s * C5_SEQ_TOKENS:(s + 1) * C5_SEQ_TOKENS] = blk
    return out


def make_kv_tensor(name: str, layer: int, which: int, rows: Optional[int] = None) -> np.ndarray:
    """One tensor of a KV-cache workload: which = 0 the keys, 1 the values of `layer`.
    Keys: N(0,1) x per-token LogNormal(0, 0.3), four channels (drawn per layer) x U(6, 14), as
    keys carry a few strong channels; values: N(0, 0.6^2) x per-token LogNormal(0, 0.3), and
    0.005 % of the elements set to +-U(8, 30)."""
    w = WORKLOADS[name]
    n = rows or KV_WORKLOADS[name][1]
    g = _rng(5, KV_WORKLOADS[name][0], layer, which)
    if which == 0:
        x = g.standard_normal((n, w.hidden))
        x *= g.lognormal(0.0, 0.3, size=(n, 1))
        ch = g.choice(w.hidden, 4, replace=False)
        x[:, ch] *= g.uniform(6.0, 14.0, size=4)
    else:
        x = 0.6 * g.standard_normal((n, w.hidden))
        x *= g.lognormal(0.0, 0.3, size=(n, 1))
        k = max(1, int(round(5e-5 * x.size)))
        idx = g.choice(x.size, k, replace=False)
        x.reshape(-1)[idx] = g.uniform(8.0, 30.0, size=k) * g.choice([-1.0, 1.0], size=k)
    return _cast(x, w.dtype)


def make_kv(name: str, layers: Optional[int] = None, rows: Optional[int] = None):
    """The tensors of a KV-cache workload in table order: K_1, V_1, K_2, V_2, ..."""
    L = layers or KV_WORKLOADS[name][0]
    return [make_kv_tensor(name, l, kv, rows) for l in range(L) for kv in (0, 1)]


def make(name: str, **kw) -> np.ndarray:
    if name == "C1":
        return make_c1()
    if name == "C2":
        return make_c2(**kw)
    if name == "C3":
        return make_c3(kw.pop("step", 0), **kw)
    if name == "C4":
        return make_c4(**kw)
    if name == "C5":
        return make_c5(**kw)
    raise KeyError(name)


def edge_rows(hidden: int, dtype: str, tau: float, seed: int = 7) -> np.ndarray:
    """A small tensor of degenerate rows for parity tests: all zero, all outliers,
    exact +-tau ties, one ulp below tau, NaN / +-Inf, negative zero, subnormals,
    a single non-zero element, constant rows, and rows of tiny magnitude."""
    g = np.random.Generator(np.random.PCG64(seed))
    rows = []
    z = np.zeros(hidden)
    rows.append(z.copy())                                            # all zero
    rows.append(np.full(hidden, 2.0 * tau))                          # all outliers
    r = g.standard_normal(hidden); r[::7] = tau; r[3::11] = -tau     # exact ties
    rows.append(r)
    r = g.standard_normal(hidden)                                    # just below tau
    below = np.nextafter(np.float16(tau), np.float16(0)) if dtype == "f16" else None
    if below is None:
        b = np.float32(tau).view(np.uint32) - np.uint32(0x10000)
        below = np.array([b], np.uint32).view(np.float32)[0]
    r[5::13] = float(below); r[6::13] = -float(below)
    rows.append(r)
    r = g.standard_normal(hidden); r[1] = np.nan; r[2] = np.inf; r[hidden - 1] = -np.inf
    rows.append(r)
    r = g.standard_normal(hidden); r[::2] = -0.0                     # negative zeros
    rows.append(r)
    tiny = 6e-8 if dtype == "f16" else 1e-39
    rows.append(g.integers(-3, 4, hidden) * tiny)                    # subnormal magnitudes
    r = z.copy(); r[hidden // 2] = -1.5                              # single non-zero
    rows.append(r)
    rows.append(np.full(hidden, 0.75))                               # constant row
    rows.append(g.standard_normal(hidden) * 1e-3)                    # small but normal
    rows.append(g.standard_normal(hidden) * 40.0)                    # mostly outliers
    r = g.standard_normal(hidden); r[0] = 5 * tau; r[-1] = -5 * tau  # outliers at both ends
    rows.append(r)
    x = np.stack(rows)
    with np.errstate(over="ignore", invalid="ignore"):
        bits = _cast(x, dtype)
    if dtype == "bf16":
        # the integer rounding trick above is for finite values: patch specials
        bits[4, 1] = 0x7FC1; bits[4, 2] = 0x7F80; bits[4, hidden - 1] = 0xFF80
    else:
        bits[4, 1] = 0x7E01
    return bits
