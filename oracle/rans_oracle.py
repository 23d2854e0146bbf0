"""Entropy coding of the packed codes: range-variant asymmetric numeral systems (rANS), the coder
the paper names for the symbols TAB-Q produces (Sec. II-C.2, last paragraph).

TEST INFRASTRUCTURE ONLY (see tsq_oracle.py).  Plain Python integers, one symbol at a time.

The paper delegates the coder to a third-party package and fixes none of its parameters; the
format below is this build's own, stated in full so that the GPU coder can be checked bit for bit:

  alphabet      the b-bit codes of a token, b = the token's width; one frequency table per
                width class (all tokens of that width share it), built from the pooled counts
  table         counts -> 12-bit frequencies (normalize): f_c = max(1, floor(n_c * 4096 / N)) for
                n_c > 0; while the sum exceeds 4096 take 1 from the largest f (lowest code on
                ties); a remaining deficit goes to the code with the largest count (lowest code
                on ties)
  coder         rANS as published (Duda 2013): state x in [2^16, 2^32), 16-bit renormalisation,
                  encode s:  if x >= f_s << 20: emit x & 0xFFFF, x >>= 16
                             x = ((x // f_s) << 12) + (x % f_s) + c_s
                  decode:    slot = x & 4095, s = symbol whose [c_s, c_s + f_s) holds slot,
                             x = f_s * (x >> 12) + slot - c_s;  if x < 2^16: x = x << 16 | next word
  interleaving  64 coders per token (one per lane of a wave).  The token's codes are cut into
                runs of 32; coder l owns the runs l, l + 64, l + 128, ...  Step i (i = 0 .. 32 *
                ceil(runs / 64) - 1) handles, for every coder, element (i mod 32) of its run
                number (i div 32), if that element exists.  The encoder walks the steps
                backwards, the decoder forwards; the words of one step are stored in coder order
  token stream  the final states of the coders that own a run (min(64, runs) of them; u32,
                little-endian, coder order), then the words (u16) in the order the decoder reads
                them, zero padded to a multiple of 4 bytes
"""
from __future__ import annotations

import numpy as np

PROB_BITS = 12
M = 1 << PROB_BITS
LOW = 1 << 16
CODERS = 64
RUN = 32


def normalize(counts) -> np.ndarray:
    """Counts of one width class -> frequencies that sum to 4096 (all zero if there is nothing)."""
    n = [int(v) for v in counts]
    N = sum(n)
    f = [0] * len(n)
    if N == 0:
        return np.array(f, np.uint16)
    for c, v in enumerate(n):
        if v > 0:
            f[c] = max(1, v * M // N)
    S = sum(f)
    while S > M:
        c = max(range(len(f)), key=lambda k: (f[k], -k))
        f[c] -= 1
        S -= 1
    if S < M:
        c = max(range(len(n)), key=lambda k: (n[k], -k))
        f[c] += M - S
    return np.array(f, np.uint16)


def cumulative(freq) -> list:
    c, out = 0, []
    for v in freq:
        out.append(c)
        c += int(v)
    return out


def _element(i: int, l: int) -> int:
    return (l + CODERS * (i // RUN)) * RUN + (i % RUN)


def coders_in_use(H: int) -> int:
    return min(CODERS, (H + RUN - 1) // RUN)


def _steps(H: int) -> int:
    runs = (H + RUN - 1) // RUN
    return RUN * ((runs + CODERS - 1) // CODERS)


def encode_token(codes, freq) -> bytes:
    """codes: the H codes of a token; freq: its class's table -> the token's stream."""
    H = len(codes)
    cum = cumulative(freq)
    x = [LOW] * CODERS
    chunks = []
    for i in reversed(range(_steps(H))):
        words = []
        for l in range(CODERS):
            e = _element(i, l)
            if e >= H:
                continue
            s = int(codes[e])
            f, c = int(freq[s]), cum[s]
            assert f > 0, "a code that the table does not know"
            if x[l] >= (f << 20):
                words.append(x[l] & 0xFFFF)
                x[l] >>= 16
            x[l] = ((x[l] // f) << PROB_BITS) + (x[l] % f) + c
        chunks.append(words)
    words = [w for ch in reversed(chunks) for w in ch]
    assert all(v == LOW for v in x[coders_in_use(H):])
    out = np.array(x[:coders_in_use(H)], "<u4").tobytes() + np.array(words, "<u2").tobytes()
    return out + b"\0" * (-len(out) % 4)


def decode_token(stream: bytes, H: int, freq) -> np.ndarray:
    cum = cumulative(freq)
    sym = np.zeros(M, np.int64)
    for s, (c, f) in enumerate(zip(cum, freq)):
        sym[c:c + int(f)] = s
    k = coders_in_use(H)
    x = [int(v) for v in np.frombuffer(stream[:4 * k], "<u4")] + [LOW] * (CODERS - k)
    words = np.frombuffer(stream[4 * k:len(stream) - (len(stream) - 4 * k) % 2], "<u2")
    pos = 0
    codes = np.zeros(H, np.uint32)
    for i in range(_steps(H)):
        live = [l for l in range(CODERS) if _element(i, l) < H]
        for l in live:
            slot = x[l] & (M - 1)
            s = int(sym[slot])
            codes[_element(i, l)] = s
            x[l] = int(freq[s]) * (x[l] >> PROB_BITS) + slot - cum[s]
        for l in live:
            if x[l] < LOW:
                x[l] = (x[l] << 16) | int(words[pos])
                pos += 1
    assert all(v == LOW for v in x), "the decoder must end where the encoder began"
    return codes


# ---------------------------------------------------------------- a whole compressed tensor

def class_tables(hist: np.ndarray, bits: np.ndarray) -> np.ndarray:
    """u16 [7, 256]: row b - 2 is the table of width b (zero if no token has that width)."""
    out = np.zeros((7, 256), np.uint16)
    for b in range(2, 9):
        rows = hist[bits == b]
        if rows.shape[0]:
            out[b - 2] = normalize(rows.sum(axis=0, dtype=np.uint64))
    return out


def encode(c, hist: np.ndarray):
    """c: tsq_oracle.Compressed, hist: its code histogram -> (tables u16[7,256], offsets u64[T+1], streams bytes)."""
    from . import entropy_oracle as E
    tables = class_tables(hist, c.bits)
    off = np.zeros(c.tokens + 1, np.uint64)
    parts = []
    for t in range(c.tokens):
        s = encode_token(E.token_codes(c, t), tables[int(c.bits[t]) - 2])
        parts.append(s)
        off[t + 1] = off[t] + np.uint64(len(s))
    return tables, off, b"".join(parts)


def decode_codes(tables, off, streams: bytes, bits, hidden: int, t: int) -> np.ndarray:
    return decode_token(streams[int(off[t]):int(off[t + 1])], hidden, tables[int(bits[t]) - 2])


# ---------------------------------------------------------------- the same coder compiled (rans_oracle.c)

_C_SRC = __import__("os").path.join(__import__("os").path.dirname(__import__("os").path.abspath(__file__)), "rans_oracle.c")
_C_LIB = _C_SRC[:-2] + "_c.so"
_clib = None


def build_c(force: bool = False) -> str:
    """Compile rans_oracle.c with gcc."""
    import os
    import subprocess
    if force or not os.path.exists(_C_LIB) or os.path.getmtime(_C_LIB) < os.path.getmtime(_C_SRC):
        tmp = _C_LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _C_SRC],
                       check=True)
        os.replace(tmp, _C_LIB)
    return _C_LIB


def _c():
    global _clib
    if _clib is None:
        import ctypes as C
        L = C.CDLL(build_c())
        L.ranso_encode_token.restype = C.c_uint32
        L.ranso_encode_token.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p]
        L.ranso_encode.restype = C.c_uint64
        L.ranso_encode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p,
                                   C.c_uint64]
        _clib = L
    return _clib


def encode_token_c(codes, freq) -> bytes:
    """encode_token through the compiled coder."""
    codes = np.ascontiguousarray(codes, np.uint8)
    f = np.zeros(256, np.uint16)
    f[: len(freq)] = freq
    out = np.zeros(4 * CODERS + 2 * len(codes) + 4, np.uint8)
    n = _c().ranso_encode_token(codes.ctypes.data, len(codes), f.ctypes.data, out.ctypes.data)
    assert n > 0, "a code that the table does not know"
    return out[:n].tobytes()


def encode_codes_c(codes, bits, tables):
    """codes: u8 [T, H]; bits: u8 [T]; tables: u16 [7, 256] -> (stream offsets u64 [T+1], streams u8)."""
    codes = np.ascontiguousarray(codes, np.uint8)
    bits = np.ascontiguousarray(bits, np.uint8)
    tables = np.ascontiguousarray(tables, np.uint16)
    T, H = codes.shape
    cap = T * (4 * CODERS + 2 * H + 4)
    off = np.zeros(T + 1, np.uint64)
    streams = np.zeros(cap, np.uint8)
    n = _c().ranso_encode(codes.ctypes.data, bits.ctypes.data, tables.ctypes.data, T, H, off.ctypes.data,
                          streams.ctypes.data, cap)
    assert n > 0 or T == 0
    return off, streams[: int(n)].copy()
