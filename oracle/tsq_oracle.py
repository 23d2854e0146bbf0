"""ctypes front end of the CPU oracle (oracle/tsq_oracle.c).

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's
cpu_baseline leg may import this module; the product package must not.

The module marshals numpy arrays into the C functions and nothing else: all
arithmetic of the method (Eq. (ts), Eq. (Proposed), Algorithm 1, Eq. (dequnt))
lives in the C file, each function there citing the passage it follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tsq_oracle.c")
_HDR = os.path.join(_HERE, "tsq_oracle.h")
_LIB = os.path.join(_HERE, "libtsq_oracle.so")

F16, BF16 = 0, 1
BUDGET_LSB, BUDGET_REL_RMS = 0, 1
RETURN_LAST_PASSING, RETURN_AS_PRINTED = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (one IEEE operation per fp32 expression)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


class _Config(C.Structure):
    _fields_ = [("tokens", C.c_uint32), ("hidden", C.c_uint32), ("dtype", C.c_int32),
                ("tau", C.c_float), ("bit_mask", C.c_uint32), ("budget", C.c_float),
                ("mode", C.c_int32), ("rule", C.c_int32)]


class _TokenInfo(C.Structure):
    _fields_ = [("cnt", C.c_uint32), ("amax", C.c_float), ("bits", C.c_uint32),
                ("scale", C.c_float), ("nbytes", C.c_uint32), ("n_eval", C.c_uint32),
                ("ss0", C.c_uint64), ("sad", C.c_uint64 * 8)]


TOKEN_INFO_DTYPE = np.dtype([("cnt", "<u4"), ("amax", "<f4"), ("bits", "<u4"), ("scale", "<f4"),
                             ("nbytes", "<u4"), ("n_eval", "<u4"), ("ss0", "<u8"),
                             ("sad", "<u8", (8,))])
assert TOKEN_INFO_DTYPE.itemsize == C.sizeof(_TokenInfo)

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp = C.c_void_p
        L.tsqo_widen.restype = C.c_float
        L.tsqo_widen.argtypes = [C.c_uint16, C.c_int32]
        L.tsqo_narrow.restype = C.c_uint16
        L.tsqo_narrow.argtypes = [C.c_float, C.c_int32]
        L.tsqo_ts_row.restype = None
        L.tsqo_ts_row.argtypes = [vp, C.c_uint32, C.c_int32, C.c_float, vp, vp, vp, vp]
        L.tsqo_aiq_row.restype = None
        L.tsqo_aiq_row.argtypes = [vp, C.c_uint32, C.c_float, C.c_int, vp, vp, vp]
        L.tsqo_select_row_rule.restype = None
        L.tsqo_select_row_rule.argtypes = [vp, C.c_uint32, C.c_float, C.c_uint32, C.c_float, C.c_int32, C.c_int32, vp]
        L.tsqo_select_row.restype = None
        L.tsqo_select_row.argtypes = [vp, C.c_uint32, C.c_float, C.c_uint32, C.c_float,
                                      C.c_int32, vp]
        L.tsqo_pack_row.restype = None
        L.tsqo_pack_row.argtypes = [vp, vp, C.c_uint32, C.c_int, vp]
        L.tsqo_unpack_row.restype = None
        L.tsqo_unpack_row.argtypes = [vp, C.c_uint32, C.c_int, vp, vp]
        L.tsqo_compress.restype = C.c_int
        L.tsqo_compress.argtypes = [C.POINTER(_Config), vp, vp, vp, vp, vp, vp, C.c_uint64,
                                    vp, vp, C.c_uint64, vp, C.c_int]
        L.tsqo_decompress.restype = C.c_int
        L.tsqo_decompress.argtypes = [C.POINTER(_Config), vp, vp, vp, vp, vp, vp, vp, vp, C.c_int]
        L.tsqo_max_threads.restype = C.c_int
        L.tsqo_max_threads.argtypes = []
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def bit_mask(bit_set) -> int:
    m = 0
    for b in bit_set:
        m |= 1 << int(b)
    return m


def max_threads() -> int:
    return int(lib().tsqo_max_threads())


# ---------------------------------------------------------------- scalars / rows

def widen(raw: np.ndarray, dtype: int) -> np.ndarray:
    raw = np.ascontiguousarray(raw, dtype=np.uint16)
    L = lib()
    return np.array([L.tsqo_widen(int(v), dtype) for v in raw.ravel()],
                    dtype=np.float32).reshape(raw.shape)


def narrow(v: np.ndarray, dtype: int) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float32)
    L = lib()
    return np.array([L.tsqo_narrow(float(x), dtype) for x in v.ravel()],
                    dtype=np.uint16).reshape(v.shape)


def ts_row(x: np.ndarray, dtype: int, tau: float):
    """Eq. (ts) on one token -> (out mask u8[H], a f32[H], cnt, amax)."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    H = x.size
    out = np.zeros(H, np.uint8)
    a = np.zeros(H, np.float32)
    cnt = np.zeros(1, np.uint32)
    amax = np.zeros(1, np.float32)
    lib().tsqo_ts_row(_p(x), H, dtype, np.float32(tau), _p(out), _p(a), _p(cnt), _p(amax))
    return out, a, int(cnt[0]), np.float32(amax[0])


def aiq_row(a: np.ndarray, amax, b: int):
    """Eq. (Proposed) on magnitudes -> (m i32[H], r, s)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    m = np.zeros(a.size, np.int32)
    r = np.zeros(1, np.float32)
    s = np.zeros(1, np.float32)
    lib().tsqo_aiq_row(_p(a), a.size, np.float32(amax), int(b), _p(m), _p(r), _p(s))
    return m, np.float32(r[0]), np.float32(s[0])


def select_row(a: np.ndarray, amax, bit_set, budget: float, mode: int, rule: int = 0):
    """Algorithm 1 on one token -> numpy record (TOKEN_INFO_DTYPE).  rule: RETURN_LAST_PASSING (the
    default reading) or RETURN_AS_PRINTED (the width that failed the test is returned)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    info = np.zeros(1, TOKEN_INFO_DTYPE)
    lib().tsqo_select_row_rule(_p(a), a.size, np.float32(amax), bit_mask(bit_set),
                               np.float32(budget), int(mode), int(rule), _p(info))
    return info[0]


def row_bytes(H: int, b: int) -> int:
    return 4 * ((H * b + 31) // 32)


def pack_row(m: np.ndarray, neg: np.ndarray, b: int) -> np.ndarray:
    m = np.ascontiguousarray(m, dtype=np.int32)
    neg = np.ascontiguousarray(neg, dtype=np.uint8)
    dst = np.zeros(row_bytes(m.size, b), np.uint8)
    lib().tsqo_pack_row(_p(m), _p(neg), m.size, int(b), _p(dst))
    return dst


def unpack_row(src: np.ndarray, H: int, b: int):
    src = np.ascontiguousarray(src, dtype=np.uint8)
    assert src.size >= row_bytes(H, b)
    m = np.zeros(H, np.int32)
    neg = np.zeros(H, np.uint8)
    lib().tsqo_unpack_row(_p(src), H, int(b), _p(m), _p(neg))
    return m, neg


# ---------------------------------------------------------------- whole tensor

@dataclass
class Compressed:
    tokens: int
    hidden: int
    dtype: int
    bits: np.ndarray      # u8  [T]
    scale: np.ndarray     # f32 [T]
    pay_off: np.ndarray   # u64 [T+1]
    row_ptr: np.ndarray   # u64 [T+1]
    payload: np.ndarray   # u8  [pay_off[T]]
    out_col: np.ndarray   # u16 [nnz]
    out_val: np.ndarray   # u16 [nnz]
    info: np.ndarray      # TOKEN_INFO_DTYPE [T]

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])

    @property
    def payload_bytes(self) -> int:
        return int(self.pay_off[-1])


def compress(x: np.ndarray, dtype: int, tau: float, bit_set, budget: float, mode: int,
             nthreads: int = 1, rule: int = 0) -> Compressed:
    """TS + TAB-Q of a [T, H] array of raw 16-bit values."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    T, H = x.shape
    cfg = _Config(T, H, dtype, tau, bit_mask(bit_set), budget, mode, rule)
    bmax = max(bit_set)
    bits = np.zeros(T, np.uint8)
    scale = np.zeros(T, np.float32)
    pay_off = np.zeros(T + 1, np.uint64)
    row_ptr = np.zeros(T + 1, np.uint64)
    info = np.zeros(T, TOKEN_INFO_DTYPE)
    # generous first guess for the side stream; retried at the exact size if too small
    pay_cap = T * row_bytes(H, bmax)
    out_cap = max(1024, (T * H) // 16)
    while True:
        payload = np.zeros(pay_cap, np.uint8)
        out_col = np.zeros(out_cap, np.uint16)
        out_val = np.zeros(out_cap, np.uint16)
        rc = lib().tsqo_compress(C.byref(cfg), _p(x), _p(bits), _p(scale), _p(pay_off),
                                 _p(row_ptr), _p(payload), pay_cap, _p(out_col), _p(out_val),
                                 out_cap, _p(info), int(nthreads))
        if rc == 0:
            break
        if rc == 3:
            out_cap = int(row_ptr[-1])
            continue
        raise ValueError("tsqo_compress rejected the configuration (rc=%d)" % rc)
    nnz = int(row_ptr[-1])
    return Compressed(T, H, dtype, bits, scale, pay_off, row_ptr,
                      payload[: int(pay_off[-1])].copy(), out_col[:nnz].copy(),
                      out_val[:nnz].copy(), info)


def decompress(c: Compressed, nthreads: int = 1) -> np.ndarray:
    """Eq. (dequnt): -> [T, H] raw 16-bit values."""
    cfg = _Config(c.tokens, c.hidden, c.dtype, 1.0, 0, 0.0, 0, 0)
    out = np.zeros((c.tokens, c.hidden), np.uint16)
    payload = np.ascontiguousarray(c.payload)
    if payload.size == 0:
        payload = np.zeros(4, np.uint8)
    col = c.out_col if c.out_col.size else np.zeros(1, np.uint16)
    val = c.out_val if c.out_val.size else np.zeros(1, np.uint16)
    rc = lib().tsqo_decompress(C.byref(cfg), _p(c.bits), _p(c.scale), _p(c.pay_off),
                               _p(c.row_ptr), _p(payload), _p(col), _p(val), _p(out),
                               int(nthreads))
    if rc != 0:
        raise ValueError("tsqo_decompress failed (rc=%d)" % rc)
    return out


def compressed_bytes(c: Compressed) -> int:
    """Size of the compressed representation: 128-byte header, one width byte and
    one fp32 scale per token, two (T+1)-entry u64 offset arrays, the packed
    payload, and 4 bytes (u16 column + 16-bit value) per outlier."""
    T = c.tokens
    return 128 + 5 * T + 16 * (T + 1) + c.payload_bytes + 4 * c.nnz
