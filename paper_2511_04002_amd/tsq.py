"""Thin Python binding of the C-ABI library (include/tsq.h, tsq_measure.h, tsq_ranges.h): argument marshalling
only.  Every step of the method runs in the HIP kernels of libtsq.so; there is
no CPU fallback, and a missing library is an error.

PyTorch is used for device memory and streams, nothing else.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Iterable, Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
# TSQ_LIBRARY may name another build of the same library (e.g. one with different compile flags)
_LIB_PATH = os.environ.get("TSQ_LIBRARY") or os.path.join(_HERE, "libtsq.so")

TSQ_OK, TSQ_ERR_INVALID_ARG, TSQ_ERR_UNSUPPORTED, TSQ_ERR_CAPACITY = 0, 1, 2, 3
TSQ_ERR_HIP, TSQ_ERR_FORMAT, TSQ_ERR_INTERNAL, TSQ_ERR_NO_MEMORY = 4, 5, 6, 7
TSQ_F16, TSQ_BF16 = 0, 1
TSQ_BUDGET_LSB, TSQ_BUDGET_REL_RMS = 0, 1
TSQ_PIPE_AUTO, TSQ_PIPE_STAGED, TSQ_PIPE_FUSED = 0, 1, 2
TSQ_RETURN_LAST_PASSING, TSQ_RETURN_AS_PRINTED = 0, 1

EXPORTS = ("tsq_plan_create", "tsq_plan_destroy", "tsq_plan_layout", "tsq_plan_blob_bytes",
           "tsq_plan_workspace_bytes", "tsq_workspace_reset", "tsq_compress", "tsq_compress_blocking",
           "tsq_compress_static", "tsq_static_workspace_bytes",
           "tsq_decompress", "tsq_compress_batch", "tsq_decompress_batch",
           "tsq_code_histogram", "tsq_blob_info", "tsq_prefix_bytes", "tsq_status_string",
           # tsq_measure.h
           "tsq_compress_timed", "tsq_measure_copy", "tsq_measure_read",
           # tsq_ranges.h
           "tsq_check_payload_span", "tsq_check_csr_slice", "tsq_check_csr_slice_holds", "tsq_check_column",
           "tsq_check_stream_span", "tsq_check_stream_move", "tsq_check_frequency_slot", "tsq_check_workspace_shape",
           "tsq_check_quotients", "tsq_entropy_prefix_bytes",
           "tsq_entropy_blob_bytes", "tsq_entropy_workspace_bytes", "tsq_entropy_encode", "tsq_entropy_decode",
           "tsq_entropy_info", "tsq_link_outage_probability", "tsq_link_latency", "tsq_link_best_rate", "tsq_early_exit_decide",
           "tsq_early_exit_walk")
TSQ_EXIT_CONTINUE, TSQ_EXIT_COMPRESSED, TSQ_EXIT_WITHOUT_KV, TSQ_EXIT_FEWER_TOKENS, TSQ_EXIT_COMPLETED = 0, 1, 2, 3, 4


class tsq_config(C.Structure):
    _fields_ = [("tokens", C.c_uint32), ("hidden", C.c_uint32), ("dtype", C.c_int32),
                ("tau", C.c_float), ("bit_mask", C.c_uint32), ("budget", C.c_float),
                ("mode", C.c_int32), ("pipeline", C.c_int32), ("max_outliers", C.c_uint64),
                ("return_rule", C.c_int32), ("reserved", C.c_int32)]


class tsq_layout(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("blob_bytes", "workspace_bytes", "off_bits", "off_scale", "off_pay_off",
                 "off_row_ptr", "off_payload", "off_out_col", "off_out_val", "payload_capacity",
                 "outlier_capacity")]


class tsq_info(C.Structure):
    _fields_ = [("nnz", C.c_uint64), ("payload_bytes", C.c_uint64),
                ("compressed_bytes", C.c_uint64), ("width_hist", C.c_uint64 * 9),
                ("status", C.c_uint32), ("reserved", C.c_uint32)]


class tsq_entropy_layout(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("off_tables", "off_stream_off", "off_streams", "stream_capacity",
                                          "stream_bytes", "coded_bytes")]


class tsq_link(C.Structure):
    _fields_ = [("bandwidth_hz", C.c_double), ("snr", C.c_double), ("outage", C.c_double)]


class tsq_exit_input(C.Structure):
    _fields_ = [("link", tsq_link), ("rate", C.c_double), ("deadline", C.c_double), ("tokens", C.c_uint32),
                ("compute_latency", C.POINTER(C.c_double)), ("raw_bits", C.c_double),
                ("compressed_bits_with_kv", C.c_double), ("hidden_prefix_bits", C.POINTER(C.c_uint64))]


tsq_exit_latency_fn = C.CFUNCTYPE(C.c_double, C.c_uint32, C.c_uint32, C.c_void_p)
tsq_exit_bits_fn = C.CFUNCTYPE(C.c_double, C.c_uint32, C.c_uint32, C.c_int32, C.c_int32, C.c_uint32, C.c_void_p)


class tsq_exit_walk_input(C.Structure):
    _fields_ = [("link", tsq_link), ("rate", C.c_double), ("deadline", C.c_double), ("max_tokens", C.c_uint32),
                ("layers", C.c_uint32), ("compute_latency", tsq_exit_latency_fn), ("bits", tsq_exit_bits_fn),
                ("user", C.c_void_p)]


class tsq_exit_walk_result(C.Structure):
    _fields_ = [("action", C.c_int32), ("with_kv", C.c_int32), ("tokens", C.c_uint32), ("layer", C.c_uint32),
                ("sent_tokens", C.c_uint32), ("steps", C.c_uint32), ("latency", C.c_double)]


class tsq_exit_decision(C.Structure):
    _fields_ = [("action", C.c_int32), ("with_kv", C.c_int32), ("tokens", C.c_uint32), ("reserved", C.c_uint32),
                ("latency", C.c_double)]


class TsqError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, tsq_status_string(status), status))


_lib = None


def lib():
    """Loads libtsq.so.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libtsq.so is missing: run `python -m paper_2511_04002_amd.build` "
                               "(hipcc, gfx950); the library has no CPU fallback")
        L = C.CDLL(_LIB_PATH)
        vp, u = C.c_void_p, C.c_int
        L.tsq_plan_create.restype = u
        L.tsq_plan_create.argtypes = [C.POINTER(tsq_config), C.POINTER(vp)]
        L.tsq_plan_destroy.restype = None
        L.tsq_plan_destroy.argtypes = [vp]
        L.tsq_plan_layout.restype = u
        L.tsq_plan_layout.argtypes = [vp, C.POINTER(tsq_layout)]
        L.tsq_plan_blob_bytes.restype = C.c_size_t
        L.tsq_plan_blob_bytes.argtypes = [vp]
        L.tsq_plan_workspace_bytes.restype = C.c_size_t
        L.tsq_plan_workspace_bytes.argtypes = [vp]
        L.tsq_workspace_reset.restype = u
        L.tsq_workspace_reset.argtypes = [vp, vp, vp]
        L.tsq_compress.restype = u
        L.tsq_compress.argtypes = [vp, vp, vp, vp, vp]
        L.tsq_compress_static.restype = u
        L.tsq_compress_static.argtypes = [vp, vp, vp, vp]
        L.tsq_static_workspace_bytes.restype = C.c_size_t
        L.tsq_static_workspace_bytes.argtypes = []
        L.tsq_compress_timed.restype = u
        L.tsq_compress_timed.argtypes = [vp, vp, vp, vp, vp, C.POINTER(C.c_float)]
        L.tsq_compress_blocking.restype = u
        L.tsq_compress_blocking.argtypes = [vp, vp, vp, vp, vp, C.POINTER(tsq_info)]
        L.tsq_prefix_bytes.restype = u
        L.tsq_prefix_bytes.argtypes = [vp, vp, C.POINTER(C.c_uint32), C.c_uint32, C.POINTER(C.c_uint64), vp]
        L.tsq_entropy_prefix_bytes.restype = u
        L.tsq_entropy_prefix_bytes.argtypes = [vp, vp, vp, C.POINTER(C.c_uint32), C.c_uint32, C.POINTER(C.c_uint64), vp]
        L.tsq_measure_copy.restype = u
        L.tsq_measure_copy.argtypes = [vp, vp, C.c_size_t, vp]
        L.tsq_measure_read.restype = u
        L.tsq_measure_read.argtypes = [vp, C.c_size_t, vp, vp]
        u32, u64 = C.c_uint32, C.c_uint64
        for name, args in (("tsq_check_payload_span", [u32, u64, u32, u64]), ("tsq_check_csr_slice", [u64, u64, u64]),
                           ("tsq_check_csr_slice_holds", [u64, u64, u64, u32]), ("tsq_check_column", [u32, u32]),
                           ("tsq_check_stream_span", [u64, u64, u64, u32, u32]),
                           ("tsq_check_stream_move", [u32, u32, u32, u64, u64]),
                           ("tsq_check_workspace_shape", [u32, u32, u32, u32])):
            getattr(L, name).restype = C.c_int
            getattr(L, name).argtypes = args
        L.tsq_check_quotients.restype = None
        L.tsq_check_quotients.argtypes = [vp, vp, vp, u64]
        L.tsq_check_frequency_slot.restype = u32
        L.tsq_check_frequency_slot.argtypes = [u32]
        L.tsq_decompress.restype = u
        L.tsq_decompress.argtypes = [vp, vp, vp, vp]
        L.tsq_compress_batch.restype = u
        L.tsq_compress_batch.argtypes = [vp, vp, C.c_uint32, vp, vp, vp]
        L.tsq_decompress_batch.restype = u
        L.tsq_decompress_batch.argtypes = [vp, vp, vp, C.c_uint32, vp]
        L.tsq_code_histogram.restype = u
        L.tsq_code_histogram.argtypes = [vp, vp, vp, vp]
        L.tsq_blob_info.restype = u
        L.tsq_blob_info.argtypes = [vp, vp, C.POINTER(tsq_info), vp]
        L.tsq_entropy_blob_bytes.restype = C.c_size_t
        L.tsq_entropy_blob_bytes.argtypes = [vp]
        L.tsq_entropy_workspace_bytes.restype = C.c_size_t
        L.tsq_entropy_workspace_bytes.argtypes = [vp]
        L.tsq_entropy_encode.restype = u
        L.tsq_entropy_encode.argtypes = [vp, vp, vp, vp, vp]
        L.tsq_entropy_decode.restype = u
        L.tsq_entropy_decode.argtypes = [vp, vp, vp, vp]
        L.tsq_entropy_info.restype = u
        L.tsq_entropy_info.argtypes = [vp, vp, C.POINTER(tsq_entropy_layout), vp]
        L.tsq_link_outage_probability.restype = C.c_double
        L.tsq_link_outage_probability.argtypes = [C.POINTER(tsq_link), C.c_double]
        L.tsq_link_latency.restype = C.c_double
        L.tsq_link_latency.argtypes = [C.POINTER(tsq_link), C.c_double, C.c_double]
        L.tsq_link_best_rate.restype = C.c_double
        L.tsq_link_best_rate.argtypes = [C.POINTER(tsq_link), C.c_double, C.c_double, C.c_uint32]
        L.tsq_early_exit_decide.restype = u
        L.tsq_early_exit_decide.argtypes = [C.POINTER(tsq_exit_input), C.POINTER(tsq_exit_decision)]
        L.tsq_early_exit_walk.restype = u
        L.tsq_early_exit_walk.argtypes = [C.POINTER(tsq_exit_walk_input), C.POINTER(tsq_exit_walk_result)]
        L.tsq_status_string.restype = C.c_char_p
        L.tsq_status_string.argtypes = [u]
        _lib = L
    return _lib


# ------------------------------------------------------------------ the C entry points, same names

def tsq_status_string(status: int) -> str:
    return lib().tsq_status_string(int(status)).decode()


def tsq_plan_create(cfg: tsq_config) -> int:
    """-> opaque plan handle (int).  Raises TsqError on a rejected configuration."""
    h = C.c_void_p()
    st = lib().tsq_plan_create(C.byref(cfg), C.byref(h))
    if st != TSQ_OK:
        raise TsqError(st, "tsq_plan_create")
    return h.value


def tsq_plan_destroy(plan: int) -> None:
    lib().tsq_plan_destroy(plan)


def tsq_plan_layout(plan: int) -> tsq_layout:
    out = tsq_layout()
    st = lib().tsq_plan_layout(plan, C.byref(out))
    if st != TSQ_OK:
        raise TsqError(st, "tsq_plan_layout")
    return out


def tsq_plan_blob_bytes(plan: int) -> int:
    return int(lib().tsq_plan_blob_bytes(plan))


def tsq_plan_workspace_bytes(plan: int) -> int:
    return int(lib().tsq_plan_workspace_bytes(plan))


def tsq_workspace_reset(plan: int, d_ws: int, stream: int = 0) -> None:
    st = lib().tsq_workspace_reset(plan, d_ws, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_workspace_reset")


def tsq_compress(plan: int, d_in: int, d_blob: int, d_ws: int, stream: int = 0) -> None:
    st = lib().tsq_compress(plan, d_in, d_blob, d_ws, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_compress")


def tsq_compress_static(plan: int, d_in: int, d_blob: int, stream: int = 0) -> None:
    st = lib().tsq_compress_static(plan, d_in, d_blob, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_compress_static")


def tsq_static_workspace_bytes() -> int:
    return int(lib().tsq_static_workspace_bytes())


def tsq_compress_timed(plan: int, d_in: int, d_blob: int, d_ws: int, stream: int = 0):
    """-> per-kernel milliseconds [4] (synchronizes the stream)."""
    ms = (C.c_float * 4)()
    st = lib().tsq_compress_timed(plan, d_in, d_blob, d_ws, stream, ms)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_compress_timed")
    return list(ms)


def tsq_measure_copy(d_dst: int, d_src: int, nbytes: int, stream: int = 0) -> None:
    st = lib().tsq_measure_copy(d_dst, d_src, nbytes, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_measure_copy")


def tsq_measure_read(d_src: int, nbytes: int, d_sink: int, stream: int = 0) -> None:
    st = lib().tsq_measure_read(d_src, nbytes, d_sink, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_measure_read")


def tsq_compress_blocking(plan: int, d_in: int, d_blob: int, d_ws: int, stream: int = 0, check: bool = True) -> tsq_info:
    """Synchronizes.  -> tsq_info of the final blob (return_status = what the call returned)."""
    out = tsq_info()
    st = lib().tsq_compress_blocking(plan, d_in, d_blob, d_ws, stream, C.byref(out))
    if st != TSQ_OK and check:
        raise TsqError(st, "tsq_compress_blocking")
    out.return_status = st
    return out


def tsq_prefix_bytes(plan: int, d_blob: int, k=None, n: int = 0, stream: int = 0):
    """-> list of compressed sizes in bytes of the first k tokens, for the counts in `k` (or for
    k = 0 .. n-1 when k is None).  Synchronizes."""
    if k is not None:
        n = len(k)
        ks = (C.c_uint32 * n)(*[int(v) for v in k])
    else:
        ks = None
    out = (C.c_uint64 * n)()
    st = lib().tsq_prefix_bytes(plan, d_blob, ks, n, out, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_prefix_bytes")
    return list(out)


def tsq_entropy_prefix_bytes(plan: int, d_blob: int, d_eblob: int, k=None, n: int = 0, stream: int = 0):
    """-> list of sizes in bytes of what carries the first k tokens with the codes entropy-coded, for the counts
    in `k` (or for k = 0 .. n-1 when k is None).  Synchronizes."""
    if k is not None:
        n = len(k)
        ks = (C.c_uint32 * n)(*[int(v) for v in k])
    else:
        ks = None
    out = (C.c_uint64 * n)()
    st = lib().tsq_entropy_prefix_bytes(plan, d_blob, d_eblob, ks, n, out, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_entropy_prefix_bytes")
    return list(out)


def tsq_decompress(plan: int, d_blob: int, d_out: int, stream: int = 0) -> None:
    st = lib().tsq_decompress(plan, d_blob, d_out, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_decompress")


def tsq_compress_batch(plan: int, d_in_ptrs: int, rows_per_tensor: int, d_blob: int, d_ws: int,
                       stream: int = 0) -> None:
    st = lib().tsq_compress_batch(plan, d_in_ptrs, rows_per_tensor, d_blob, d_ws, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_compress_batch")


def tsq_decompress_batch(plan: int, d_blob: int, d_out_ptrs: int, rows_per_tensor: int, stream: int = 0) -> None:
    st = lib().tsq_decompress_batch(plan, d_blob, d_out_ptrs, rows_per_tensor, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_decompress_batch")


def tsq_code_histogram(plan: int, d_blob: int, d_hist: int, stream: int = 0) -> None:
    st = lib().tsq_code_histogram(plan, d_blob, d_hist, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_code_histogram")


def tsq_blob_info(plan: int, d_blob: int, stream: int = 0, check: bool = True) -> tsq_info:
    out = tsq_info()
    st = lib().tsq_blob_info(plan, d_blob, C.byref(out), stream)
    if st != TSQ_OK and check:
        raise TsqError(st, "tsq_blob_info")
    out.return_status = st
    return out


def tsq_entropy_blob_bytes(plan: int) -> int:
    return int(lib().tsq_entropy_blob_bytes(plan))


def tsq_entropy_workspace_bytes(plan: int) -> int:
    return int(lib().tsq_entropy_workspace_bytes(plan))


def tsq_entropy_encode(plan: int, d_blob: int, d_eblob: int, d_ews: int, stream: int = 0) -> None:
    st = lib().tsq_entropy_encode(plan, d_blob, d_eblob, d_ews, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_entropy_encode")


def tsq_entropy_decode(plan: int, d_eblob: int, d_blob: int, stream: int = 0) -> None:
    st = lib().tsq_entropy_decode(plan, d_eblob, d_blob, stream)
    if st != TSQ_OK:
        raise TsqError(st, "tsq_entropy_decode")


def tsq_entropy_info(plan: int, d_eblob: int, stream: int = 0, check: bool = True) -> tsq_entropy_layout:
    out = tsq_entropy_layout()
    st = lib().tsq_entropy_info(plan, d_eblob, C.byref(out), stream)
    if st != TSQ_OK and check:
        raise TsqError(st, "tsq_entropy_info")
    out.return_status = st
    return out


def tsq_link_outage_probability(link: tsq_link, rate: float) -> float:
    return float(lib().tsq_link_outage_probability(C.byref(link), rate))


def tsq_link_latency(link: tsq_link, bits: float, rate: float) -> float:
    return float(lib().tsq_link_latency(C.byref(link), bits, rate))


def tsq_link_best_rate(link: tsq_link, rate_lo: float, rate_hi: float, steps: int) -> float:
    return float(lib().tsq_link_best_rate(C.byref(link), rate_lo, rate_hi, steps))


def tsq_early_exit_decide(link: tsq_link, rate: float, deadline: float, compute_latency, raw_bits: float,
                          compressed_bits_with_kv: float, hidden_prefix_bits) -> tsq_exit_decision:
    """compute_latency, hidden_prefix_bits: sequences of w + 1 entries (k = 0 .. w tokens)."""
    w = len(compute_latency) - 1
    assert w >= 0 and len(hidden_prefix_bits) == w + 1
    lc = (C.c_double * (w + 1))(*[float(v) for v in compute_latency])
    hp = (C.c_uint64 * (w + 1))(*[int(v) for v in hidden_prefix_bits])
    inp = tsq_exit_input(link, rate, deadline, w, lc, raw_bits, compressed_bits_with_kv, hp)
    out = tsq_exit_decision()
    st = lib().tsq_early_exit_decide(C.byref(inp), C.byref(out))
    if st != TSQ_OK:
        raise TsqError(st, "tsq_early_exit_decide")
    return out


def tsq_early_exit_walk(link: tsq_link, rate: float, deadline: float, max_tokens: int, layers: int,
                        compute_latency, bits) -> tsq_exit_walk_result:
    """compute_latency(w, layer) -> seconds; bits(w, layer, with_kv, compressed, keep) -> bits."""
    failure = []

    def lat_cb(w, layer, _user):
        try:
            return float(compute_latency(w, layer))
        except BaseException as e:           # an exception cannot cross the C frames: end the walk, raise afterwards
            failure.append(e)
            return float("nan")

    def bits_cb(w, layer, with_kv, compressed, keep, _user):
        try:
            return float(bits(w, layer, with_kv, compressed, keep))
        except BaseException as e:
            failure.append(e)
            return float("nan")

    inp = tsq_exit_walk_input(link, rate, deadline, max_tokens, layers, tsq_exit_latency_fn(lat_cb),
                              tsq_exit_bits_fn(bits_cb), None)
    out = tsq_exit_walk_result()
    st = lib().tsq_early_exit_walk(C.byref(inp), C.byref(out))
    if failure:
        raise failure[0]
    if st != TSQ_OK:
        raise TsqError(st, "tsq_early_exit_walk")
    return out


# ------------------------------------------------------------------ convenience over torch tensors

def bit_mask(bit_set: Iterable[int]) -> int:
    m = 0
    for b in bit_set:
        m |= 1 << int(b)
    return m


_DTYPES = {"f16": TSQ_F16, "bf16": TSQ_BF16}
_MODES = {"lsb": TSQ_BUDGET_LSB, "rel_rms": TSQ_BUDGET_REL_RMS}
_PIPES = {"auto": TSQ_PIPE_AUTO, "staged": TSQ_PIPE_STAGED, "fused": TSQ_PIPE_FUSED}
_RULES = {"last_passing": TSQ_RETURN_LAST_PASSING, "as_printed": TSQ_RETURN_AS_PRINTED}


class Plan:
    """Owns one tsq_plan plus helpers that allocate torch buffers and pass their pointers."""

    def __init__(self, tokens: int, hidden: int, dtype: str, tau: float, bit_set: Iterable[int],
                 budget: float, mode: str = "rel_rms", pipeline: str = "auto", max_outliers: int = 0,
                 return_rule: str = "last_passing"):
        self.cfg = tsq_config(tokens, hidden, _DTYPES[dtype], tau, bit_mask(bit_set), budget,
                              _MODES[mode], _PIPES[pipeline], max_outliers, _RULES[return_rule], 0)
        self.handle = tsq_plan_create(self.cfg)
        self.layout = tsq_plan_layout(self.handle)
        self.tokens, self.hidden, self.dtype = tokens, hidden, dtype

    def __del__(self):
        h = getattr(self, "handle", None)
        # (at interpreter shutdown the module's globals may be gone before the last plan is)
        if h and tsq_plan_destroy is not None:
            tsq_plan_destroy(h)
            self.handle = None

    @staticmethod
    def _stream() -> int:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)

    def new_blob(self):
        import torch
        return torch.empty(int(self.layout.blob_bytes), dtype=torch.uint8, device="cuda")

    def new_workspace(self):
        import torch
        ws = torch.empty(int(self.layout.workspace_bytes), dtype=torch.uint8, device="cuda")
        tsq_workspace_reset(self.handle, ws.data_ptr(), self._stream())
        return ws

    def new_output(self):
        import torch
        return torch.empty((self.tokens, self.hidden), dtype=torch.int16, device="cuda")

    def compress(self, x, blob=None, ws=None):
        """x: contiguous CUDA tensor [tokens, hidden] of a 16-bit dtype (raw bits are what counts)."""
        assert x.is_cuda and x.is_contiguous() and x.element_size() == 2
        assert x.numel() == self.tokens * self.hidden
        blob = self.new_blob() if blob is None else blob
        ws = self.new_workspace() if ws is None else ws
        tsq_compress(self.handle, x.data_ptr(), blob.data_ptr(), ws.data_ptr(), self._stream())
        return blob

    def decompress(self, blob, out=None):
        out = self.new_output() if out is None else out
        assert out.is_cuda and out.is_contiguous() and out.element_size() == 2
        tsq_decompress(self.handle, blob.data_ptr(), out.data_ptr(), self._stream())
        return out

    @staticmethod
    def pointer_table(tensors):
        """Device array of the tensors' data pointers (what the *_batch calls take)."""
        import torch
        for x in tensors:
            assert x.is_cuda and x.is_contiguous() and x.element_size() == 2
        return torch.tensor([x.data_ptr() for x in tensors], dtype=torch.int64, device="cuda")

    def compress_batch(self, tensors, blob=None, ws=None, table=None):
        """tensors: equally shaped contiguous CUDA tensors [rows, hidden] whose rows add up to the
        plan's tokens.  `table` (from pointer_table) may be passed to reuse it across calls; it must
        stay alive until the call has run."""
        rows = tensors[0].numel() // self.hidden
        assert all(x.numel() == rows * self.hidden for x in tensors) and rows * len(tensors) == self.tokens
        table = self.pointer_table(tensors) if table is None else table
        blob = self.new_blob() if blob is None else blob
        ws = self.new_workspace() if ws is None else ws
        tsq_compress_batch(self.handle, table.data_ptr(), rows, blob.data_ptr(), ws.data_ptr(), self._stream())
        return blob, table

    def decompress_batch(self, blob, outs, table=None):
        rows = outs[0].numel() // self.hidden
        assert all(x.numel() == rows * self.hidden for x in outs) and rows * len(outs) == self.tokens
        table = self.pointer_table(outs) if table is None else table
        tsq_decompress_batch(self.handle, blob.data_ptr(), table.data_ptr(), rows, self._stream())
        return table

    def code_histogram(self, blob, hist=None):
        """-> CUDA int32 tensor [tokens, 256]: how often each code occurs in each token."""
        import torch
        if hist is None:
            hist = torch.empty((self.tokens, 256), dtype=torch.int32, device="cuda")
        assert hist.is_cuda and hist.is_contiguous() and hist.numel() == self.tokens * 256
        tsq_code_histogram(self.handle, blob.data_ptr(), hist.data_ptr(), self._stream())
        return hist

    def new_entropy_blob(self):
        import torch
        return torch.empty(tsq_entropy_blob_bytes(self.handle), dtype=torch.uint8, device="cuda")

    def new_entropy_workspace(self):
        import torch
        return torch.empty(tsq_entropy_workspace_bytes(self.handle), dtype=torch.uint8, device="cuda")

    def entropy_encode(self, blob, eblob=None, ews=None):
        eblob = self.new_entropy_blob() if eblob is None else eblob
        ews = self.new_entropy_workspace() if ews is None else ews
        tsq_entropy_encode(self.handle, blob.data_ptr(), eblob.data_ptr(), ews.data_ptr(), self._stream())
        return eblob

    def entropy_decode(self, eblob, blob):
        tsq_entropy_decode(self.handle, eblob.data_ptr(), blob.data_ptr(), self._stream())
        return blob

    def entropy_sections(self, eblob):
        """Host copies of the eblob's sections, the streams cut to their actual length."""
        import numpy as np
        import torch
        info = tsq_entropy_info(self.handle, eblob.data_ptr(), self._stream())
        torch.cuda.synchronize()
        raw = eblob.cpu().numpy()
        T = self.tokens
        return {"tables": raw[info.off_tables: info.off_tables + 7 * 512].view(np.uint16).reshape(7, 256).copy(),
                "stream_off": raw[info.off_stream_off: info.off_stream_off + 8 * (T + 1)].view(np.uint64).copy(),
                "streams": raw[info.off_streams: info.off_streams + info.stream_bytes].copy(),
                "info": info}

    def info(self, blob, check: bool = True) -> tsq_info:
        return tsq_blob_info(self.handle, blob.data_ptr(), self._stream(), check)

    def prefix_bytes(self, blob, k=None):
        """Compressed size of the first k tokens for every k in `k` (default: k = 0 .. tokens)."""
        return tsq_prefix_bytes(self.handle, blob.data_ptr(), k, self.tokens + 1 if k is None else 0, self._stream())

    def entropy_prefix_bytes(self, blob, eblob, k=None):
        """Size of what carries the first k tokens with the codes entropy-coded, for every k in `k` (default: k = 0 .. tokens)."""
        return tsq_entropy_prefix_bytes(self.handle, blob.data_ptr(), eblob.data_ptr(), k,
                                        self.tokens + 1 if k is None else 0, self._stream())

    def sections(self, blob) -> Dict[str, "object"]:
        """Host copies (numpy) of the blob's sections, cut to their actual lengths."""
        import numpy as np
        import torch
        torch.cuda.synchronize()
        L, T = self.layout, self.tokens
        raw = blob.cpu().numpy()

        def view(off, nbytes, dt):
            return raw[int(off): int(off) + int(nbytes)].view(dt).copy()

        pay_off = view(L.off_pay_off, 8 * (T + 1), np.uint64)
        row_ptr = view(L.off_row_ptr, 8 * (T + 1), np.uint64)
        nnz = min(int(row_ptr[-1]), int(L.outlier_capacity))
        return {
            "header": view(0, 128, np.uint8),
            "bits": view(L.off_bits, T, np.uint8),
            "scale": view(L.off_scale, 4 * T, np.float32),
            "pay_off": pay_off,
            "row_ptr": row_ptr,
            "payload": view(L.off_payload, min(int(pay_off[-1]), int(L.payload_capacity)), np.uint8),
            "out_col": view(L.off_out_col, 2 * nnz, np.uint16),
            "out_val": view(L.off_out_val, 2 * nnz, np.uint16),
        }
