"""Host-only checks of the C-ABI library: it loads, exports every function that
the headers under include/ declare, and its plan validation and layout behave as the header
says.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

from paper_2511_04002_amd import build as tsq_build
from paper_2511_04002_amd import tsq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    tsq_build.build()
    return tsq.lib()


def declared_functions():
    names = set()
    for header in ("tsq.h", "tsq_measure.h", "tsq_ranges.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"typedef[^;{]*\(\s*\*\s*tsq_[a-z_]+\s*\)[^;]*;", "", text)      # function-pointer types
        names |= set(re.findall(r"\b(tsq_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert set(names) == set(tsq.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def cfg(**kw):
    base = dict(tokens=128, hidden=768, dtype=tsq.TSQ_F16, tau=6.0, bit_mask=tsq.bit_mask((2, 4, 8)),
                budget=0.05, mode=tsq.TSQ_BUDGET_REL_RMS, pipeline=tsq.TSQ_PIPE_AUTO, max_outliers=0)
    base.update(kw)
    return tsq.tsq_config(**base)


@pytest.mark.parametrize("kw,status", [
    (dict(tokens=0), tsq.TSQ_ERR_INVALID_ARG),
    (dict(hidden=0), tsq.TSQ_ERR_INVALID_ARG),
    (dict(dtype=7), tsq.TSQ_ERR_INVALID_ARG),
    (dict(tau=0.0), tsq.TSQ_ERR_INVALID_ARG),
    (dict(tau=-1.0), tsq.TSQ_ERR_INVALID_ARG),
    (dict(tau=float("inf")), tsq.TSQ_ERR_INVALID_ARG),
    (dict(tau=float("nan")), tsq.TSQ_ERR_INVALID_ARG),
    (dict(bit_mask=0), tsq.TSQ_ERR_INVALID_ARG),
    (dict(bit_mask=1 << 1), tsq.TSQ_ERR_INVALID_ARG),
    (dict(bit_mask=(1 << 9) | (1 << 4)), tsq.TSQ_ERR_INVALID_ARG),
    (dict(budget=-0.1), tsq.TSQ_ERR_INVALID_ARG),
    (dict(budget=float("nan")), tsq.TSQ_ERR_INVALID_ARG),
    (dict(mode=5), tsq.TSQ_ERR_INVALID_ARG),
    (dict(pipeline=9), tsq.TSQ_ERR_INVALID_ARG),
    (dict(return_rule=2), tsq.TSQ_ERR_INVALID_ARG),
    (dict(return_rule=-1), tsq.TSQ_ERR_INVALID_ARG),
    (dict(reserved=1), tsq.TSQ_ERR_INVALID_ARG),
    (dict(tokens=1 << 20, hidden=4096), tsq.TSQ_ERR_INVALID_ARG),       # tokens*hidden >= 2^32
    (dict(hidden=772), tsq.TSQ_ERR_UNSUPPORTED),                        # not a multiple of 8
    (dict(hidden=65536), tsq.TSQ_ERR_UNSUPPORTED),
])
def test_plan_create_rejects(L, kw, status):
    with pytest.raises(tsq.TsqError) as e:
        tsq.tsq_plan_create(cfg(**kw))
    assert e.value.status == status


def test_null_arguments(L):
    h = C.c_void_p()
    assert L.tsq_plan_create(None, C.byref(h)) == tsq.TSQ_ERR_INVALID_ARG
    c = cfg()
    assert L.tsq_plan_create(C.byref(c), None) == tsq.TSQ_ERR_INVALID_ARG
    plan = tsq.tsq_plan_create(c)
    try:
        assert L.tsq_compress(plan, None, None, None, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_decompress(plan, None, None, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_blob_info(plan, None, None, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_workspace_reset(plan, None, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_compress_batch(plan, None, 1, None, None, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_decompress_batch(plan, None, None, 1, None) == tsq.TSQ_ERR_INVALID_ARG
        # rows per tensor must be at least 1 and divide the plan's tokens; the table is 8-byte aligned
        T = c.tokens
        assert L.tsq_compress_batch(plan, 0x1000, 0, 0x2000, 0x3000, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_compress_batch(plan, 0x1000, T + 1, 0x2000, 0x3000, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_compress_batch(plan, 0x1004, T, 0x2000, 0x3000, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_decompress_batch(plan, 0x2000, 0x1000, 0, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_decompress_batch(plan, 0x2000, 0x1000, T + 1, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_decompress_batch(plan, 0x2000, 0x1004, T, None) == tsq.TSQ_ERR_INVALID_ARG
        # misaligned device pointers are refused before any launch
        assert L.tsq_compress(plan, 0x1008, 0x2000, 0x3000, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_compress(plan, 0x1000, 0x2010, 0x3000, None) == tsq.TSQ_ERR_INVALID_ARG
        # the calls that synchronize check their host pointers first
        info = tsq.tsq_info()
        assert L.tsq_compress_blocking(plan, 0x1000, 0x2000, 0x3000, None, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_compress_blocking(plan, None, 0x2000, 0x3000, None, C.byref(info)) == tsq.TSQ_ERR_INVALID_ARG
        out = (C.c_uint64 * 2)()
        ks = (C.c_uint32 * 2)(0, c.tokens + 1)
        assert L.tsq_prefix_bytes(plan, None, None, 2, out, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_prefix_bytes(plan, 0x2000, None, 0, out, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_prefix_bytes(plan, 0x2000, None, 2, None, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_prefix_bytes(plan, 0x2000, None, c.tokens + 2, out, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_prefix_bytes(plan, 0x2000, ks, 2, out, None) == tsq.TSQ_ERR_INVALID_ARG      # a count beyond the tokens
        assert L.tsq_entropy_prefix_bytes(plan, None, 0x3000, None, 2, out, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_entropy_prefix_bytes(plan, 0x2000, None, None, 2, out, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_entropy_prefix_bytes(plan, 0x2000, 0x3000, None, 0, out, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_entropy_prefix_bytes(plan, 0x2000, 0x3000, None, 2, None, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_entropy_prefix_bytes(plan, 0x2000, 0x3000, None, c.tokens + 2, out, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_entropy_prefix_bytes(plan, 0x2000, 0x3000, ks, 2, out, None) == tsq.TSQ_ERR_INVALID_ARG
        assert L.tsq_compress_static(plan, None, 0x2000, None) == tsq.TSQ_ERR_INVALID_ARG
    finally:
        tsq.tsq_plan_destroy(plan)
    # the measurement calls: sizes are multiples of 16 bytes, pointers 16-byte aligned
    assert L.tsq_measure_copy(None, 0x1000, 64, None) == tsq.TSQ_ERR_INVALID_ARG
    assert L.tsq_measure_copy(0x2000, 0x1000, 0, None) == tsq.TSQ_ERR_INVALID_ARG
    assert L.tsq_measure_copy(0x2000, 0x1000, 72, None) == tsq.TSQ_ERR_INVALID_ARG
    assert L.tsq_measure_copy(0x2008, 0x1000, 64, None) == tsq.TSQ_ERR_INVALID_ARG
    assert L.tsq_measure_read(0x1000, 64, None, None) == tsq.TSQ_ERR_INVALID_ARG
    assert L.tsq_measure_read(0x1004, 64, 0x3000, None) == tsq.TSQ_ERR_INVALID_ARG
    assert tsq.tsq_status_string(tsq.TSQ_ERR_NO_MEMORY) == "host allocation failed"
    plan = tsq.tsq_plan_create(c)
    try:
        pass
    finally:
        tsq.tsq_plan_destroy(plan)
    assert L.tsq_plan_blob_bytes(None) == 0 and L.tsq_plan_workspace_bytes(None) == 0
    L.tsq_plan_destroy(None)


def test_budget_may_be_infinite_and_zero(L):
    for b in (0.0, float("inf")):
        tsq.tsq_plan_destroy(tsq.tsq_plan_create(cfg(budget=b)))


@pytest.mark.parametrize("T,H,bits,cap", [(128, 768, (2, 4, 8), 0), (2048, 4096, (2, 3, 4, 6, 8), 1 << 20),
                                          (7, 40, (3,), 5), (1, 8, (2, 8), 0)])
def test_layout(L, T, H, bits, cap):
    plan = tsq.tsq_plan_create(cfg(tokens=T, hidden=H, bit_mask=tsq.bit_mask(bits), max_outliers=cap))
    try:
        lay = tsq.tsq_plan_layout(plan)
        offs = [lay.off_bits, lay.off_scale, lay.off_pay_off, lay.off_row_ptr, lay.off_payload,
                lay.off_out_col, lay.off_out_val]
        sizes = [T, 4 * T, 8 * (T + 1), 8 * (T + 1), lay.payload_capacity, 2 * lay.outlier_capacity,
                 2 * lay.outlier_capacity]
        assert offs[0] >= 128
        for o in offs:
            assert o % 256 == 0
        for (o, s), nxt in zip(zip(offs, sizes), offs[1:] + [lay.blob_bytes]):
            assert o + s <= nxt                                        # sections do not overlap
        assert lay.payload_capacity == T * 4 * ((H * max(bits) + 31) // 32)
        assert lay.outlier_capacity == (min(cap, T * H) if cap else T * H)
        assert lay.blob_bytes == tsq.tsq_plan_blob_bytes(plan)
        assert lay.workspace_bytes == tsq.tsq_plan_workspace_bytes(plan) > 0
    finally:
        tsq.tsq_plan_destroy(plan)


@pytest.mark.parametrize("T,H", [(128, 768), (2048, 4096), (7, 40), (1, 8), (100000, 8), (300, 32768)])
def test_entropy_sizes(L, T, H):
    """The coded blob holds a 256-byte header, seven tables, T + 1 offsets and room for the longest
    possible streams (per token 64 states and one 16-bit word per element); the encoder's workspace
    holds a slot of that size per token on top of its counters."""
    plan = tsq.tsq_plan_create(cfg(tokens=T, hidden=H))
    try:
        slot = 256 + 2 * ((H + 1) // 2 * 2)
        eb, ew = tsq.tsq_entropy_blob_bytes(plan), tsq.tsq_entropy_workspace_bytes(plan)
        need = 256 + 7 * 512 + 8 * (T + 1) + T * slot
        assert eb % 256 == 0 and need <= eb <= need + 4 * 256
        assert ew % 256 == 0 and ew >= T * slot + 4 * T + 16 * 7 * 1024
        assert ew <= T * slot + 8 * T + (1 << 20)
    finally:
        tsq.tsq_plan_destroy(plan)
    assert tsq.tsq_entropy_blob_bytes(0) == 0 and tsq.tsq_entropy_workspace_bytes(0) == 0


def test_status_strings(L):
    seen = {tsq.tsq_status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert tsq.tsq_status_string(99) == "unknown status"


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_04002_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
