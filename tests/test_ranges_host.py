"""The range predicates that the kernels apply to offsets, sizes and indices read from a blob, an
entropy-coded blob or a workspace, driven on the host (include/tsq_ranges.h runs the same source the
kernels compile) with the wrapping offsets and the noise that the GPU failure-path tests feed the
kernels.  Each predicate is compared with the condition it stands for, written here with Python's
unbounded integers, where nothing can wrap."""
import numpy as np
import pytest

from paper_2511_04002_amd import build as tsq_build
from paper_2511_04002_amd import tsq

U64 = (1 << 64) - 1
U32 = (1 << 32) - 1


@pytest.fixture(scope="module")
def L():
    tsq_build.build()
    return tsq.lib()


def edge_values_64(g, around):
    """Values near 0, near 2^64 and near the given limits, plus noise."""
    out = [0, 1, 2, 3, 4, 5, 7, 8, U64, U64 - 1, U64 - 3, U64 - 4, 1 << 63, (1 << 63) - 4, 1 << 32, (1 << 32) - 4]
    for a in around:
        out += [max(0, a - 8), max(0, a - 4), max(0, a - 1), a, min(U64, a + 1), min(U64, a + 4)]
    out += [int(v) for v in g.integers(0, 1 << 63, 24, dtype=np.uint64) * 2 + g.integers(0, 2, 24, dtype=np.uint64)]
    return out


def test_payload_span(L):
    g = np.random.Generator(np.random.PCG64(1))
    for hidden in (8, 40, 768, 4096, 8192, 32768):
        for cap in (0, 4, 4 * ((hidden * 8 + 31) // 32), 3 * 4 * ((hidden * 8 + 31) // 32) + 4, 1 << 33, U64):
            for b in (0, 1, 2, 3, 5, 8, 9, 15, 255, U32):
                nbytes = 4 * ((hidden * b + 31) // 32) if b <= 8 else None
                for po in edge_values_64(g, (cap, max(0, cap - (nbytes or 0)))):
                    want = 2 <= b <= 8 and po % 4 == 0 and po + nbytes <= cap
                    assert L.tsq_check_payload_span(hidden, cap, b, po) == int(want), (hidden, cap, b, po)


def test_csr_slices(L):
    g = np.random.Generator(np.random.PCG64(2))
    for cap in (0, 1, 1000, 1 << 32, U64):
        vals = edge_values_64(g, (cap,))
        for rp0 in vals:
            for rp1 in vals[::3]:
                ok = rp0 <= rp1 <= cap
                assert L.tsq_check_csr_slice(rp0, rp1, cap) == int(ok)
                for cnt in (0, 1, 5, U32):
                    assert L.tsq_check_csr_slice_holds(rp0, rp1, cap, cnt) == int(ok and rp1 - rp0 == cnt)
    for hidden in (8, 4096, 32768):
        for col in (0, hidden - 1, hidden, hidden + 1, 65535, U32):
            assert L.tsq_check_column(col, hidden) == int(col < hidden)


def test_stream_spans(L):
    g = np.random.Generator(np.random.PCG64(3))
    for coders, slot in ((1, 256 + 16), (24, 256 + 1536), (64, 256 + 16384), (64, 256 + 65536)):
        for cap in (0, 4 * coders, slot, 1000 * slot, U64):
            vals = edge_values_64(g, (cap, 4 * coders, slot))
            for a in vals:
                for b in vals[::2]:
                    want = a <= b <= cap and a % 4 == 0 and 4 * coders <= b - a <= slot
                    assert L.tsq_check_stream_span(a, b, cap, coders, slot) == int(want), (a, b, cap, coders, slot)
            for nbytes in (0, 4 * coders - 1, 4 * coders, 4 * coders + 1, slot - 1, slot, slot + 1, U32, U32 - 2):
                for at in vals:
                    padded = (nbytes + 3) // 4 * 4
                    want = 4 * coders <= nbytes <= slot and at + padded <= cap
                    assert L.tsq_check_stream_move(nbytes, coders, slot, at, cap) == int(want), (nbytes, at, cap)


def test_slot_and_shape(L):
    g = np.random.Generator(np.random.PCG64(4))
    for x in [0, 1, 4095, 4096, 4097, U32, 1 << 16, (1 << 16) - 1] + [int(v) for v in g.integers(0, 1 << 32, 200)]:
        s = L.tsq_check_frequency_slot(x)
        assert s == x % 4096 and s < 4096
    for a in (0, 1, 600, U32):
        for b in (0, 8, 4096, U32):
            assert L.tsq_check_workspace_shape(a, b, 600, 4096) == int((a, b) == (600, 4096))
