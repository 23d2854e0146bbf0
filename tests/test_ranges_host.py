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


def test_encoder_quotient_is_exact_or_one_less(L):
    """The entropy encoder divides a state x < f << 20 by a frequency 1 <= f <= 4096 through a binary32 product
    with a reciprocal rounded down a little, and repairs the result by the size of the remainder.  That is
    exact only if the product's integer part is floor(x / f) or one less, for EVERY admissible pair; here the
    very routine the kernel compiles is run on the host for every f, on the pairs where a rounding could
    hurt (just below, at and just above multiples of f; the largest quotients, where the product has the
    fewest spare bits; states with all mantissa bits set) and on noise."""
    g = np.random.Generator(np.random.PCG64(7))
    xs, fs = [], []
    for f in range(1, 4097):
        top = (f << 20) - 1                                   # the largest admissible state
        qs = np.concatenate([
            np.array([1, 2, 3, 255, 256, 4095, 4096, 65535, 65536, (1 << 19) - 1, 1 << 19, (1 << 20) - 2, (1 << 20) - 1], np.int64),
            g.integers(1, 1 << 20, 40)])
        for r in (-1, 0, 1, f // 2, f - 1):
            x = qs * f + r
            x = x[(x >= 0) & (x <= top)]
            xs.append(x); fs.append(np.full(x.size, f, np.int64))
        x = g.integers(0, top + 1, 60)
        xs.append(x); fs.append(np.full(x.size, f, np.int64))
        # states whose binary32 conversion rounds up: low bits all ones
        x = np.minimum(top, (g.integers(1 << 24, 1 << 32, 20) | 0xFF))
        xs.append(x); fs.append(np.full(x.size, f, np.int64))
        xs.append(np.array([top, top - 1, 0, f - 1, f], np.int64)); fs.append(np.full(5, f, np.int64))
    x = np.concatenate(xs).astype(np.uint32); f = np.concatenate(fs).astype(np.uint32)
    assert np.all(x.astype(np.int64) < (f.astype(np.int64) << 20))
    q = np.zeros(x.size, np.uint32)
    L.tsq_check_quotients(x.ctypes.data, f.ctypes.data, q.ctypes.data, x.size)
    true = x.astype(np.int64) // f.astype(np.int64)
    d = true - q.astype(np.int64)
    assert d.min() >= 0 and d.max() <= 1, (x[d.argmax()], f[d.argmax()], x[d.argmin()], f[d.argmin()])
    # both cases occur, so the test exercises the correction
    assert (d == 0).any() and (d == 1).any()
    # what the encoder makes of it: remainder below 2f, and the repaired pair is the true one
    r1 = x.astype(np.int64) - q.astype(np.int64) * f.astype(np.int64)
    assert np.all((r1 >= 0) & (r1 < 2 * f.astype(np.int64)))
    assert np.array_equal(np.where(r1 >= f, q.astype(np.int64) + 1, q.astype(np.int64)), true)
