"""Pins of the rANS oracle (oracle/rans_oracle.py): a table worked by hand, a stream worked by
hand, the coder's defining identity (decode inverts encode), and Shannon's bound."""
import math

import numpy as np
import pytest

from paper_2511_04002_amd import synth


@pytest.fixture(scope="module")
def R(oracle):
    from oracle import rans_oracle
    return rans_oracle


@pytest.fixture(scope="module")
def E(oracle):
    from oracle import entropy_oracle
    return entropy_oracle


def test_normalize_by_hand(R):
    assert R.normalize([0, 0, 0, 0]).tolist() == [0, 0, 0, 0]
    assert R.normalize([5, 0, 0, 0]).tolist() == [4096, 0, 0, 0]
    assert R.normalize([1, 1, 1, 1]).tolist() == [1024] * 4
    assert R.normalize([3, 1]).tolist() == [3072, 1024]
    # floors 1365 + 1365 + 1365 = 4095: the deficit of 1 goes to the first of the largest counts
    assert R.normalize([1, 1, 1]).tolist() == [1366, 1365, 1365]
    # a rare code is lifted to 1 and the most frequent one absorbs what the floors lost:
    # 10^6 * 4096 // 1000001 = 4095, the rare code -> 1, sum already 4096
    assert R.normalize([10 ** 6, 1]).tolist() == [4095, 1]
    # many rare codes: 200 codes of count 1 and one of 10^9 -> floors 4095 + 200 * 1 = 4295, 199 too many:
    # they are taken one by one from the largest entry
    f = R.normalize([10 ** 9] + [1] * 200)
    assert f.tolist() == [4096 - 200] + [1] * 200
    g = np.random.Generator(np.random.PCG64(0))
    for _ in range(200):
        k = int(g.integers(1, 257))
        n = g.integers(0, 10 ** int(g.integers(1, 8)), size=k)
        f = R.normalize(n)
        if n.sum() == 0:
            assert not f.any()
            continue
        assert int(f.sum()) == 4096 and np.all((f > 0) == (n > 0))
        # close to proportional: within one unit plus the repairs, which touch the largest entries only
        ideal = n * 4096.0 / n.sum()
        small = n < n.max()
        assert np.all(np.abs(f[small] - ideal[small]) <= 1.0 + 1e-9) or f.max() <= ideal.max() + 256


def test_single_symbol_stream_by_hand(R):
    # one code, one coder active (H = 1): freq [1024, 3072], code 1 (f = 3072, c = 1024)
    # x = 65536 < 3072 << 20: no word.  x = (65536 // 3072) << 12 + 65536 % 3072 + 1024 = 21*4096 + 1024 + 1024
    s = R.encode_token([1], np.array([1024, 3072], np.uint16))
    # one run only: one coder in use, one state in the stream
    assert np.frombuffer(s, "<u4").tolist() == [21 * 4096 + 2048] and len(s) == 4
    assert R.decode_token(s, 1, np.array([1024, 3072], np.uint16)).tolist() == [1]
    # a state that has to shed a word: start is 65536, after one rare symbol (f = 1, c = 0):
    # x = 65536 << 12 = 2^28; second rare symbol: 2^28 >= 1 << 20 -> emit 0, x = 2^12, then x = 2^24
    s = R.encode_token([0, 0], np.array([1, 4095], np.uint16))
    # both codes belong to coder 0 (elements 0 and 1 of run 0); the encoder sees element 1 first
    assert np.frombuffer(s[:4], "<u4")[0] == 1 << 24
    assert np.frombuffer(s[4:6], "<u2")[0] == 0 and len(s) == 8
    assert R.decode_token(s, 2, np.array([1, 4095], np.uint16)).tolist() == [0, 0]


@pytest.mark.parametrize("H", [1, 31, 32, 33, 2047, 2048, 2049, 5000])
@pytest.mark.parametrize("b", [2, 5, 8])
def test_decode_inverts_encode(R, H, b):
    g = np.random.Generator(np.random.PCG64(H * 10 + b))
    p = g.dirichlet(np.full(1 << b, 0.3))
    codes = g.choice(1 << b, size=H, p=p)
    freq = R.normalize(np.bincount(codes, minlength=256))
    s = R.encode_token(codes, freq)
    assert len(s) % 4 == 0
    assert np.array_equal(R.decode_token(s, H, freq), codes)
    # size: within the ideal code length of this table, plus the 64 states, plus 2 bytes per coder for the
    # word in flight, plus padding -- and not below the ideal minus the states' head start
    ideal_bits = float(sum(math.log2(4096.0 / int(freq[c])) for c in codes))
    k = R.coders_in_use(H)
    assert len(s) >= 4 * k
    assert 8 * len(s) <= ideal_bits + k * 32 + k * 16 + 32
    assert 8 * len(s) >= ideal_bits - 32


def test_whole_tensor_round_trip_and_size(oracle, R, E):
    x = synth.make_c2(tokens=24)
    c = oracle.compress(x, oracle.F16, 8.0, (2, 3, 4, 6, 8), 0.2, oracle.BUDGET_REL_RMS)
    hist = E.code_histogram(c)
    tables, off, streams = R.encode(c, hist)
    assert len(set(c.bits.tolist())) >= 2
    for b in range(2, 9):
        assert int(tables[b - 2].sum()) == (4096 if (c.bits == b).any() else 0)
    total = 0.0
    for t in range(c.tokens):
        codes = R.decode_codes(tables, off, streams, c.bits, c.hidden, t)
        assert np.array_equal(codes, E.token_codes(c, t))
        total += sum(math.log2(4096.0 / int(tables[int(c.bits[t]) - 2][k])) for k in codes)
    # the streams cost what the tables promise, plus 256 bytes of states per token (and change)
    assert int(off[-1]) == len(streams)
    k = R.coders_in_use(c.hidden)
    assert 8 * len(streams) <= total + c.tokens * (k * 32 + k * 16 + 32)
    # and the tables promise close to the pooled entropy of the report
    pooled = E.report(hist, c.bits, c.hidden)["per_width_table"] * c.tokens * c.hidden
    assert total <= pooled * 1.01 + 4096


@pytest.mark.parametrize("H", [1, 2, 31, 32, 33, 2047, 2048, 2049, 5000])
def test_compiled_coder_is_the_python_coder(R, H):
    """rans_oracle.c against encode_token (which the hand-worked streams above pin), token by token and as a
    whole tensor."""
    # the hand-worked streams once more
    assert R.encode_token_c([1], np.array([1024, 3072], np.uint16)) == np.array([21 * 4096 + 2048], "<u4").tobytes()
    s = R.encode_token_c([0, 0], np.array([1, 4095], np.uint16))
    assert np.frombuffer(s[:4], "<u4")[0] == 1 << 24 and np.frombuffer(s[4:6], "<u2")[0] == 0 and len(s) == 8
    g = np.random.Generator(np.random.PCG64(H))
    T = 7
    bits = g.choice([2, 3, 5, 8], size=T).astype(np.uint8)
    codes = np.zeros((T, H), np.uint8)
    tables = np.zeros((7, 256), np.uint16)
    for b in set(bits.tolist()):
        p = g.dirichlet(np.full(1 << b, 0.3))
        rows = np.flatnonzero(bits == b)
        codes[rows] = g.choice(1 << b, size=(len(rows), H), p=p)
        tables[b - 2] = R.normalize(np.bincount(codes[rows].ravel(), minlength=256))
    off, streams = R.encode_codes_c(codes, bits, tables)
    at = 0
    for t in range(T):
        want = R.encode_token(codes[t], tables[int(bits[t]) - 2])
        assert R.encode_token_c(codes[t], tables[int(bits[t]) - 2]) == want
        assert int(off[t]) == at and streams[at: at + len(want)].tobytes() == want
        at += len(want)
    assert int(off[T]) == at == len(streams)
