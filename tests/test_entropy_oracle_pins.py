"""Pins of the symbol-statistics oracle (oracle/entropy_oracle.py) against things other than itself."""
import numpy as np
import pytest

from paper_2511_04002_amd import synth


@pytest.fixture(scope="module")
def E(oracle):
    from oracle import entropy_oracle
    return entropy_oracle


def test_histogram_of_eight_bit_tokens_is_the_byte_count_of_the_payload(oracle, E):
    # at b = 8 the payload bytes ARE the codes (packing pin), so numpy.bincount on the raw bytes,
    # which never goes through the field extraction, must give the same table
    x = synth.make_c1()
    c = oracle.compress(x, oracle.F16, 6.0, (8,), 0.0, oracle.BUDGET_REL_RMS)
    h = E.code_histogram(c)
    for t in (0, 5, 127):
        lo, hi = int(c.pay_off[t]), int(c.pay_off[t + 1])
        assert np.array_equal(h[t], np.bincount(c.payload[lo:hi][: c.hidden], minlength=256))


def test_histogram_from_the_definition_of_the_codes(oracle, E):
    # dyadic rows: the quantizer is exact, so the codes follow in closed form from the input
    H, b = 96, 5
    Q = 2 ** (b - 1) - 1
    g = np.random.Generator(np.random.PCG64(3))
    k = g.integers(-Q, Q + 1, size=(4, H))
    k[:, 0] = Q                                        # the absmax element fixes s = 2^-3 exactly
    x = synth.to_f16_bits(k * 0.125)
    c = oracle.compress(x, oracle.F16, 100.0, (b,), 0.0, oracle.BUDGET_LSB)
    h = E.code_histogram(c)
    for t in range(4):
        code = np.where(k[t] < 0, (1 << (b - 1)) | -k[t], k[t])
        assert np.array_equal(h[t], np.bincount(code, minlength=256))


def test_rows_sum_to_hidden_and_stay_inside_the_width(oracle, E):
    x = synth.make_c2(tokens=64)
    c = oracle.compress(x, oracle.F16, 8.0, (2, 3, 4, 6, 8), 0.2, oracle.BUDGET_REL_RMS)
    h = E.code_histogram(c)
    assert np.all(h.sum(axis=1) == c.hidden)
    for t in range(c.tokens):
        assert not h[t, 1 << int(c.bits[t]):].any()
    # outlier slots carry code 0: at least cnt_t zeros per token
    cnt = np.diff(c.row_ptr).astype(np.int64)
    assert np.all(h[:, 0].astype(np.int64) >= cnt)
    # negative zero does not exist: the code "sign bit only" never occurs
    for t in range(c.tokens):
        assert h[t, 1 << (int(c.bits[t]) - 1)] == 0


def test_entropy_closed_forms(E):
    assert E.entropy_bits(np.array([7, 0, 0])) == 0.0                    # one symbol: nothing to code
    assert E.entropy_bits(np.array([5, 5])) == pytest.approx(10.0)       # fair coin: one bit each
    assert E.entropy_bits(np.full(256, 3)) == pytest.approx(3 * 256 * 8.0)
    assert E.entropy_bits(np.array([3, 1])) == pytest.approx(3 * np.log2(4 / 3) + 2.0)
    assert E.entropy_bits(np.zeros(4)) == 0.0
    # never above the packed size, never below zero; pooling tables cannot beat private tables
    g = np.random.Generator(np.random.PCG64(0))
    h = g.integers(0, 50, size=(6, 16))
    each = sum(E.entropy_bits(r) for r in h)
    assert 0.0 <= each <= h.sum() * 4.0 + 1e-9
    assert E.entropy_bits(h.sum(axis=0)) >= each - 1e-9


def test_report_orders_the_three_sizes(oracle, E):
    x = synth.make_c2(tokens=48)
    c = oracle.compress(x, oracle.F16, 8.0, (2, 3, 4, 6, 8), 0.05, oracle.BUDGET_REL_RMS)
    r = E.report(E.code_histogram(c), c.bits, c.hidden)
    assert r["per_token_table"] <= r["per_width_table"] + 1e-12 <= r["packed"] + 1e-12
