"""The other readings of the quantizer (oracle/variants.py): what must hold between them and the
library's reading, whatever the data."""
import numpy as np
import pytest

from paper_2511_04002_amd import synth


@pytest.fixture(scope="module")
def V(oracle):
    from oracle import variants
    return variants


def test_library_variant_is_the_oracle_itself(oracle, V):
    x = synth.make_c1()
    c = oracle.compress(x, oracle.F16, 6.0, (2, 4, 8), 0.1, oracle.BUDGET_REL_RMS)
    o = V.baseline(x, oracle.F16, 6.0, (2, 4, 8), 0.1, oracle.BUDGET_REL_RMS)
    assert np.array_equal(o.bits, c.bits)
    # its reconstruction, stored as fp16, is what decompress returns at the inlier slots
    dec = oracle.decompress(c).view(np.float16).astype(np.float32)
    out = np.zeros(x.shape, bool)
    for t in range(x.shape[0]):
        out[t, c.out_col[int(c.row_ptr[t]):int(c.row_ptr[t + 1])]] = True
    assert np.array_equal(o.recon.astype(np.float16).astype(np.float32)[~out], dec[~out])


def test_literal_break_is_one_step_further_down(oracle, V):
    x = synth.make_c2(tokens=96)
    B = (2, 3, 4, 6, 8)
    W = sorted(B, reverse=True)
    for eps in (0.0, 0.05, 0.2, float("inf")):
        lib = V.baseline(x, oracle.F16, 8.0, B, eps, oracle.BUDGET_REL_RMS)
        lit = V.literal_break(x, oracle.F16, 8.0, B, eps, oracle.BUDGET_REL_RMS)
        for a, b in zip(lib.bits.tolist(), lit.bits.tolist()):
            # either the next narrower width (the one that failed) or, if nothing failed, the same smallest one
            assert b == (W[W.index(a) + 1] if a != W[-1] else a) or (a == b == W[-1])
        assert lit.rel_rmse() >= lib.rel_rmse()
    assert set(V.literal_break(x, oracle.F16, 8.0, B, float("inf"), 1).bits.tolist()) == {2}


def test_with_minimum_equals_the_library_where_a_zero_is_present(oracle, V):
    x = synth.make_c1().copy()
    x[:, 5] = 0                                        # an exact zero in every token: T_min = 0
    a = V.baseline(x, oracle.F16, 6.0, (4, 8), 0.05, 1)
    b = V.with_minimum(x, oracle.F16, 6.0, (4, 8), 0.05, 1)
    assert np.array_equal(a.bits, b.bits)
    # the same grid; a / s and a * (1 / s) may round a tie differently, by one step, almost nowhere
    differ = a.recon != b.recon
    assert differ.mean() < 1e-3
    step = np.abs(a.inl).max(axis=1, keepdims=True) / 7.0
    assert np.all(np.abs(a.recon - b.recon) <= step * 1.001)
    # and can only help (a finer step) where the smallest magnitude is far from zero
    g = np.random.Generator(np.random.PCG64(1))
    y = synth.to_f16_bits(g.uniform(2.0, 3.0, size=(8, 256)) * g.choice([-1.0, 1.0], size=(8, 256)))
    a = V.baseline(y, oracle.F16, 6.0, (4,), 0.0, 1)
    b = V.with_minimum(y, oracle.F16, 6.0, (4,), 0.0, 1)
    assert b.rel_rmse() < 0.5 * a.rel_rmse()


def test_whole_tensor_uses_one_width_and_the_largest_magnitude(oracle, V):
    x = synth.make_c2(tokens=64)
    o = V.whole_tensor(x, oracle.F16, 8.0, (2, 3, 4, 6, 8), 0.05, 1)
    assert len(set(o.bits.tolist())) == 1
    # tokens of small scale lose precision against the per-token reading at the same width
    b = int(o.bits[0])
    per = V.baseline(x, oracle.F16, 8.0, (b,), 0.05, 1)
    assert o.rel_rmse() > per.rel_rmse()


def test_the_c_switch_gives_the_widths_of_the_python_variant(oracle, V):
    """The printed return rule twice: derived in variants.py from the default descent's record, and as the
    switch of the C descent itself, which is what the GPU path is compared with."""
    for x, dt, tau, bs in ((synth.make_c1(), oracle.F16, 6.0, (2, 4, 8)),
                           (synth.make_c2(tokens=64), oracle.F16, 8.0, (2, 3, 4, 6, 8)),
                           (synth.make_c4(tokens=32), oracle.BF16, 10.0, (2, 3, 4, 5, 6, 8))):
        for eps in (0.0, 0.05, 0.1, 0.2, 0.5):
            want = V.literal_break(x, dt, tau, bs, eps, oracle.BUDGET_REL_RMS).bits
            got = oracle.compress(x, dt, tau, bs, eps, oracle.BUDGET_REL_RMS, rule=oracle.RETURN_AS_PRINTED).bits
            assert np.array_equal(got, want), eps
