"""Parity of tsq_code_histogram with the symbol-statistics oracle: integer counts, bit-exact."""
import numpy as np
import pytest

from paper_2511_04002_amd import synth

pytestmark = pytest.mark.gpu

DT = {"f16": 0, "bf16": 1}


@pytest.fixture(scope="module")
def tsq():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_04002_amd import tsq as m
    m.lib()
    return m


@pytest.fixture(scope="module")
def E(oracle):
    from oracle import entropy_oracle
    return entropy_oracle


def check(tsq, oracle, E, x, dtype, tau, bit_set, budget, mode=1, label=""):
    import torch
    print("case", label, x.shape, dtype, tau, bit_set, budget, flush=True)
    T, H = x.shape
    ref = oracle.compress(x, DT[dtype], tau, bit_set, budget, mode, nthreads=8)
    want = E.code_histogram(ref)
    plan = tsq.Plan(T, H, dtype, tau, bit_set, budget, mode="rel_rms" if mode == 1 else "lsb",
                    max_outliers=max(ref.nnz, 1))
    blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    assert plan.info(blob).status == 0
    hist = torch.full((T, 256), -1, dtype=torch.int32, device="cuda")
    plan.code_histogram(blob, hist)
    got = hist.cpu().numpy().view(np.uint32)
    assert np.array_equal(got, want)
    return ref, got


def test_c1_and_c2(tsq, oracle, E):
    for eps in (0.05, 0.1, 0.3):
        check(tsq, oracle, E, synth.make_c1(), "f16", 6.0, (2, 4, 8), eps, label="C1")
    ref, _ = check(tsq, oracle, E, synth.make_c2(tokens=512), "f16", 8.0, (2, 3, 4, 6, 8), 0.2, label="C2")
    assert len(set(ref.bits.tolist())) >= 2


def test_c4_rows_every_width(tsq, oracle, E):
    x = synth.make_c4(tokens=1024)
    seen = set()
    for bs, eps in (((2, 3, 4, 5, 6, 8), 0.05), ((2, 3, 4, 5, 6, 8), 0.2), ((7,), 0.0), ((2, 3), 0.0), ((2, 7), 1.0)):
        ref, _ = check(tsq, oracle, E, x, "bf16", 10.0, bs, eps, label="C4 rows")
        seen |= set(ref.bits.tolist())
    assert seen == {2, 3, 4, 5, 6, 7, 8}


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H", [8, 24, 40, 264, 1000, 2056, 32768])
def test_edge_rows_and_ragged_hidden(tsq, oracle, E, dtype, H):
    x = synth.edge_rows(H, dtype, 6.0) if H >= 264 else None
    if x is None:
        g = np.random.Generator(np.random.PCG64(H))
        v = g.standard_normal((37, H)) * 3.0
        x = synth.to_f16_bits(v) if dtype == "f16" else synth.to_bf16_bits(v)
    for bs, bud, mode in (((2, 4, 5, 8), 0.05, 1), ((2, 3, 4, 5, 6, 7, 8), 0.3, 0), ((3, 6), 0.5, 1)):
        _, got = check(tsq, oracle, E, x, dtype, 6.0, bs, bud, mode, label="edge H=%d" % H)
        assert np.all(got.sum(axis=1) == H)


def test_a_foreign_blob_is_left_alone(tsq):
    import torch
    plan = tsq.Plan(16, 64, "f16", 6.0, (4, 8), 0.05)
    blob = plan.new_blob()
    blob.zero_()
    hist = torch.full((16, 256), 7, dtype=torch.int32, device="cuda")
    plan.code_histogram(blob, hist)
    torch.cuda.synchronize()
    assert bool((hist == 7).all())
