"""tsq_compress_static (compress with the library's static device workspace, for callers that cannot
allocate) against tsq_compress, through the C ABI: same blob, bit for bit, on calls in a row
that share the static array, the later ones with smaller and differently shaped inputs."""
import numpy as np
import pytest

from paper_2511_04002_amd import synth

pytestmark = pytest.mark.gpu

SECTIONS = ("bits", "scale", "pay_off", "row_ptr", "payload", "out_col", "out_val")


@pytest.fixture(scope="module")
def tsq():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_04002_amd import tsq as m
    m.lib()
    return m


def rows(seed, T, H, dtype):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, H)) * rng.lognormal(0.0, 0.6, size=(T, 1))
    x[:, rng.choice(H, 3, replace=False)] *= 40.0
    return synth._cast(x, dtype)


def both_ways(tsq, x, dtype, bit_set, budget, pipeline):
    """-> (sections of tsq_compress, sections of tsq_compress_static, restored tensor of the latter)."""
    import torch
    T, H = x.shape
    plan = tsq.Plan(T, H, dtype, 8.0, bit_set, budget, pipeline=pipeline)
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    ref = plan.sections(plan.compress(xd))
    blob = plan.new_blob()
    blob.fill_(0x5A)
    tsq.tsq_compress_static(plan.handle, xd.data_ptr(), blob.data_ptr(), plan._stream())
    assert plan.info(blob).status == 0
    got = plan.sections(blob)
    out = plan.decompress(blob).cpu().numpy().view(np.uint16)
    ref_out = plan.decompress(plan.compress(xd)).cpu().numpy().view(np.uint16)
    return ref, got, out, ref_out


@pytest.mark.parametrize("pipeline", ["fused", "staged"])
def test_static_workspace_calls_in_a_row(tsq, pipeline):
    # large, then smaller (fewer and shorter rows), then another shape, then the first again: every call
    # finds what the one before left in the array
    cases = [(1500, 4096, "f16", (2, 3, 4, 6, 8), 0.1, 11), (200, 1024, "bf16", (2, 4, 8), 0.2, 12),
             (37, 8192, "bf16", (2, 3, 4, 5, 6, 8), 0.05, 13), (1500, 4096, "f16", (2, 3, 4, 6, 8), 0.1, 11)]
    for T, H, dtype, bit_set, budget, seed in cases:
        print("case", T, H, dtype, bit_set, budget, pipeline, flush=True)
        ref, got, out, ref_out = both_ways(tsq, rows(seed, T, H, dtype), dtype, bit_set, budget, pipeline)
        for name in SECTIONS:
            assert np.array_equal(got[name], ref[name]), name
        assert np.array_equal(out, ref_out)
        assert len(set(ref["bits"].tolist())) > 1          # the calls place variable-length tokens


def test_static_workspace_limit(tsq):
    limit = tsq.tsq_static_workspace_bytes()
    assert limit == 4 << 20
    big = tsq.Plan(250000, 8, "f16", 8.0, (2, 8), 0.05)
    assert big.layout.workspace_bytes > limit
    with pytest.raises(tsq.TsqError) as e:
        tsq.tsq_compress_static(big.handle, 0x1000, 0x2000, 0)          # refused before the pointers are used
    assert e.value.status == tsq.TSQ_ERR_UNSUPPORTED
