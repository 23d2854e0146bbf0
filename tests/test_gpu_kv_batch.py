"""Parity of the KV-cache form (tsq_compress_batch / tsq_decompress_batch) with the CPU oracle.

The oracle has no batch form of its own: what the paper says about the cache (Sec. II-B,
Eq. (bkv_lth_stage): the key and value tensors of every layer; footnote of Sec. II-C.1: they go
through the same TS + TAB-Q) makes the batch the concatenation of its tensors' rows, so the
expected blob is the oracle's blob of the concatenation, to the bit, and the restored tensors
are the slices of the oracle's restored concatenation.
"""
import numpy as np
import pytest

from paper_2511_04002_amd import synth

pytestmark = pytest.mark.gpu

DT = {"f16": 0, "bf16": 1}
PIPELINES = ["fused", "staged"]
SECTIONS = ("bits", "scale", "row_ptr", "pay_off", "out_col", "out_val", "payload")


@pytest.fixture(scope="module")
def tsq():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_04002_amd import tsq as m
    m.lib()
    return m


def scattered(parts):
    """Every tensor in a device allocation of its own, with unrelated allocations in between."""
    import torch
    keep, xs = [], []
    for i, p in enumerate(parts):
        keep.append(torch.empty(256 * (1 + i % 3), dtype=torch.uint8, device="cuda"))
        xs.append(torch.from_numpy(p.view(np.int16).copy()).cuda())
    return xs, keep


def check_batch(tsq, oracle, parts, dtype, tau, bit_set, budget, pipeline, label):
    import torch
    rows, H = parts[0].shape
    print("case", label, len(parts), "x", parts[0].shape, dtype, tau, bit_set, budget, pipeline, flush=True)
    x = np.concatenate(parts)
    ref = oracle.compress(x, DT[dtype], tau, bit_set, budget, 1, nthreads=8)
    ref_out = oracle.decompress(ref, nthreads=8)

    plan = tsq.Plan(x.shape[0], H, dtype, tau, bit_set, budget, mode="rel_rms", pipeline=pipeline,
                    max_outliers=max(ref.nnz, 1))
    xs, keep = scattered(parts)
    ws = plan.new_workspace()
    blob = plan.new_blob()
    blob.fill_(0xA5)
    _, table = plan.compress_batch(xs, blob, ws)
    info = plan.info(blob)
    sec = plan.sections(blob)
    ref_sec = {"bits": ref.bits, "scale": ref.scale, "row_ptr": ref.row_ptr, "pay_off": ref.pay_off,
               "out_col": ref.out_col, "out_val": ref.out_val, "payload": ref.payload}
    for k in SECTIONS:
        a, b = sec[k], ref_sec[k]
        if k == "scale":
            a, b = a.view(np.uint32), b.view(np.uint32)
        assert np.array_equal(a, b), k
    assert info.nnz == ref.nnz and info.payload_bytes == ref.payload_bytes and info.status == 0
    assert info.compressed_bytes == oracle.compressed_bytes(ref)

    # the contiguous form gives the same blob
    blob_c = plan.new_blob()
    blob_c.fill_(0x3C)
    plan.compress(torch.from_numpy(x.view(np.int16)).cuda(), blob_c, ws)
    sec_c = plan.sections(blob_c)
    for k in SECTIONS + ("header",):
        assert np.array_equal(sec[k], sec_c[k]), "contiguous vs batch: " + k

    # restore into separate tensors, from either blob; and the batch blob into one tensor
    for src in (blob, blob_c):
        outs = [torch.full((rows, H), 0x5A5A, dtype=torch.int16, device="cuda") for _ in parts]
        plan.decompress_batch(src, outs)
        torch.cuda.synchronize()
        for i, o in enumerate(outs):
            got = o.cpu().numpy().view(np.uint16)
            assert np.array_equal(got, ref_out[i * rows:(i + 1) * rows]), "restored tensor %d" % i
    whole = plan.new_output()
    plan.decompress(blob, whole)
    assert np.array_equal(whole.cpu().numpy().view(np.uint16), ref_out)
    del keep, table
    return ref


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("name,layers,rows", [("KV7", 3, 40), ("KV13", 2, 33), ("KV7", 1, 700)])
def test_kv_cache_shapes(tsq, oracle, pipeline, name, layers, rows):
    w = synth.WORKLOADS[name]
    parts = synth.make_kv(name, layers=layers, rows=rows)
    ref = check_batch(tsq, oracle, parts, w.dtype, w.tau, w.bit_set, 0.05, pipeline, name)
    assert ref.nnz > 0
    check_batch(tsq, oracle, parts, w.dtype, w.tau, w.bit_set, 0.3, pipeline, name + " loose")


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_one_row_per_tensor_and_one_tensor(tsq, oracle, pipeline, dtype):
    # the new token's keys and values of every layer: tensors of a single row
    x = synth.edge_rows(264, dtype, 6.0)
    check_batch(tsq, oracle, [x[i:i + 1] for i in range(x.shape[0])], dtype, 6.0, (2, 4, 5, 8), 0.05, pipeline,
                "rows of their own")
    check_batch(tsq, oracle, [x], dtype, 6.0, (2, 4, 5, 8), 0.05, pipeline, "a single tensor")


@pytest.mark.parametrize("pipeline", PIPELINES)
def test_more_tensors_than_the_grid_has_workgroups(tsq, oracle, pipeline):
    g = np.random.Generator(np.random.PCG64(11))
    parts = [synth.to_f16_bits(g.standard_normal((3, 64)) * 4.0) for _ in range(1500)]
    check_batch(tsq, oracle, parts, "f16", 6.0, (2, 3, 4, 8), 0.1, pipeline, "1500 tensors of 3 rows")


def test_rows_per_tensor_must_divide_the_tokens(tsq):
    import torch
    plan = tsq.Plan(12, 64, "f16", 6.0, (4, 8), 0.05)
    table = torch.zeros(16, dtype=torch.int64, device="cuda")
    blob, ws = plan.new_blob(), plan.new_workspace()
    for rows in (0, 5, 13):
        with pytest.raises(tsq.TsqError) as e:
            tsq.tsq_compress_batch(plan.handle, table.data_ptr(), rows, blob.data_ptr(), ws.data_ptr(), 0)
        assert e.value.status == tsq.TSQ_ERR_INVALID_ARG
        with pytest.raises(tsq.TsqError) as e:
            tsq.tsq_decompress_batch(plan.handle, blob.data_ptr(), table.data_ptr(), rows, 0)
        assert e.value.status == tsq.TSQ_ERR_INVALID_ARG


def test_kv7_full_size(tsq, oracle):
    """The KV-cache workload at the size that is timed (64 tensors of 1024 x 4096), whole blob against the oracle."""
    import torch
    w = synth.WORKLOADS["KV7"]
    parts = synth.make_kv("KV7")
    x = np.concatenate(parts)
    ref = oracle.compress(x, DT[w.dtype], w.tau, w.bit_set, 0.05, 1, nthreads=8)
    plan = tsq.Plan(x.shape[0], w.hidden, w.dtype, w.tau, w.bit_set, 0.05, max_outliers=max(ref.nnz, 1))
    xs = [torch.from_numpy(p.view(np.int16)).cuda() for p in parts]
    blob, _ = plan.compress_batch(xs)
    assert plan.info(blob).status == 0
    sec = plan.sections(blob)
    for k, want in (("bits", ref.bits), ("row_ptr", ref.row_ptr), ("pay_off", ref.pay_off), ("out_col", ref.out_col),
                    ("out_val", ref.out_val), ("payload", ref.payload)):
        assert np.array_equal(sec[k], want), k
    assert np.array_equal(sec["scale"].view(np.uint32), ref.scale.view(np.uint32))
    outs = [torch.empty_like(t) for t in xs]
    plan.decompress_batch(blob, outs)
    ref_out = oracle.decompress(ref, nthreads=8)
    rows = parts[0].shape[0]
    for i in (0, 1, 31, 63):
        assert np.array_equal(outs[i].cpu().numpy().view(np.uint16), ref_out[i * rows:(i + 1) * rows])
