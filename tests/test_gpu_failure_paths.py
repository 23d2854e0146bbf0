"""Error paths of the single-pass compress that the host can force without breaking a kernel: a
workspace that was not reset for the plan's shape is left alone and reported as TSQ_ERR_FORMAT; one of
the right shape in an arbitrary state ends in TSQ_ERR_INTERNAL in the blob's header (every device-side
wait is bounded), never in a hang; tsq_workspace_reset brings the workspace back."""
import numpy as np
import pytest

from paper_2511_04002_amd import synth

pytestmark = pytest.mark.gpu

SECTIONS = ("bits", "row_ptr", "pay_off", "out_col", "out_val", "payload")


@pytest.fixture(scope="module")
def tsq():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_04002_amd import tsq as m
    m.lib()
    return m


CTL_ERROR, CTL_TOKENS, CTL_HIDDEN = 1, 2, 3       # 32-bit words at the start of a workspace


@pytest.mark.parametrize("pipeline", ["fused", "staged"])
def test_a_workspace_of_another_shape_is_left_alone_and_reported(tsq, oracle, pipeline):
    """A workspace that was never reset (all-ones bytes here), and one reset for a plan of another shape:
    the call stores a header with TSQ_ERR_FORMAT and nothing else, the workspace keeps every byte, and the
    plan it was reset for still gets the oracle's blob from it."""
    import torch
    x = synth.make_c2(tokens=600)
    T, H = x.shape
    plan = tsq.Plan(T, H, "f16", 8.0, (2, 3, 4, 6, 8), 0.05, pipeline=pipeline)
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    blob = plan.new_blob()
    ws = torch.empty(int(plan.layout.workspace_bytes), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    print("compress on a workspace of all-ones bytes", flush=True)
    plan.compress(xd, blob, ws)
    info = plan.info(blob, check=False)
    assert info.return_status == tsq.TSQ_ERR_FORMAT and info.status == tsq.TSQ_ERR_FORMAT
    assert bool((ws == 0xFF).all())
    # a smaller plan's workspace
    small = tsq.Plan(200, H, "f16", 8.0, (2, 3, 4, 6, 8), 0.05, pipeline=pipeline)
    ws2 = small.new_workspace()
    torch.cuda.synchronize()
    before = ws2.clone()
    print("compress on the workspace of a 200-token plan", flush=True)
    plan.compress(xd, blob, ws2)
    assert plan.info(blob, check=False).return_status == tsq.TSQ_ERR_FORMAT
    assert torch.equal(ws2, before)
    out = torch.full((T, H), 0x1234, dtype=torch.int16, device="cuda")
    plan.decompress(blob, out)                              # refused: the output stays as it was
    torch.cuda.synchronize()
    assert bool((out == 0x1234).all())
    ref = oracle.compress(x[:200], oracle.F16, 8.0, (2, 3, 4, 6, 8), 0.05, 1)
    b2 = small.compress(xd[:200].contiguous(), None, ws2)
    assert small.info(b2).status == 0
    sec = small.sections(b2)
    for k in SECTIONS:
        assert np.array_equal(sec[k], getattr(ref, k)), k


def test_a_failed_workspace_stays_failed_until_it_is_reset(tsq, oracle):
    """The error word of a workspace set by hand (as a call whose wait expired leaves it): every call on it,
    also on a blob that still holds a good header from before, ends with TSQ_ERR_INTERNAL; the blocking call
    with TSQ_PIPE_AUTO resets the workspace and compresses again with the staged kernels."""
    import torch
    x = synth.make_c2(tokens=900)
    T, H = x.shape
    ref = oracle.compress(x, oracle.F16, 8.0, (2, 3, 4, 6, 8), 0.05, 1, nthreads=8)
    plan = tsq.Plan(T, H, "f16", 8.0, (2, 3, 4, 6, 8), 0.05, pipeline="auto")
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    ws = plan.new_workspace()
    blob = plan.compress(xd, None, ws)
    assert plan.info(blob).status == 0                      # a good header is in the blob now
    ws.view(torch.int32)[CTL_ERROR] = 1
    for i in range(2):
        print("call %d on the failed workspace" % i, flush=True)
        plan.compress(xd, blob, ws)
        info = plan.info(blob, check=False)
        assert info.return_status == tsq.TSQ_ERR_INTERNAL and info.status == tsq.TSQ_ERR_INTERNAL
    print("the blocking call", flush=True)
    info = tsq.tsq_compress_blocking(plan.handle, xd.data_ptr(), blob.data_ptr(), ws.data_ptr(), plan._stream())
    assert info.return_status == tsq.TSQ_OK and info.status == 0 and info.nnz == ref.nnz
    sec = plan.sections(blob)
    for k in SECTIONS:
        assert np.array_equal(sec[k], getattr(ref, k)), k
    # the workspace is usable again by the ordinary call
    blob.zero_()
    plan.compress(xd, blob, ws)
    assert plan.info(blob).status == 0
    assert np.array_equal(plan.sections(blob)["payload"], ref.payload)
    # the blocking call on a workspace that was never reset
    ws.fill_(0xFF)
    info = tsq.tsq_compress_blocking(plan.handle, xd.data_ptr(), blob.data_ptr(), ws.data_ptr(), plan._stream())
    assert info.return_status == tsq.TSQ_OK and np.array_equal(plan.sections(blob)["payload"], ref.payload)
    # a plan that insists on the single pass gets the error, not the second try
    fused = tsq.Plan(T, H, "f16", 8.0, (2, 3, 4, 6, 8), 0.05, pipeline="fused")
    ws.view(torch.int32)[CTL_ERROR] = 1
    info = tsq.tsq_compress_blocking(fused.handle, xd.data_ptr(), blob.data_ptr(), ws.data_ptr(), plan._stream(), check=False)
    assert info.return_status == tsq.TSQ_ERR_INTERNAL


def test_a_workspace_in_an_arbitrary_state_is_reported_and_recovers(tsq, oracle):
    """A workspace of all-ones bytes behind a control block that carries the right shape: the error word is
    set, the table words carry no valid tag and the ticket counters wrap around.  Every token index the kernel
    forms from them is still checked against the token count, and every store against its section, so the
    call runs to its end and says TSQ_ERR_INTERNAL; after a reset the same buffers give the oracle's blob."""
    import torch
    x = synth.make_c2(tokens=3000)                         # more tokens than workgroups: tickets are drawn
    T, H = x.shape
    ref = oracle.compress(x, oracle.F16, 8.0, (2, 3, 4, 6, 8), 0.05, 1, nthreads=8)
    plan = tsq.Plan(T, H, "f16", 8.0, (2, 3, 4, 6, 8), 0.05, pipeline="fused", max_outliers=max(ref.nnz, 1))
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    ws = torch.empty(int(plan.layout.workspace_bytes), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    ws.view(torch.int32)[CTL_TOKENS] = T
    ws.view(torch.int32)[CTL_HIDDEN] = H
    blob = plan.new_blob()
    blob.zero_()
    print("compress on a workspace of all-ones bytes with the right shape in it", flush=True)
    plan.compress(xd, blob, ws)
    info = plan.info(blob, check=False)
    assert info.return_status == tsq.TSQ_ERR_INTERNAL
    # decompress refuses such a blob: the output stays as it was
    out = torch.full((T, H), 0x1234, dtype=torch.int16, device="cuda")
    plan.decompress(blob, out)
    torch.cuda.synchronize()
    assert bool((out == 0x1234).all())

    print("the same call after tsq_workspace_reset", flush=True)
    tsq.tsq_workspace_reset(plan.handle, ws.data_ptr(), 0)
    plan.compress(xd, blob, ws)
    assert plan.info(blob).status == 0
    sec = plan.sections(blob)
    for k in SECTIONS:
        assert np.array_equal(sec[k], getattr(ref, k)), k
    assert np.array_equal(sec["scale"].view(np.uint32), ref.scale.view(np.uint32))
    # and once more, without a reset in between: a completed call leaves the workspace ready
    blob.zero_()
    plan.compress(xd, blob, ws)
    assert plan.info(blob).status == 0
    assert np.array_equal(plan.sections(blob)["payload"], ref.payload)


def test_a_damaged_eblob_is_decoded_to_the_end_and_touches_only_the_payload(tsq, oracle):
    """Tables, stream bytes and stream offsets of a valid eblob overwritten with noise: the decoder
    checks every offset against the stream capacity, reads past a stream's end as zeros and keeps
    every table index inside its table, so it writes (wrong) codes into the payload section and
    nothing else.  What is compared is everything outside the payload section."""
    import torch
    x = synth.make_c4(tokens=300)
    T, H = x.shape
    w = synth.WORKLOADS["C4"]
    plan = tsq.Plan(T, H, w.dtype, w.tau, w.bit_set, 0.05)
    blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    assert plan.info(blob).status == 0
    eblob = plan.entropy_encode(blob)
    info = plan.entropy_sections(eblob)["info"]
    L = plan.layout
    lo, hi = int(L.off_payload), int(L.off_payload) + int(L.payload_capacity)
    before = blob.cpu().numpy().copy()
    g = torch.Generator(device="cuda")
    g.manual_seed(7)

    def noise(n):
        return torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda", generator=g)

    cases = {"tables": (int(info.off_tables), 7 * 512),
             "streams": (int(info.off_streams), int(info.stream_bytes)),
             "offsets": (int(info.off_stream_off), 8 * (T + 1))}
    for name, (at, n) in cases.items():
        print("decode with noise in the", name, flush=True)
        bad = eblob.clone()
        bad[at: at + n] = noise(n)
        work = blob.clone()
        plan.entropy_decode(bad, work)
        torch.cuda.synchronize()
        after = work.cpu().numpy()
        assert np.array_equal(after[:lo], before[:lo]) and np.array_equal(after[hi:], before[hi:]), name
    # the undamaged eblob still restores the payload
    work = blob.clone()
    work[lo:hi] = 0
    plan.entropy_decode(eblob, work)
    assert np.array_equal(plan.sections(work)["payload"], plan.sections(blob)["payload"])


def test_a_damaged_blob_is_decompressed_without_leaving_its_sections(tsq, oracle):
    """Widths, payload offsets, CSR row pointers and columns of a valid blob overwritten (with noise,
    and with offsets just below 2^64, which would wrap if they were added to a length before being
    compared): every token is either restored from inside the sections or skipped.  The tokens whose
    metadata stayed intact must still come out as the oracle restores them."""
    import torch
    x = synth.make_c4(tokens=300)
    T, H = x.shape
    w = synth.WORKLOADS["C4"]
    ref = oracle.compress(x, oracle.BF16, w.tau, w.bit_set, 0.05, 1, nthreads=8)
    want = oracle.decompress(ref, nthreads=8)
    plan = tsq.Plan(T, H, w.dtype, w.tau, w.bit_set, 0.05, max_outliers=max(ref.nnz, 1))
    blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    assert plan.info(blob).status == 0
    L = plan.layout
    g = np.random.Generator(np.random.PCG64(99))

    def run(name, at, raw_bytes, intact):
        print("decompress with a damaged", name, flush=True)
        bad = blob.clone()
        bad[at: at + len(raw_bytes)] = torch.from_numpy(raw_bytes).cuda()
        out = torch.full((T, H), 0x1234, dtype=torch.int16, device="cuda")
        plan.decompress(bad, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(np.uint16)
        for t in intact:
            assert np.array_equal(got[t], want[t]), (name, t)

    # token 7's payload offset just below 2^64; all other tokens untouched
    po = plan.sections(blob)["pay_off"].copy()
    po[7] = np.uint64(2 ** 64 - 4)
    run("payload offset (wrapping)", int(L.off_pay_off), po.view(np.uint8), [t for t in range(T) if t != 7])
    po[7] = np.uint64(2 ** 64 - 8192)
    run("payload offset (wrapping by a row)", int(L.off_pay_off), po.view(np.uint8), [0, 6, 8, T - 1])
    run("payload offsets (noise)", int(L.off_pay_off), g.integers(0, 256, 8 * (T + 1), dtype=np.uint8), [])
    run("widths (noise)", int(L.off_bits), g.integers(0, 256, T, dtype=np.uint8), [])
    # row pointers: noise in the upper half of the tokens (a pointer pair that is out of order or beyond
    # the capacity skips the token), columns: noise everywhere (a column beyond the row is ignored)
    rp = plan.sections(blob)["row_ptr"].copy()
    rp[T // 2:] = g.integers(0, 2 ** 63, T + 1 - T // 2, dtype=np.uint64)
    run("row pointers (noise)", int(L.off_row_ptr), rp.view(np.uint8), list(range(0, T // 2 - 1)))
    run("columns (noise)", int(L.off_out_col), g.integers(0, 256, 2 * max(ref.nnz, 1), dtype=np.uint8), [])


def test_calls_that_alternate_between_two_streams_do_not_stall_each_other(tsq, oracle):
    """Two single-pass kernels that shared the device could hold the compute units that the other one's
    workgroups still needed, until their bounded waits expired; the library therefore orders such calls.
    Many short calls, alternating between two streams with a workspace each: every blob complete and
    equal to the oracle's."""
    import torch
    x = synth.make_c2(tokens=2048)
    T, H = x.shape
    ref = oracle.compress(x, oracle.F16, 8.0, (2, 3, 4, 6, 8), 0.05, 1, nthreads=8)
    plan = tsq.Plan(T, H, "f16", 8.0, (2, 3, 4, 6, 8), 0.05, pipeline="fused", max_outliers=max(ref.nnz, 1))
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    lanes = [(torch.cuda.Stream(), plan.new_workspace(), [plan.new_blob() for _ in range(2)], plan.new_output())
             for _ in range(2)]
    torch.cuda.synchronize()
    for i in range(600):
        stream, ws, blobs, out = lanes[i % 2]
        with torch.cuda.stream(stream):
            plan.compress(xd, blobs[(i // 2) % 2], ws)
            plan.decompress(blobs[(i // 2) % 2], out)
        if i % 100 == 99:
            print("step", i, flush=True)
    torch.cuda.synchronize()
    for _, _, blobs, out in lanes:
        for b in blobs:
            assert plan.info(b).status == 0
            assert np.array_equal(plan.sections(b)["payload"], ref.payload)
        assert np.array_equal(out.cpu().numpy().view(np.uint16), oracle.decompress(ref, nthreads=8))


@pytest.mark.parametrize("shape", ["C2", "C4 rows"])
def test_a_decompress_stream_behind_a_compress_stream(tsq, oracle, shape):
    """The launch pattern that bench.py calls two streams: every compress call on one stream, every decompress
    call on a second one, behind its compress call by an event, a blob written again only after the call that
    read it.  A step's restore kernel then runs beside the next step's single-pass kernel, whose workgroups
    wait for one another; many steps, different inputs per buffer set, every output equal to the oracle's."""
    import torch
    if shape == "C2":
        base, dtype, tau, bits, odt = synth.make_c2(tokens=2048), "f16", 8.0, (2, 3, 4, 6, 8), oracle.F16
    else:
        base, dtype, tau, bits, odt = synth.make_c4(tokens=1536), "bf16", 10.0, (2, 3, 4, 5, 6, 8), oracle.BF16
    T, H = base.shape
    nset = 3
    xs = [np.ascontiguousarray(np.roll(base, 7 * k, axis=0)) for k in range(nset)]     # a tensor of its own per set
    refs = [oracle.compress(x, odt, tau, bits, 0.05, 1, nthreads=8) for x in xs]
    plan = tsq.Plan(T, H, dtype, tau, bits, 0.05, pipeline="fused", max_outliers=max(max(r.nnz for r in refs), 1))
    xd = [torch.from_numpy(x.view(np.int16)).cuda() for x in xs]
    blobs, outs, ws = [plan.new_blob() for _ in range(nset)], [plan.new_output() for _ in range(nset)], plan.new_workspace()
    first, second = torch.cuda.Stream(), torch.cuda.Stream()
    written, read = [torch.cuda.Event() for _ in range(nset)], [torch.cuda.Event() for _ in range(nset)]
    torch.cuda.synchronize()
    steps = 300
    for i in range(steps):
        k = i % nset
        with torch.cuda.stream(first):
            if i >= nset:
                first.wait_event(read[k])
            plan.compress(xd[k], blobs[k], ws)
            written[k].record(first)
        with torch.cuda.stream(second):
            second.wait_event(written[k])
            plan.decompress(blobs[k], outs[k])
            read[k].record(second)
        if i % 100 == 99:
            print("step", i, flush=True)
    torch.cuda.synchronize()
    for k in range(nset):
        assert plan.info(blobs[k]).status == 0
        sec = plan.sections(blobs[k])
        assert np.array_equal(sec["payload"], refs[k].payload) and np.array_equal(sec["out_col"], refs[k].out_col)
        assert np.array_equal(outs[k].cpu().numpy().view(np.uint16), oracle.decompress(refs[k], nthreads=8))
