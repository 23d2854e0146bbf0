"""Parity of the rANS stage (tsq_entropy_encode / tsq_entropy_decode) with its oracle: tables,
stream offsets and stream bytes bit-exact; decode restores the payload byte for byte."""
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
def RE(oracle):
    from oracle import entropy_oracle, rans_oracle
    return rans_oracle, entropy_oracle


def check(tsq, oracle, RE, x, dtype, tau, bit_set, budget, mode=1, label=""):
    import torch
    R, E = RE
    print("case", label, x.shape, dtype, tau, bit_set, budget, flush=True)
    T, H = x.shape
    ref = oracle.compress(x, DT[dtype], tau, bit_set, budget, mode, nthreads=8)
    tables, off, streams = R.encode(ref, E.code_histogram(ref))

    plan = tsq.Plan(T, H, dtype, tau, bit_set, budget, mode="rel_rms" if mode == 1 else "lsb",
                    max_outliers=max(ref.nnz, 1))
    blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    assert plan.info(blob).status == 0
    eblob = plan.new_entropy_blob()
    eblob.fill_(0xA5)
    plan.entropy_encode(blob, eblob)
    sec = plan.entropy_sections(eblob)
    assert np.array_equal(sec["tables"], tables), "tables"
    assert np.array_equal(sec["stream_off"], off), "stream offsets"
    assert sec["info"].stream_bytes == len(streams)
    assert sec["streams"].tobytes() == streams, "streams"
    assert sec["info"].coded_bytes == 256 + 7 * 512 + 8 * (T + 1) + len(streams)

    # decode into a blob whose payload section has been wiped
    L = plan.layout
    blob2 = blob.clone()
    blob2[int(L.off_payload): int(L.off_payload) + int(L.payload_capacity)] = 0xEE
    plan.entropy_decode(eblob, blob2)
    a, b = plan.sections(blob), plan.sections(blob2)
    assert np.array_equal(a["payload"], b["payload"]) and np.array_equal(a["payload"], ref.payload)
    out = plan.decompress(blob2)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), oracle.decompress(ref, nthreads=8))
    return ref, len(streams)


def test_c1_and_mixed_widths(tsq, oracle, RE):
    for eps in (0.05, 0.1, 0.3):
        check(tsq, oracle, RE, synth.make_c1(), "f16", 6.0, (2, 4, 8), eps, label="C1")
    ref, n = check(tsq, oracle, RE, synth.make_c2(tokens=128), "f16", 8.0, (2, 3, 4, 6, 8), 0.2, label="C2 rows")
    assert len(set(ref.bits.tolist())) >= 2
    assert n < ref.payload_bytes                    # the coder pays: fewer bytes than the packed payload


def test_c4_rows_every_width(tsq, oracle, RE):
    x = synth.make_c4(tokens=96)
    seen = set()
    for bs, eps in (((2, 3, 4, 5, 6, 8), 0.05), ((2, 3, 4, 5, 6, 8), 0.2), ((7,), 0.0), ((2, 3), 0.0)):
        ref, _ = check(tsq, oracle, RE, x, "bf16", 10.0, bs, eps, label="C4 rows")
        seen |= set(ref.bits.tolist())
    assert seen >= {2, 3, 4, 5, 6, 7, 8}


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H", [8, 24, 40, 264, 1000, 2056, 4096 + 8])
def test_edge_rows_and_ragged_hidden(tsq, oracle, RE, dtype, H):
    x = synth.edge_rows(H, dtype, 6.0) if H >= 264 else None
    if x is None:
        g = np.random.Generator(np.random.PCG64(H))
        v = g.standard_normal((37, H)) * 3.0
        x = synth.to_f16_bits(v) if dtype == "f16" else synth.to_bf16_bits(v)
    for bs, bud, mode in (((2, 4, 5, 8), 0.05, 1), ((2, 3, 4, 5, 6, 7, 8), 0.3, 0)):
        check(tsq, oracle, RE, x, dtype, 6.0, bs, bud, mode, label="edge H=%d" % H)


@pytest.mark.parametrize("H", [8192 + 264, 16384 + 24, 32768])
def test_rows_of_more_than_four_runs_per_lane(tsq, oracle, RE, H):
    """Rows beyond 8192 elements: the counting kernel takes a lane's runs four at a time and goes round more
    than once, the coders and the gather loop further than on any benchmarked shape; the longest row the
    library takes is among them."""
    g = np.random.Generator(np.random.PCG64(H))
    v = g.standard_t(4, size=(5, H)) * g.lognormal(0.0, 0.6, (5, 1)) * 2.0
    check(tsq, oracle, RE, synth.to_bf16_bits(v), "bf16", 10.0, (2, 3, 5, 8), 0.1, label="long rows H=%d" % H)
    check(tsq, oracle, RE, synth.to_f16_bits(v), "f16", 6.0, (4, 7), 0.3, 0, label="long rows H=%d" % H)


@pytest.mark.parametrize("seed", range(3))
def test_random_configurations(tsq, oracle, RE, seed):
    g = np.random.Generator(np.random.PCG64(2000 + seed))
    for k in range(6):
        H = 8 * int(g.integers(1, 300))
        T = int(g.integers(1, 60))
        dtype = ("f16", "bf16")[int(g.integers(0, 2))]
        widths = sorted(set(int(b) for b in g.choice(np.arange(2, 9), size=int(g.integers(1, 8)))))
        budget = float(g.choice([0.0, 0.05, 0.1, 0.2, 0.5]))
        v = g.standard_t(4, size=(T, H)) * 10.0 ** g.uniform(-2, 1) * g.lognormal(0.0, 0.6, (T, 1))
        if g.random() < 0.3:
            v[g.random((T, H)) < 0.4] = 0.0
        x = synth.to_f16_bits(v) if dtype == "f16" else synth.to_bf16_bits(v)
        check(tsq, oracle, RE, x, dtype, float(g.choice([2.0, 6.0, 50.0])), widths, budget, label="random %d.%d" % (seed, k))


@pytest.mark.parametrize("T,H", [(1000, 96), (5000, 32)])
def test_many_tokens_ending_inside_a_block_of_offsets(tsq, oracle, RE, T, H):
    """Token counts that are not multiples of the 256 tokens whose stream lengths are summed together,
    and more tokens than counting workgroups."""
    g = np.random.Generator(np.random.PCG64(77 + T))
    v = g.standard_t(4, size=(T, H)) * g.lognormal(0.0, 0.8, (T, 1))
    check(tsq, oracle, RE, synth.to_f16_bits(v), "f16", 6.0, (2, 3, 4, 6, 8), 0.1, label="%d tokens" % T)


def test_more_tokens_than_the_counting_kernel_takes_in_one_go(tsq, oracle, RE):
    """100000 tokens of 8 elements: every counting workgroup goes through its tokens in several
    portions.  The oracle codes a token in Python, so tables and offsets are compared in full (the
    offsets against the lengths the oracle's coder gives for sampled tokens and against each other),
    streams on sampled tokens, and the payload must come back byte for byte."""
    import torch
    R, E = RE
    T, H = 100000, 8
    g = np.random.Generator(np.random.PCG64(4242))
    v = g.standard_t(4, size=(T, H)) * g.lognormal(0.0, 0.8, (T, 1))
    x = synth.to_f16_bits(v)
    ref = oracle.compress(x, 0, 6.0, (2, 3, 4, 6, 8), 0.1, 1, nthreads=8)
    tables = R.class_tables(E.code_histogram(ref), ref.bits)
    plan = tsq.Plan(T, H, "f16", 6.0, (2, 3, 4, 6, 8), 0.1, max_outliers=max(ref.nnz, 1))
    blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    assert plan.info(blob).status == 0
    eblob = plan.entropy_encode(blob)
    sec = plan.entropy_sections(eblob)
    assert np.array_equal(sec["tables"], tables), "tables"
    off = sec["stream_off"].astype(np.int64)
    # one coder per token here (one run): a stream is its state and at most 8 words, padded to 4 bytes
    d = np.diff(off)
    assert off[0] == 0 and np.all(d >= 4) and np.all(d <= 4 + 16) and np.all(d % 4 == 0)
    assert int(off[-1]) == sec["info"].stream_bytes
    for t in sorted(set(g.integers(0, T, 300).tolist()) | {0, 255, 256, 257, T - 1}):
        want = R.encode_token(E.token_codes(ref, t), tables[int(ref.bits[t]) - 2])
        assert sec["streams"][int(off[t]): int(off[t + 1])].tobytes() == want, "token %d" % t
    L = plan.layout
    blob2 = blob.clone()
    blob2[int(L.off_payload): int(L.off_payload) + int(L.payload_capacity)] = 0
    plan.entropy_decode(eblob, blob2)
    assert np.array_equal(plan.sections(blob2)["payload"], ref.payload)


def test_the_blob_of_a_batch_call(tsq, oracle, RE):
    """The stage takes any blob of the plan: here the one that the batch form writes for the key and value
    tensors of a KV cache (one blob for all of them), against the oracle on the concatenated tensor."""
    import torch
    R, E = RE
    parts = synth.make_kv("KV7", layers=3, rows=40)
    w = synth.WORKLOADS["KV7"]
    x = np.concatenate(parts)
    T, H = x.shape
    ref = oracle.compress(x, DT[w.dtype], w.tau, w.bit_set, 0.1, 1, nthreads=8)
    tables, off, streams = R.encode(ref, E.code_histogram(ref))
    plan = tsq.Plan(T, H, w.dtype, w.tau, w.bit_set, 0.1, max_outliers=max(ref.nnz, 1))
    tensors = [torch.from_numpy(p.view(np.int16)).cuda() for p in parts]
    blob, _table = plan.compress_batch(tensors)
    assert plan.info(blob).status == 0
    eblob = plan.entropy_encode(blob)
    sec = plan.entropy_sections(eblob)
    assert np.array_equal(sec["tables"], tables) and np.array_equal(sec["stream_off"], off)
    assert sec["streams"].tobytes() == streams
    L = plan.layout
    blob2 = blob.clone()
    blob2[int(L.off_payload): int(L.off_payload) + int(L.payload_capacity)] = 0x5A
    plan.entropy_decode(eblob, blob2)
    outs = [torch.empty_like(t) for t in tensors]
    plan.decompress_batch(blob2, outs)
    want = oracle.decompress(ref, nthreads=8)
    got = np.concatenate([o.cpu().numpy().view(np.uint16) for o in outs])
    assert np.array_equal(got, want)


def test_a_foreign_blob_gives_no_valid_eblob(tsq):
    import torch
    plan = tsq.Plan(16, 64, "f16", 6.0, (4, 8), 0.05)
    blob = plan.new_blob()
    blob.zero_()
    eblob = plan.entropy_encode(blob)
    info = tsq.tsq_entropy_info(plan.handle, eblob.data_ptr(), 0, check=False)
    assert info.return_status == tsq.TSQ_ERR_FORMAT
    # and decode of a foreign eblob leaves the blob alone
    x = torch.from_numpy(synth.to_f16_bits(np.ones((16, 64))).view(np.int16)).cuda()
    good = plan.compress(x)
    before = good.clone()
    plan.entropy_decode(eblob, good)
    torch.cuda.synchronize()
    assert torch.equal(before, good)


def test_c4_full_size_every_stream_and_round_trip(tsq, oracle, RE):
    """The full target tensor in the launch configuration that is timed: tables, offsets and the streams of
    all 8192 tokens against the oracle (its compiled coder, which the Python coder pins), and the round trip
    of the whole payload."""
    import torch
    R, E = RE
    w = synth.WORKLOADS["C4"]
    x = synth.make_c4()
    T, H = x.shape
    ref = oracle.compress(x, oracle.BF16, w.tau, w.bit_set, 0.05, 1, nthreads=8)
    print("oracle: codes and counts of %d tokens" % T, flush=True)
    codes = np.empty((T, H), np.uint8)
    hist = np.zeros((T, 256), np.uint32)
    for t in range(T):
        codes[t] = E.token_codes(ref, t)
        hist[t] = np.bincount(codes[t], minlength=256)
    tables = R.class_tables(hist, ref.bits)
    print("oracle: streams", flush=True)
    want_off, want_streams = R.encode_codes_c(codes, ref.bits, tables)
    # the compiled coder against the Python one on a few tokens of this very tensor
    for t in (0, 4097, T - 1):
        a, b = int(want_off[t]), int(want_off[t + 1])
        assert want_streams[a:b].tobytes() == R.encode_token(codes[t], tables[int(ref.bits[t]) - 2])
    plan = tsq.Plan(T, H, w.dtype, w.tau, w.bit_set, 0.05, max_outliers=max(ref.nnz, 1))
    blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    eblob = plan.entropy_encode(blob)
    sec = plan.entropy_sections(eblob)
    assert np.array_equal(sec["tables"], tables)
    assert np.array_equal(sec["stream_off"], want_off), "stream offsets"
    assert int(want_off[-1]) == sec["info"].stream_bytes
    assert np.array_equal(sec["streams"], want_streams), "streams"
    L = plan.layout
    blob2 = blob.clone()
    blob2[int(L.off_payload): int(L.off_payload) + int(L.payload_capacity)] = 0
    plan.entropy_decode(eblob, blob2)
    assert np.array_equal(plan.sections(blob2)["payload"], ref.payload)
    assert sec["info"].stream_bytes < 0.85 * ref.payload_bytes
