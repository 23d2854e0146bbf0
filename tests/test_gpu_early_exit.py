"""The early-exit driver end to end: sizes measured on the GPU, decisions by the library, checked
against the ladder written out in the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_decisions_from_measured_sizes_follow_the_ladder(oracle):
    import torch
    assert torch.cuda.is_available()
    from oracle import link_oracle as LO
    from paper_2511_04002_amd import early_exit, synth, tsq
    tokens, layers = 96, 3
    raw, with_kv, pre = early_exit.measure(tokens, layers)
    # the sizes are the oracle's sizes: hidden state, then the cache as one concatenated tensor
    w2, wk = synth.WORKLOADS["C2"], synth.WORKLOADS["KV7"]
    ch = oracle.compress(synth.make_c2(tokens=tokens), oracle.F16, w2.tau, w2.bit_set, 0.05, 1)
    ck = oracle.compress(np.concatenate(synth.make_kv("KV7", layers=layers, rows=tokens)), oracle.F16, wk.tau,
                         wk.bit_set, 0.05, 1)
    assert pre[-1] == 8 * oracle.compressed_bytes(ch)
    assert with_kv == 8.0 * (oracle.compressed_bytes(ch) + oracle.compressed_bytes(ck))
    assert pre[0] == 8 * (128 + 16) and all(b > a for a, b in zip(pre, pre[1:]))
    assert raw > with_kv > pre[-1]
    W, gamma, eps = 10e6, 10.0, 1e-3
    link = tsq.tsq_link(W, gamma, eps)
    rate = tsq.tsq_link_best_rate(link, 1e5, 1e8, 2000)
    lc = [0.0] + [0.01 + 0.001 * k for k in range(1, tokens + 1)]
    seen = set()
    for D in (1e4, 100.0, 30.0, 10.0, 3.0, 1.0, 0.3, 0.1, 0.03, 0.0):
        got = tsq.tsq_early_exit_decide(link, rate, D, lc, raw, with_kv, pre)
        want = LO.early_exit(W, gamma, eps, rate, D, lc, raw, with_kv, pre)
        assert (got.action, got.with_kv, got.tokens) == want[:3]
        assert got.latency == pytest.approx(want[3], rel=1e-12)
        seen.add(got.action)
    assert len(seen) >= 3


def test_prefix_sizes_are_those_of_the_shorter_tensor(oracle):
    """tsq_prefix_bytes(k) is what compressing the first k tokens alone reports, for every k."""
    import torch
    from paper_2511_04002_amd import synth, tsq
    w2 = synth.WORKLOADS["C2"]
    tokens = 40
    x = synth.make_c2(tokens=tokens)
    plan = tsq.Plan(tokens, w2.hidden, w2.dtype, w2.tau, w2.bit_set, 0.2, max_outliers=tokens * w2.hidden // 8)
    blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    pre = plan.prefix_bytes(blob)
    assert len(pre) == tokens + 1 and pre[0] == 128 + 16
    for k in (1, 2, 7, 39, 40):
        c = oracle.compress(x[:k], oracle.F16, w2.tau, w2.bit_set, 0.2, 1)
        assert pre[k] == oracle.compressed_bytes(c)
    assert plan.prefix_bytes(blob, [40, 0, 7]) == [pre[40], pre[0], pre[7]]
    assert pre[tokens] == plan.info(blob).compressed_bytes
    with pytest.raises(tsq.TsqError):
        plan.prefix_bytes(blob, [41])


def test_walk_with_sizes_measured_step_by_step(oracle):
    """Algorithm 2 with both loops: the library's walk over sizes that the GPU measures at the steps that need
    them, against the oracle's walk over sizes that the oracle compresses."""
    from oracle import link_oracle as LO
    from paper_2511_04002_amd import early_exit, synth, tsq
    max_tokens, layers = 12, 3
    sizes = early_exit.StepSizes(max_tokens, layers)
    w2, wk = synth.WORKLOADS["C2"], synth.WORKLOADS["KV7"]
    hid = synth.make_c2(tokens=max_tokens)
    kv = synth.make_kv("KV7", layers=layers, rows=max_tokens)
    memo = {}

    def oracle_bits(w, layer, with_kv, compressed, keep):
        if not compressed:
            return 16.0 * (keep * w2.hidden + (2 * layer * w * w2.hidden if with_kv else 0))
        key = (w, layer, with_kv, keep)
        if key not in memo:
            c = oracle.compress(hid[:w], oracle.F16, w2.tau, w2.bit_set, 0.05, 1)
            # first `keep` tokens of the w-token blob: header + metadata + their codes + their CSR entries
            b = 128 + 5 * keep + 16 * (keep + 1) + int(c.pay_off[keep]) + 4 * int(c.row_ptr[keep])
            if with_kv:
                ck = oracle.compress(np.concatenate([t[:w] for t in kv[: 2 * layer]]), oracle.F16, wk.tau, wk.bit_set,
                                     0.05, 1)
                b += oracle.compressed_bytes(ck)
            memo[key] = 8.0 * b
        return memo[key]

    W, gamma, eps = 10e6, 10.0, 1e-3
    link = tsq.tsq_link(W, gamma, eps)
    rate = tsq.tsq_link_best_rate(link, 1e5, 1e8, 2000)

    def lc(w, layer):
        return (0.002 + 0.0005 * w) * layer if w else 0.0
    seen = set()
    for D in (10.0, 1.0, 0.5, 0.2, 0.1, 0.05, 0.03, 0.02, 0.01, 0.003):
        got = tsq.tsq_early_exit_walk(link, rate, D, max_tokens, layers, lc, sizes.bits)
        want = LO.early_exit_walk(W, gamma, eps, rate, D, max_tokens, layers, lc, oracle_bits)
        assert (got.action, got.with_kv, got.tokens, got.layer, got.sent_tokens) == want[:5], D
        assert got.latency == pytest.approx(want[5], rel=1e-12)
        seen.add(got.action)
    assert len(seen) >= 2 and sizes.compress_calls > 0


def test_prefix_sizes_with_the_codes_entropy_coded(oracle):
    """tsq_entropy_prefix_bytes(k): the blob's metadata and CSR entries of k tokens, and in place of their codes
    the coded blob's header, tables, k + 1 offsets and the first k streams, counted here from the byte strings
    that the oracle's coder gives; for k = tokens it is the blob's size with the payload swapped for the coded
    blob."""
    import torch
    from oracle import entropy_oracle as E, rans_oracle as R
    from paper_2511_04002_amd import synth, tsq
    w2 = synth.WORKLOADS["C2"]
    tokens = 24
    x = synth.make_c2(tokens=tokens)
    ref = oracle.compress(x, oracle.F16, w2.tau, w2.bit_set, 0.1, 1)
    hist = E.code_histogram(ref)
    tables = R.class_tables(hist, ref.bits)
    streams = [R.encode_token(E.token_codes(ref, t), tables[int(ref.bits[t]) - 2]) for t in range(tokens)]
    plan = tsq.Plan(tokens, w2.hidden, w2.dtype, w2.tau, w2.bit_set, 0.1, max_outliers=tokens * w2.hidden // 8)
    blob = plan.compress(torch.from_numpy(x.view(np.int16)).cuda())
    eblob = plan.entropy_encode(blob)
    got = plan.entropy_prefix_bytes(blob, eblob)
    assert len(got) == tokens + 1
    for k in range(tokens + 1):
        padded = sum((len(s) + 3) // 4 * 4 for s in streams[:k])
        coded = 256 + tables.nbytes + 8 * (k + 1) + padded
        assert tables.nbytes == 7 * 512
        assert got[k] == 128 + 5 * k + 16 * (k + 1) + 4 * int(ref.row_ptr[k]) + coded, k
    info = plan.info(blob)
    einfo = tsq.tsq_entropy_info(plan.handle, eblob.data_ptr(), plan._stream())
    assert got[tokens] == info.compressed_bytes - info.payload_bytes + einfo.coded_bytes
    assert got[tokens] < info.compressed_bytes                       # the stage pays on this tensor
    assert plan.entropy_prefix_bytes(blob, eblob, [tokens, 0, 5]) == [got[tokens], got[0], got[5]]
    with pytest.raises(tsq.TsqError):
        plan.entropy_prefix_bytes(blob, eblob, [tokens + 1])
    with pytest.raises(tsq.TsqError):
        plan.entropy_prefix_bytes(blob, blob, [1])                   # not a coded blob


def test_decisions_with_entropy_coded_sizes_follow_the_ladder(oracle):
    from oracle import link_oracle as LO
    from paper_2511_04002_amd import early_exit, tsq
    tokens, layers = 48, 2
    raw, with_kv, pre = early_exit.measure(tokens, layers, entropy=True)
    raw0, with_kv0, pre0 = early_exit.measure(tokens, layers)
    assert raw == raw0 and with_kv < with_kv0 and pre[-1] < pre0[-1]
    assert all(b > a for a, b in zip(pre, pre[1:]))
    W, gamma, eps = 10e6, 10.0, 1e-3
    link = tsq.tsq_link(W, gamma, eps)
    rate = tsq.tsq_link_best_rate(link, 1e5, 1e8, 2000)
    lc = [0.0] + [0.01 + 0.001 * k for k in range(1, tokens + 1)]
    for D in (1e3, 10.0, 1.0, 0.3, 0.1, 0.03, 0.0):
        got = tsq.tsq_early_exit_decide(link, rate, D, lc, raw, with_kv, pre)
        want = LO.early_exit(W, gamma, eps, rate, D, lc, raw, with_kv, pre)
        assert (got.action, got.with_kv, got.tokens) == want[:3]
