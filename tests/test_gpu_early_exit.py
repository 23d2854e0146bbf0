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
