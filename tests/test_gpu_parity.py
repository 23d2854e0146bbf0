"""Parity of the HIP path with the CPU oracle, through the C ABI.

Bar: bit-exact widths, scales, offsets, CSR columns / values and packed bytes;
decoded values bit-exact as well (the stated tolerance is 1e-6 relative in fp32
arithmetic; decode is one exact integer->float conversion, one fp32 multiply and
one round-to-nearest-even store, so both sides agree to the bit and the test
asserts that, after asserting the stated tolerance).
"""
import numpy as np
import pytest

from paper_2511_04002_amd import synth

pytestmark = pytest.mark.gpu

F16, BF16 = 0, 1
DT = {"f16": F16, "bf16": BF16}
MODE = {"lsb": 0, "rel_rms": 1}
PIPELINES = ["fused", "staged"]


@pytest.fixture(scope="module")
def tsq():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_04002_amd import tsq as m
    m.lib()                                   # fails loudly if libtsq.so is missing
    return m


def widen(raw, dt):
    if dt == F16:
        return raw.view(np.float16).astype(np.float32)
    return (raw.astype(np.uint32) << 16).view(np.float32)


def check_parity(tsq, oracle, x, dtype, tau, bit_set, budget, mode="rel_rms", pipeline="staged",
                 max_outliers=0, label="", rule="last_passing"):
    import torch
    print("case", label, x.shape, dtype, tau, bit_set, budget, mode, pipeline, rule, flush=True)
    T, H = x.shape
    ref = oracle.compress(x, DT[dtype], tau, bit_set, budget, MODE[mode], nthreads=8,
                          rule=oracle.RETURN_AS_PRINTED if rule == "as_printed" else oracle.RETURN_LAST_PASSING)
    ref_out = oracle.decompress(ref, nthreads=8)

    plan = tsq.Plan(T, H, dtype, tau, bit_set, budget, mode=mode, pipeline=pipeline,
                    max_outliers=max_outliers or max(ref.nnz, 1), return_rule=rule)
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    ws = plan.new_workspace()
    blob = plan.new_blob()
    blob.fill_(0xA5)                                    # stale bytes must not matter
    plan.compress(xd, blob, ws)
    info = plan.info(blob)
    sec = plan.sections(blob)

    assert np.array_equal(sec["bits"], ref.bits), "widths"
    assert np.array_equal(sec["scale"].view(np.uint32), ref.scale.view(np.uint32)), "scales"
    assert np.array_equal(sec["row_ptr"], ref.row_ptr), "row_ptr"
    assert np.array_equal(sec["pay_off"], ref.pay_off), "pay_off"
    assert np.array_equal(sec["out_col"], ref.out_col), "CSR columns"
    assert np.array_equal(sec["out_val"], ref.out_val), "CSR values"
    assert np.array_equal(sec["payload"], ref.payload), "packed bytes"
    assert info.nnz == ref.nnz and info.payload_bytes == ref.payload_bytes and info.status == 0
    assert info.compressed_bytes == oracle.compressed_bytes(ref)
    assert list(info.width_hist) == np.bincount(ref.bits, minlength=9).tolist()

    out = plan.new_output()
    out.fill_(0x5A5A)
    plan.decompress(blob, out)
    got = out.cpu().numpy().view(np.uint16)
    gv, rv = widen(got, DT[dtype]).astype(np.float64), widen(ref_out, DT[dtype]).astype(np.float64)
    fin = np.isfinite(rv)
    assert np.array_equal(np.isfinite(gv), fin)
    assert np.all(np.abs(gv[fin] - rv[fin]) <= 1e-6 * np.abs(rv[fin])), "decoded values, 1e-6 relative"
    assert np.array_equal(got, ref_out), "decoded bits"

    # same input -> same bytes (a second run into a differently pre-filled blob)
    blob2 = plan.new_blob()
    blob2.fill_(0x3C)
    plan.compress(xd, blob2, ws)
    sec2 = plan.sections(blob2)
    for k in ("bits", "scale", "row_ptr", "pay_off", "out_col", "out_val", "payload", "header"):
        assert np.array_equal(sec[k], sec2[k]), "determinism: " + k
    return ref, info


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("budget,mode", [(0.05, "rel_rms"), (0.1, "rel_rms"), (0.2, "lsb"), (0.0, "rel_rms"),
                                         (float("inf"), "lsb")])
def test_c1_tiny(tsq, oracle, pipeline, budget, mode):
    check_parity(tsq, oracle, synth.make_c1(), "f16", 6.0, (2, 4, 8), budget, mode, pipeline, label="C1")


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("eps", [0.05, 0.2])
def test_c2_prefill_7b(tsq, oracle, pipeline, eps):
    ref, _ = check_parity(tsq, oracle, synth.make_c2(), "f16", 8.0, (2, 3, 4, 6, 8), eps, "rel_rms", pipeline,
                          label="C2")
    assert len(set(ref.bits.tolist())) >= 2


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("eps", [0.05, 0.2])
def test_c3_decode_steps(tsq, oracle, pipeline, eps):
    # ten of the 64 decode steps, at the budget the benchmark uses (0.05: every token 8 bits wide) and at
    # the one that mixes widths
    for step in (0, 1, 2, 7, 16, 31, 32, 47, 62, 63):
        check_parity(tsq, oracle, synth.make_c3(step), "f16", 8.0, (2, 4, 8), eps, "rel_rms", pipeline,
                     label="C3 step %d" % step)


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("eps", [0.05, 0.2])
def test_c4_prefill_70b_full_size(tsq, oracle, pipeline, eps):
    ref, _ = check_parity(tsq, oracle, synth.make_c4(), "bf16", 10.0, (2, 3, 4, 5, 6, 8), eps, "rel_rms", pipeline,
                          label="C4")
    assert len(set(ref.bits.tolist())) >= 3


@pytest.mark.parametrize("pipeline", PIPELINES)
def test_algorithm_1_with_its_return_as_printed(tsq, oracle, pipeline):
    """The descent that returns the quantization at the width that failed the test (tsq_config.return_rule =
    TSQ_RETURN_AS_PRINTED) against the oracle's switch of the same name: whole blobs and decoded bits, on the
    five workload shapes, in both budget modes, and on the width sets where the next candidate is far below."""
    changed = 0
    for name, x, dt, tau, bs in (("C1", synth.make_c1(), "f16", 6.0, (2, 4, 8)),
                                 ("C2", synth.make_c2(tokens=700), "f16", 8.0, (2, 3, 4, 6, 8)),
                                 ("C3", synth.make_c3(5), "f16", 8.0, (2, 4, 8)),
                                 ("C4", synth.make_c4(tokens=1100), "bf16", 10.0, (2, 3, 4, 5, 6, 8)),
                                 ("C5", synth.make_c5_seq(3, 300), "bf16", 8.0, (2, 3, 4, 5, 6, 7, 8))):
        for budget, mode in ((0.05, "rel_rms"), (0.2, "rel_rms"), (0.0, "rel_rms"), (0.2, "lsb"), (float("inf"), "lsb")):
            ref, _ = check_parity(tsq, oracle, x, dt, tau, bs, budget, mode, pipeline, label=name + " as printed",
                                  rule="as_printed")
            base = oracle.compress(x, DT[dt], tau, bs, budget, MODE[mode], nthreads=8)
            assert np.all(ref.bits <= base.bits)
            changed += int((ref.bits < base.bits).sum())
    assert changed > 1000
    x = synth.edge_rows(2056, "bf16", 6.0)
    for bs in ((8,), (2, 8), (7, 8), (2, 3, 4, 5, 6, 7, 8)):
        check_parity(tsq, oracle, x, "bf16", 6.0, bs, 0.1, "rel_rms", pipeline, label="edge as printed", rule="as_printed")


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("tau", synth.C5_TAUS)
@pytest.mark.parametrize("bit_set", synth.C5_BIT_SETS)
def test_c5_stress_two_sequences(tsq, oracle, pipeline, tau, bit_set):
    x = np.concatenate([synth.make_c5_seq(0, 1024), synth.make_c5_seq(31, 1024)])
    check_parity(tsq, oracle, x, "bf16", tau, bit_set, 0.05, "rel_rms", pipeline, label="C5 subset")


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H", [8, 24, 32, 40, 264, 1000, 2056, 4096 + 8, 32768])
def test_edge_rows_and_ragged_hidden(tsq, oracle, pipeline, dtype, H):
    x = synth.edge_rows(H, dtype, 6.0) if H >= 264 else None
    if x is None:
        g = np.random.Generator(np.random.PCG64(H))
        v = g.standard_normal((37, H)) * 3.0
        x = synth.to_f16_bits(v) if dtype == "f16" else synth.to_bf16_bits(v)
    for bs, bud, mode in (((2, 4, 5, 8), 0.05, "rel_rms"), ((2, 3, 4, 5, 6, 7, 8), 0.3, "lsb"), ((7,), 0.1, "lsb"),
                          ((3, 6), 0.5, "rel_rms")):
        check_parity(tsq, oracle, x, dtype, 6.0, bs, bud, mode, pipeline, label="edge H=%d" % H)


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_many_absmax_values_exercise_the_divisions(tsq, oracle, pipeline, dtype):
    # one row per absmax pattern: r = Q/amax and s = amax/Q must be correctly rounded for all of them
    g = np.random.Generator(np.random.PCG64(3))
    T, H = 4096, 64
    if dtype == "f16":
        pats = np.linspace(1, 0x7BFF, T).astype(np.uint16)
    else:
        pats = np.concatenate([np.linspace(0x0001, 0x0D80, T // 4), np.linspace(0x0D80, 0x7F7F, T - T // 4)]).astype(np.uint16)
    frac = g.random((T, H))
    x = np.empty((T, H), np.uint16)
    for t in range(T):
        # magnitudes below the row's absmax pattern, random signs, absmax itself at a random slot
        row = (frac[t] * pats[t]).astype(np.uint16)
        row[g.integers(0, H)] = pats[t]
        x[t] = row | (g.integers(0, 2, H).astype(np.uint16) << 15)
    tau = 3.0e38 if dtype == "bf16" else 65504.0
    check_parity(tsq, oracle, x, dtype, tau, (2, 3, 4, 5, 6, 7, 8), 0.05, "rel_rms", pipeline, label="absmax sweep")
    check_parity(tsq, oracle, x, dtype, tau, (3, 5, 8), 0.25, "lsb", pipeline, label="absmax sweep lsb")


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_exact_halves_round_to_even(tsq, oracle, pipeline, dtype):
    # rows whose scaled magnitudes a*r are exactly k + 1/2: the code must be the even neighbour
    for b in range(2, 9):
        Q = 2 ** (b - 1) - 1
        p = 3
        k = np.arange(0, max(Q, 1))
        vals = np.concatenate([(k + 0.5) * 2.0 ** -p, [Q * 2.0 ** -p]])          # absmax = Q*2^-p: r = 2^p
        reps = -(-256 // vals.size)
        row = np.tile(vals, reps)[:256]
        row[-1] = Q * 2.0 ** -p
        x = np.stack([row, -row, row[::-1].copy()])
        bits = synth.to_f16_bits(x) if dtype == "f16" else synth.to_bf16_bits(x)
        ref, _ = check_parity(tsq, oracle, bits, dtype, 1.0e4, (b,), 0.05, "rel_rms", pipeline,
                              label="ties b=%d" % b)
        m, neg = oracle.unpack_row(ref.payload[: 4 * ((256 * b + 31) // 32)], 256, b)
        kk = np.tile(np.concatenate([k, [Q]]), reps)[:255]
        tie = kk != Q
        expect = np.where(kk % 2 == 0, kk, kk + 1)
        assert np.array_equal(m[:255][tie], expect[tie])


@pytest.mark.parametrize("pipeline", PIPELINES)
def test_all_width_subsets_small(tsq, oracle, pipeline):
    import itertools
    x = synth.make_c2(tokens=32)[:, :1024].copy()
    subsets = [s for n in (1, 2, 3, 7) for s in itertools.combinations(range(2, 9), n)]
    for i, bs in enumerate(subsets):
        bud, mode = ((0.05, "rel_rms"), (0.2, "rel_rms"), (0.25, "lsb"))[i % 3]
        check_parity(tsq, oracle, x, "f16", 4.0, bs, bud, mode, pipeline, label="subset %s" % (bs,))


@pytest.mark.parametrize("pipeline", PIPELINES)
def test_side_stream_overflow_is_reported_and_decompress_refuses(tsq, oracle, pipeline):
    import torch
    x = synth.make_c2(tokens=64)
    ref = oracle.compress(x, F16, 8.0, (2, 4, 8), 0.05, 1, nthreads=4)
    assert ref.nnz > 40
    plan = tsq.Plan(64, 4096, "f16", 8.0, (2, 4, 8), 0.05, pipeline=pipeline, max_outliers=ref.nnz - 1)
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    blob = plan.compress(xd)
    info = plan.info(blob, check=False)
    assert info.return_status == tsq.TSQ_ERR_CAPACITY and info.status == tsq.TSQ_ERR_CAPACITY
    assert info.nnz == ref.nnz                                  # the true count is still reported
    sec = plan.sections(blob)
    assert np.array_equal(sec["bits"], ref.bits) and np.array_equal(sec["row_ptr"], ref.row_ptr)
    out = plan.new_output()
    out.fill_(0x1234)
    plan.decompress(blob, out)
    assert bool((out == 0x1234).all())                          # nothing written
    # the exact capacity works
    plan2 = tsq.Plan(64, 4096, "f16", 8.0, (2, 4, 8), 0.05, pipeline=pipeline, max_outliers=ref.nnz)
    blob2 = plan2.compress(xd)
    assert plan2.info(blob2).status == 0
    assert np.array_equal(plan2.decompress(blob2).cpu().numpy().view(np.uint16), oracle.decompress(ref))


def test_decompress_refuses_a_foreign_blob(tsq):
    import torch
    plan = tsq.Plan(16, 256, "f16", 6.0, (4, 8), 0.05)
    blob = plan.new_blob()
    blob.zero_()
    out = plan.new_output()
    out.fill_(0x0BAD)
    plan.decompress(blob, out)
    assert bool((out == 0x0BAD).all())
    info = plan.info(blob, check=False)
    assert info.return_status == tsq.TSQ_ERR_FORMAT


@pytest.mark.parametrize("pipeline", PIPELINES)
def test_workspace_and_plan_serve_many_calls(tsq, oracle, pipeline):
    # one plan, one workspace, eleven calls on changing inputs: whatever a call leaves in the
    # workspace (tags, ticket counters, epoch) must not leak into the next one
    import torch
    T, H = 700, 2048
    g = np.random.Generator(np.random.PCG64(11))
    xs = []
    for k in range(3):
        v = g.standard_normal((T, H)) * g.lognormal(0.0, 0.6, (T, 1))
        v[:, g.choice(H, 5, replace=False)] *= 40.0
        xs.append(synth.to_bf16_bits(v))
    refs = [oracle.compress(x, BF16, 8.0, (2, 4, 5, 8), 0.1, 1, nthreads=8) for x in xs]
    plan = tsq.Plan(T, H, "bf16", 8.0, (2, 4, 5, 8), 0.1, pipeline=pipeline)
    ws = plan.new_workspace()
    blob = plan.new_blob()
    out = plan.new_output()
    for call in range(11):
        k = (call * 2) % 3
        print("call", call, "input", k, flush=True)
        plan.compress(torch.from_numpy(xs[k].view(np.int16)).cuda(), blob, ws)
        info = plan.info(blob)
        sec = plan.sections(blob)
        ref = refs[k]
        assert info.status == 0 and info.nnz == ref.nnz and info.payload_bytes == ref.payload_bytes
        for name, want in (("bits", ref.bits), ("row_ptr", ref.row_ptr), ("pay_off", ref.pay_off),
                           ("out_col", ref.out_col), ("out_val", ref.out_val), ("payload", ref.payload)):
            assert np.array_equal(sec[name], want), (call, name)
        plan.decompress(blob, out)
        assert np.array_equal(out.cpu().numpy().view(np.uint16), oracle.decompress(ref, nthreads=8)), call


@pytest.mark.parametrize("pipeline", PIPELINES)
@pytest.mark.parametrize("T,H", [(1, 64), (2, 64), (63, 64), (64, 64), (65, 64), (130, 256), (1025, 256),
                                 (4097, 64), (9000, 64), (40000, 96), (5000, 2048 + 64)])
def test_token_counts_around_the_grid_size(tsq, oracle, pipeline, T, H):
    # fewer tokens than workgroups, exactly as many, and several per workgroup (short rows keep
    # many workgroups resident, so the larger counts need more than one round of tickets)
    g = np.random.Generator(np.random.PCG64(T * 131 + H))
    v = g.standard_normal((T, H)) * g.lognormal(0.0, 0.8, (T, 1))
    v[g.random((T, H)) < 0.004] *= 30.0
    x = synth.to_f16_bits(v)
    check_parity(tsq, oracle, x, "f16", 6.0, (2, 3, 4, 6, 8), 0.15, "rel_rms", pipeline, label="T=%d H=%d" % (T, H))


@pytest.mark.parametrize("pipeline", PIPELINES)
def test_tokens_with_more_outliers_than_the_stash_holds(tsq, oracle, pipeline):
    # rows with more outliers per wave than the single-pass kernel keeps in LDS (232 per wave of 2048 elements
    # for this row length) take its re-read path; counts on both sides of that limit, mixed with ordinary
    # rows and with rows that are all outliers
    g = np.random.Generator(np.random.PCG64(5))
    T, H = 300, 4096
    v = g.standard_normal((T, H))
    heavy = g.choice(T, 40, replace=False)
    for i, t in enumerate(heavy):
        n = (420, 460, 500, 513, 600, 1024, 2048, 4096)[i % 8]
        v[t, g.choice(H, n, replace=False)] = 50.0 * g.choice([-1.0, 1.0], n)
    x = synth.to_bf16_bits(v)
    ref, _ = check_parity(tsq, oracle, x, "bf16", 6.0, (2, 4, 8), 0.05, "rel_rms", pipeline, label="heavy rows")
    cnt = np.diff(ref.row_ptr.astype(np.int64))
    assert (cnt > 512).sum() >= 20 and (cnt > 410).sum() >= 40 and cnt.max() == H


@pytest.mark.parametrize("pipeline", PIPELINES)
def test_calls_captured_in_a_hip_graph_replay_correctly(tsq, oracle, pipeline):
    # compress + decompress captured once, replayed on changing input with eager work and synchronisation in
    # between; every replay must give what the eager calls give (the workspace state moves on from call to call)
    import torch
    T, H = 700, 4096
    g = np.random.Generator(np.random.PCG64(21))
    plan = tsq.Plan(T, H, "f16", 6.0, (2, 3, 4, 6, 8), 0.1, pipeline=pipeline)
    x_static = torch.zeros((T, H), dtype=torch.int16, device="cuda")
    blob, out, ws = plan.new_blob(), plan.new_output(), plan.new_workspace()
    plan.compress(x_static, blob, ws)                         # warm-up outside the capture (first-call set-up)
    plan.decompress(blob, out)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            plan.compress(x_static, blob, ws)
            plan.decompress(blob, out)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        v = g.standard_normal((T, H)) * g.lognormal(0.0, 0.7, (T, 1)) * (1.0 + rep)
        v[g.random((T, H)) < 0.003] *= 20.0
        x = synth.to_f16_bits(v)
        x_static.copy_(torch.from_numpy(x.view(np.int16)))
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.compress(x, F16, 6.0, (2, 3, 4, 6, 8), 0.1, 1, nthreads=8)
        sec = plan.sections(blob)
        assert plan.info(blob).status == 0
        for k, want in (("bits", ref.bits), ("row_ptr", ref.row_ptr), ("pay_off", ref.pay_off),
                        ("out_col", ref.out_col), ("out_val", ref.out_val), ("payload", ref.payload)):
            assert np.array_equal(sec[k], want), "replay %d: %s" % (rep, k)
        assert np.array_equal(out.cpu().numpy().view(np.uint16), oracle.decompress(ref, nthreads=8)), "replay %d" % rep
        # eager work between the replays: another call on the same workspace
        plan.compress(x_static, plan.new_blob(), ws)
        torch.cuda.synchronize()


@pytest.mark.parametrize("seed", range(6))
def test_random_configurations(tsq, oracle, seed):
    # shapes, thresholds, width sets, budgets and data scales drawn at random (seeded): ten cases per seed
    g = np.random.Generator(np.random.PCG64(1000 + seed))
    for k in range(10):
        H = 8 * int(g.integers(1, 600))
        T = int(g.integers(1, 400))
        dtype = ("f16", "bf16")[int(g.integers(0, 2))]
        tau = float(g.choice([0.5, 2.0, 4.0, 6.0, 10.0, 16.0, 100.0]))
        widths = sorted(set(int(b) for b in g.choice(np.arange(2, 9), size=int(g.integers(1, 8)))))
        mode = ("lsb", "rel_rms")[int(g.integers(0, 2))]
        budget = float(g.choice([0.0, 0.02, 0.05, 0.1, 0.2, 0.3, 0.5, 1.0])) if mode == "rel_rms" else \
            float(g.choice([0.0, 0.05, 0.2, 0.3, 0.5, 2.0]))
        scale = 10.0 ** g.uniform(-3, 1.3)
        v = g.standard_t(4, size=(T, H)) * scale * g.lognormal(0.0, 0.6, (T, 1))
        if g.random() < 0.5:
            v[:, g.choice(H, max(1, H // 200), replace=False)] *= 25.0
        if g.random() < 0.3:
            v[g.random((T, H)) < 0.3] = 0.0
        with np.errstate(over="ignore"):
            x = synth.to_f16_bits(v) if dtype == "f16" else synth.to_bf16_bits(np.clip(v, -3e38, 3e38))
        pipeline = PIPELINES[int(g.integers(0, 2))]
        check_parity(tsq, oracle, x, dtype, tau, widths, budget, mode, pipeline, label="random %d.%d" % (seed, k))


def test_c5_stress_full_size_whole_blob_all_six_sweep_points(tsq, oracle):
    """The whole heavy-outlier workload (131072 x 8192 bf16, 2 GiB) in the configuration bench.py times, at
    every threshold and bit set of the sweep: every section of the blob and every decoded element against
    the oracle's (the oracle compresses the 2 GiB with all host threads in a few seconds)."""
    import torch
    eps = 0.05
    print("generating C5", flush=True)
    x = synth.make_c5(workers=8)
    T, H = x.shape
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    out = torch.empty((T, H), dtype=torch.int16, device="cuda")
    threads = min(16, oracle.max_threads())
    for tau in synth.C5_TAUS:
        for bit_set in synth.C5_BIT_SETS:
            label = "C5 tau %g bits %s" % (tau, bit_set)
            print(label + ": oracle", flush=True)
            ref = oracle.compress(x, BF16, tau, bit_set, eps, 1, nthreads=threads)
            plan = tsq.Plan(T, H, "bf16", tau, bit_set, eps, max_outliers=max(ref.nnz, 1))
            print(label + ": compress, decompress", flush=True)
            blob = plan.compress(xd)
            info = plan.info(blob)
            assert info.status == 0 and info.nnz == ref.nnz and info.payload_bytes == ref.payload_bytes, label
            assert info.compressed_bytes == oracle.compressed_bytes(ref)
            out.fill_(0x5A5A)
            plan.decompress(blob, out)
            sec = plan.sections(blob)
            del blob
            for k in ("bits", "row_ptr", "pay_off", "out_col", "out_val", "payload"):
                assert np.array_equal(sec[k], getattr(ref, k)), label + ": " + k
            assert np.array_equal(sec["scale"].view(np.uint32), ref.scale.view(np.uint32)), label
            del sec
            ref_out = oracle.decompress(ref, nthreads=threads)
            del ref
            got = out.cpu().numpy().view(np.uint16)
            assert np.array_equal(got, ref_out), label + ": decoded bits"
            del got, ref_out
