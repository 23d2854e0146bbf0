"""Pins for the CPU oracle: each test checks it against something other than
itself — a definition written independently in numpy, a library routine
(numpy / scipy / torch CPU), an exact-rational brute force, a closed form or an
invariant of the method (paper Sec. II-C: Eq. (ts), Eq. (Proposed), Algorithm 1,
Eq. (dequnt)).  The paper prints no worked numeric example of these steps, so
there are no printed values to match.
"""
from fractions import Fraction
import itertools

import numpy as np
import pytest

from paper_2511_04002_amd import synth

F16, BF16 = 0, 1
LSB, REL = 0, 1


# ------------------------------------------------------------------ helpers
# (independent of the oracle: numpy / torch / Fractions only)

def np_widen(raw, dtype):
    raw = np.asarray(raw, np.uint16)
    if dtype == F16:
        return raw.view(np.float16).astype(np.float32)
    return (raw.astype(np.uint32) << 16).view(np.float32)


def f16_bits(vals):
    return np.asarray(vals, np.float64).astype(np.float16).view(np.uint16)


def bf16_bits_exact(vals):
    """bf16 patterns of values that are exactly representable in bf16."""
    u = np.asarray(vals, np.float32).view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value is not a bf16 number"
    return (u >> 16).astype(np.uint16)


def rhe(fr: Fraction) -> int:
    """Round a non-negative rational to the nearest integer, ties to even."""
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def brute_select(a_fr, amax_fr, bit_set, budget_fr, mode, as_printed=False):
    """Algorithm 1 in exact rationals, for rows where binary32 is exact.  as_printed: the width that
    fails the test is the one returned (the printed order of steps) instead of the last that passed."""
    H = len(a_fr)
    ws = sorted(bit_set, reverse=True)
    Q = {b: 2 ** (b - 1) - 1 for b in ws}

    def codes(b):
        if amax_fr == 0:
            return [0] * H
        return [min(rhe(x * Q[b] / amax_fr), Q[b]) for x in a_fr]

    m0 = codes(ws[0])
    ss0 = sum(v * v for v in m0)
    sel, sads = ws[0], []
    for b in ws[1:]:
        mb = codes(b)
        sad = sum(abs((r0 >> (ws[0] - b)) - v) for r0, v in zip(m0, mb))
        sads.append(sad)
        if mode == LSB:
            viol = Fraction(sad) > budget_fr * H
        else:
            viol = Fraction(Q[ws[0]] * sad) ** 2 > (budget_fr * Q[b]) ** 2 * H * ss0
        if viol:
            if as_printed:
                sel = b
            break
        sel = b
    return sel, ss0, sads


# ------------------------------------------------------------------ 16-bit formats

def test_widen_all_patterns_match_numpy_and_torch(oracle):
    import torch
    raw = np.arange(65536, dtype=np.uint16)
    got16 = oracle.widen(raw, F16)
    ref16 = np_widen(raw, F16)
    fin = ~np.isnan(ref16)
    assert np.array_equal(got16[fin].view(np.uint32), ref16[fin].view(np.uint32))
    assert np.all(np.isnan(got16[~fin]))
    gotb = oracle.widen(raw, BF16)
    refb = torch.from_numpy(raw.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    finb = ~np.isnan(refb)
    assert np.array_equal(gotb[finb].view(np.uint32), refb[finb].view(np.uint32))
    assert np.all(np.isnan(gotb[~finb]))


def test_narrow_matches_numpy_f16_and_torch_bf16(oracle):
    import torch
    g = np.random.Generator(np.random.PCG64(11))
    vals = np.concatenate([
        g.standard_normal(4000) * 10.0 ** g.integers(-9, 5, 4000),
        # binary16 ties, subnormal range, overflow edge
        np.array([0.0, -0.0, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -24, 2.0 ** -25,
                  3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 65504.0, 65519.9, 65520.0,
                  70000.0, -65520.0, 1e-8, 5.9e-8, 6.1e-5, np.inf, -np.inf]),
        np_widen(np.arange(0, 0x7C00, 7, dtype=np.uint16), F16).astype(np.float64),
    ]).astype(np.float32)
    vals = vals[~np.isnan(vals)]
    with np.errstate(over="ignore"):
        ref16 = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.narrow(vals, F16), ref16)
    # midpoints between neighbouring binary16 values (exact in binary32)
    h = np.arange(0x0001, 0x7BFF, 37, dtype=np.uint16)
    mid = (np_widen(h, F16).astype(np.float64) + np_widen(h + 1, F16).astype(np.float64)) / 2
    mid32 = mid.astype(np.float32)
    assert np.array_equal(mid32.astype(np.float64), mid)
    assert np.array_equal(oracle.narrow(mid32, F16), mid32.astype(np.float16).view(np.uint16))
    refb = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.narrow(vals, BF16), refb)
    # bf16 ties: fp32 patterns whose low half is exactly 0x8000
    t = (g.integers(0x0080, 0x7F00, 2000).astype(np.uint32) << 16 | 0x8000).view(np.float32)
    reft = torch.from_numpy(t.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.narrow(t, BF16), reft)


def test_narrow_widen_identity(oracle):
    raw = np.arange(65536, dtype=np.uint16)
    for dt in (F16, BF16):
        v = np_widen(raw, dt)
        ok = ~np.isnan(v)
        assert np.array_equal(oracle.narrow(v[ok], dt), raw[ok])


# ------------------------------------------------------------------ Eq. (ts)

@pytest.mark.parametrize("dt", [F16, BF16])
def test_ts_mask_and_count_definition(oracle, dt):
    g = np.random.Generator(np.random.PCG64(5))
    H, tau = 997, 2.5
    x = g.standard_normal(H) * 2.0
    raw = f16_bits(x) if dt == F16 else synth.to_bf16_bits(x)
    out, a, cnt, amax = oracle.ts_row(raw, dt, tau)
    v = np_widen(raw, dt)
    ref_out = np.abs(v) >= np.float32(tau)                         # Eq. (ts), as printed
    assert np.array_equal(out.astype(bool), ref_out)
    assert cnt == int(ref_out.sum())
    assert np.array_equal(a, np.where(ref_out, np.float32(0), np.abs(v)))
    assert amax == np.abs(v)[~ref_out].max()
    # T_above + T_below == T, elementwise
    t_above = np.where(ref_out, v, 0)
    t_below = np.where(out.astype(bool), 0, v)
    assert np.array_equal(t_above + t_below, v)


def test_ts_ties_specials_and_one_ulp_below(oracle):
    tau = 6.0
    below = np.nextafter(np.float16(tau), np.float16(0))
    raw = np.array([np.float16(tau), np.float16(-tau), below, -below,
                    np.float16(np.inf), np.float16(-np.inf), np.float16(0), np.float16(-0.0)],
                   np.float16).view(np.uint16)
    raw = np.concatenate([raw, np.array([0x7E01, 0xFE02], np.uint16)])     # NaNs
    out, a, cnt, amax = oracle.ts_row(raw, F16, tau)
    assert out.tolist() == [1, 1, 0, 0, 1, 1, 0, 0, 1, 1]
    assert cnt == 6 and amax == np.float32(below)
    assert a[0] == 0 and a[4] == 0 and a[8] == 0
    # bf16: tau itself and the next pattern down
    t = bf16_bits_exact([10.0])[0]
    rawb = np.array([t, t | 0x8000, t - 1, (t - 1) | 0x8000, 0x7FC0, 0x7F80, 0xFF80], np.uint16)
    outb, _, cntb, amaxb = oracle.ts_row(rawb, BF16, 10.0)
    assert outb.tolist() == [1, 1, 0, 0, 1, 1, 1] and cntb == 5
    assert amaxb == np_widen(np.array([t - 1], np.uint16), BF16)[0]


def test_csr_matches_scipy(oracle):
    import scipy.sparse as sp
    x = synth.make_c2(tokens=64)
    tau = 3.0                                                       # low threshold: many outliers
    c = oracle.compress(x, F16, tau, (2, 4, 8), 0.05, REL)
    v = np_widen(x, F16)
    dense = np.where(np.abs(v) >= np.float32(tau), v, np.float32(0))
    ref = sp.csr_matrix(dense)
    ref.sort_indices()
    assert np.array_equal(c.row_ptr, ref.indptr.astype(np.uint64))
    assert np.array_equal(c.out_col, ref.indices.astype(np.uint16))
    assert np.array_equal(np_widen(c.out_val, F16), ref.data)
    # and the values are the input's raw bits
    rows = np.repeat(np.arange(64), np.diff(c.row_ptr).astype(np.int64))
    assert np.array_equal(c.out_val, x[rows, c.out_col])
    assert c.nnz == int((np.abs(v) >= np.float32(tau)).sum())


def test_offsets_are_exclusive_cumsums(oracle):
    x = synth.make_c2(tokens=96)
    c = oracle.compress(x, F16, 8.0, (2, 3, 4, 6, 8), 0.2, REL)
    assert len(set(c.bits.tolist())) >= 3                          # really variable length
    nbytes = np.array([4 * ((x.shape[1] * int(b) + 31) // 32) for b in c.bits], np.uint64)
    assert np.array_equal(c.pay_off, np.concatenate([[0], np.cumsum(nbytes)]).astype(np.uint64))
    assert np.array_equal(c.row_ptr,
                          np.concatenate([[0], np.cumsum(c.info["cnt"])]).astype(np.uint64))
    assert np.array_equal(c.info["nbytes"], nbytes.astype(np.uint32))


# ------------------------------------------------------------------ Eq. (Proposed)

@pytest.mark.parametrize("b", [2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("p", [0, 3, 9])
def test_aiq_dyadic_rows_are_lossless(oracle, b, p):
    Q = 2 ** (b - 1) - 1
    g = np.random.Generator(np.random.PCG64(100 * b + p))
    k = g.integers(0, Q + 1, 64)
    k[7] = Q                                                        # the absmax element
    a = (k * 2.0 ** -p).astype(np.float32)
    m, r, s = oracle.aiq_row(a, a.max(), b)
    # closed form: amax = Q*2^-p  =>  s = 2^-p and r = 2^p exactly, m = a/s exactly
    assert s == np.float32(2.0 ** -p) and r == np.float32(2.0 ** p)
    assert np.array_equal(m, k)
    assert np.array_equal(m.astype(np.float32) * s, a)


@pytest.mark.parametrize("b", [3, 4, 6, 8])
def test_aiq_halfway_goes_to_even(oracle, b):
    Q = 2 ** (b - 1) - 1
    p = 4
    k = np.arange(0, Q)                                              # k + 1/2 for k = 0 .. Q-1
    a = np.concatenate([(k + 0.5) * 2.0 ** -p, [Q * 2.0 ** -p]]).astype(np.float32)
    m, r, s = oracle.aiq_row(a, a.max(), b)
    expect = np.concatenate([np.where(k % 2 == 0, k, k + 1), [Q]])   # even neighbour
    assert np.array_equal(m, expect)
    # half-away-from-zero would give k+1 everywhere, truncation k everywhere
    assert not np.array_equal(expect[:-1], k + 1) and not np.array_equal(expect[:-1], k)


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("b", [2, 3, 4, 5, 6, 7, 8])
def test_aiq_error_bound_and_range(oracle, dt, b):
    g = np.random.Generator(np.random.PCG64(b))
    x = g.standard_t(4.0, 4096) * np.exp(g.normal(0, 2))
    raw = f16_bits(x) if dt == F16 else synth.to_bf16_bits(x)
    out, a, cnt, amax = oracle.ts_row(raw, dt, 6.0)
    m, r, s = oracle.aiq_row(a, amax, b)
    Q = 2 ** (b - 1) - 1
    assert m.min() >= 0 and m.max() == Q
    assert m[np.argmax(a)] == Q                                      # the absmax element is full scale
    a64, s64 = a.astype(np.float64), float(s)
    assert np.all(np.abs(a64 - m * s64) <= (0.5 + 1e-4) * s64)
    assert abs(s64 - float(amax) / Q) <= 2.0 ** -24 * s64
    assert np.all(m[out.astype(bool)] == 0)


def test_aiq_zero_and_tiny_rows(oracle):
    a = np.zeros(32, np.float32)
    m, r, s = oracle.aiq_row(a, 0.0, 8)
    assert r == 0 and s == 0 and not m.any()
    # below the floor the reciprocal could overflow binary32: treated as a zero row
    tiny = np.float32(2.0 ** -110)
    m, r, s = oracle.aiq_row(np.full(8, tiny, np.float32), tiny, 8)
    assert r == 0 and s == 0 and not m.any()
    # at the floor everything is finite and full scale is reached
    fl = np.float32(2.0 ** -100)
    m, r, s = oracle.aiq_row(np.array([fl, fl / 2, 0], np.float32), fl, 8)
    assert np.isfinite(r) and s > 0 and m.tolist() == [127, 64, 0]


# ------------------------------------------------------------------ Algorithm 1

def _dyadic_rows(g, rows, H, frac_bits=6):
    """Rows whose absmax is a power of two and whose entries have few bits, so
    that every binary32 operation of the selection is exact."""
    out = []
    for _ in range(rows):
        e = int(g.integers(-3, 3))
        k = g.integers(0, 2 ** frac_bits + 1, H)
        k[int(g.integers(0, H))] = 2 ** frac_bits
        out.append([Fraction(int(v), 2 ** frac_bits) * Fraction(2) ** e for v in k])
    return out


@pytest.mark.parametrize("mode", [LSB, REL])
def test_selection_matches_exact_rational_brute_force(oracle, mode):
    g = np.random.Generator(np.random.PCG64(42 + mode))
    subsets = [s for n in (1, 2, 3) for s in itertools.combinations(range(2, 9), n)]
    budgets = ([Fraction(0), Fraction(1, 8), Fraction(1, 4), Fraction(1, 2), Fraction(2)] if mode == LSB
               else [Fraction(0), Fraction(1, 32), Fraction(1, 16), Fraction(1, 8), Fraction(1, 2)])
    checked, widths_seen = 0, set()
    for H in (8, 32, 33):
        for row in _dyadic_rows(g, 6, H):
            a = np.array([float(v) for v in row], np.float32)
            amax_fr = max(row)
            for bs in subsets:
                for bud in budgets:
                    sel, ss0, sads = brute_select(row, amax_fr, bs, bud, mode)
                    info = oracle.select_row(a, float(amax_fr), bs, float(bud), mode)
                    assert int(info["bits"]) == sel, (H, bs, bud)
                    assert int(info["ss0"]) == ss0
                    assert info["sad"][1:1 + len(sads)].tolist() == sads
                    assert int(info["n_eval"]) == len(sads)
                    assert float(info["scale"]) == float(np.float32(float(amax_fr)) /
                                                         np.float32(2 ** (sel - 1) - 1))
                    checked += 1
                    widths_seen.add(sel)
    assert checked > 5000 and widths_seen == set(range(2, 9))


def test_selection_returns_last_passing_width_not_the_violating_one(oracle):
    # one full-scale element, the rest at 0.4 of full scale, H = 8, B = {8, 4, 2}
    # 8-bit codes: 127 and rint(50.8)=51; 4-bit: 7 and rint(2.8)=3; 2-bit: 1 and 0
    # candidate 4: |127>>4 - 7| + 7*|51>>4 - 3| = 0 + 0 = 0           -> passes any budget
    # candidate 2: |127>>6 - 1| + 7*|51>>6 - 0| = 0                    -> passes too
    a = np.array([1.0] + [0.4] * 7, np.float32)
    info = oracle.select_row(a, 1.0, (2, 4, 8), 0.0, LSB)
    assert int(info["bits"]) == 2 and info["sad"][1:3].tolist() == [0, 0]
    # rest at 0.45: 8-bit rint(57.15)=57 -> 57>>4 = 3 ; 4-bit rint(3.15)=3 ; 2-bit rint(.45)=0 -> 0
    # rest at 0.55: 8-bit rint(69.85)=70 -> 70>>4 = 4 ; 4-bit rint(3.85)=4 ; 70>>6 = 1 ; 2-bit rint(.55)=1
    # rest at 0.3 : 8-bit rint(38.1)=38 -> 38>>4 = 2 ; 4-bit rint(2.1)=2 ; 38>>6=0 ; 2-bit 0
    # rest at 0.25: 8-bit rint(31.75)=32 -> 2 ; 4-bit rint(1.75)=2
    # rest at 0.21: 8-bit rint(26.67)=27 -> 27>>4 = 1 ; 4-bit rint(1.47)=1
    # rest at 0.22: 8-bit rint(27.94)=28 -> 1 ; 4-bit rint(1.54)=2 -> SAD_4 = 7
    a = np.array([1.0] + [0.22] * 7, np.float32)
    i0 = oracle.select_row(a, 1.0, (2, 4, 8), 0.5, LSB)        # 7 > 0.5*8 -> violates at 4: keep 8
    assert int(i0["bits"]) == 8 and int(i0["sad"][1]) == 7 and int(i0["n_eval"]) == 1
    i1 = oracle.select_row(a, 1.0, (2, 4, 8), 0.875, LSB)      # 7 > 7 is false -> 4 passes
    # candidate 2: |127>>6 - 1| + 7*|28>>6 - rint(0.22)| = 0 -> passes -> 2
    assert int(i1["bits"]) == 2 and int(i1["n_eval"]) == 2
    i2 = oracle.select_row(a, 1.0, (4, 8), 0.875, LSB)
    assert int(i2["bits"]) == 4 and float(i2["scale"]) == float(np.float32(1.0) / np.float32(7.0))


@pytest.mark.parametrize("mode", [LSB, REL])
def test_printed_return_rule_matches_exact_rational_brute_force(oracle, mode):
    """Algorithm 1 with the return as printed (the quantization at the width that failed): the same
    statistics, and the width one candidate further down wherever the descent stopped."""
    g = np.random.Generator(np.random.PCG64(142 + mode))
    subsets = [s for n in (1, 2, 3, 4) for s in itertools.combinations(range(2, 9), n)][::2]
    budgets = ([Fraction(0), Fraction(1, 8), Fraction(1, 2), Fraction(2)] if mode == LSB
               else [Fraction(0), Fraction(1, 32), Fraction(1, 8), Fraction(1, 2)])
    checked, moved = 0, 0
    for H in (8, 33):
        for row in _dyadic_rows(g, 5, H):
            a = np.array([float(v) for v in row], np.float32)
            amax_fr = max(row)
            for bs in subsets:
                ws = sorted(bs, reverse=True)
                for bud in budgets:
                    sel, ss0, sads = brute_select(row, amax_fr, bs, bud, mode, as_printed=True)
                    keep, _, _ = brute_select(row, amax_fr, bs, bud, mode)
                    info = oracle.select_row(a, float(amax_fr), bs, float(bud), mode, oracle.RETURN_AS_PRINTED)
                    assert int(info["bits"]) == sel, (H, bs, bud)
                    assert int(info["ss0"]) == ss0 and info["sad"][1:1 + len(sads)].tolist() == sads
                    assert int(info["n_eval"]) == len(sads)
                    assert float(info["scale"]) == float(np.float32(float(amax_fr)) / np.float32(2 ** (sel - 1) - 1))
                    # either the same width (nothing failed) or the next allowed width below the kept one
                    assert sel == keep or sel == ws[ws.index(keep) + 1]
                    moved += sel != keep
                    checked += 1
    assert checked > 1500 and moved > 200


def test_printed_return_rule_by_hand_and_as_a_blob(oracle):
    # the row of the test above: one full-scale element, seven at 0.22; B = {8, 4, 2}; SAD_4 = 7
    a = np.array([1.0] + [0.22] * 7, np.float32)
    i0 = oracle.select_row(a, 1.0, (2, 4, 8), 0.5, LSB, oracle.RETURN_AS_PRINTED)     # 7 > 4: fails at 4 -> 4 is returned
    assert int(i0["bits"]) == 4 and int(i0["n_eval"]) == 1 and float(i0["scale"]) == float(np.float32(1.0) / np.float32(7.0))
    i1 = oracle.select_row(a, 1.0, (2, 4, 8), 0.875, LSB, oracle.RETURN_AS_PRINTED)   # nothing fails -> 2, as before
    assert int(i1["bits"]) == 2 and int(i1["n_eval"]) == 2
    i2 = oracle.select_row(a, 1.0, (8,), 0.0, LSB, oracle.RETURN_AS_PRINTED)          # no candidate at all
    assert int(i2["bits"]) == 8
    # whole tensors: widths per token from select_row, everything else follows from the widths exactly as
    # in the default reading (codes, offsets, sizes, round trip within half a step of the returned width)
    x = synth.make_c2(tokens=48)
    for eps in (0.05, 0.2):
        c0 = oracle.compress(x, F16, 8.0, (2, 3, 4, 6, 8), eps, REL)
        c1 = oracle.compress(x, F16, 8.0, (2, 3, 4, 6, 8), eps, REL, rule=oracle.RETURN_AS_PRINTED)
        assert np.all(c1.bits <= c0.bits) and np.any(c1.bits < c0.bits)
        assert np.array_equal(c1.row_ptr, c0.row_ptr) and np.array_equal(c1.out_col, c0.out_col)
        sizes = np.array([oracle.row_bytes(x.shape[1], int(b)) for b in c1.bits], np.uint64)
        assert np.array_equal(c1.pay_off, np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64))
        for t in (0, 7, 47):
            _, at, _, amax = oracle.ts_row(x[t], F16, 8.0)
            info = oracle.select_row(at, amax, (2, 3, 4, 6, 8), eps, REL, oracle.RETURN_AS_PRINTED)
            assert int(c1.bits[t]) == int(info["bits"]) and float(c1.scale[t]) == float(info["scale"])
            m, _, s = oracle.aiq_row(at, amax, int(c1.bits[t]))
            got_m, _ = oracle.unpack_row(c1.payload[int(c1.pay_off[t]): int(c1.pay_off[t + 1])], x.shape[1], int(c1.bits[t]))
            assert np.array_equal(got_m, m)
        out = oracle.widen(oracle.decompress(c1), F16)
        v = oracle.widen(x, F16)
        inl = np.abs(v) < 8.0
        step = np.repeat(c1.scale[:, None], x.shape[1], axis=1)
        assert np.all(np.abs(out[inl] - v[inl]) <= 0.5001 * step[inl] + 1e-3 * np.abs(v[inl]))


def test_selection_limit_cases_and_monotonicity(oracle):
    g = np.random.Generator(np.random.PCG64(9))
    x = synth.make_c2(tokens=24)
    for t in range(24):
        out, a, cnt, amax = oracle.ts_row(x[t], F16, 8.0)
        for b in range(2, 9):                                       # |B| = 1
            assert int(oracle.select_row(a, amax, (b,), 0.05, REL)["bits"]) == b
        for mode in (LSB, REL):
            bs = (2, 3, 4, 6, 8)
            assert int(oracle.select_row(a, amax, bs, np.inf, mode)["bits"]) == 2
            i0 = oracle.select_row(a, amax, bs, 0.0, mode)
            if int(i0["sad"][1]) > 0:                                # zero budget: any deviation violates
                assert int(i0["bits"]) == 8 and int(i0["n_eval"]) == 1
            prev = 9
            for bud in (0.0, 0.01, 0.03, 0.05, 0.1, 0.2, 0.3, 0.5, 1.0, 4.0):
                cur = int(oracle.select_row(a, amax, bs, bud, mode)["bits"])
                assert cur <= prev                                   # loosening never widens
                prev = cur
    z = np.zeros(64, np.float32)                                     # all-zero row
    for mode in (LSB, REL):
        i = oracle.select_row(z, 0.0, (3, 5, 8), 0.0, mode)
        assert int(i["bits"]) == 3 and float(i["scale"]) == 0.0


def test_rel_rms_is_invariant_to_power_of_two_scaling(oracle):
    x = synth.make_c2(tokens=16)
    v = np_widen(x, F16).astype(np.float64)
    for k in (1, 2):
        y = f16_bits(v * 2.0 ** k)
        c0 = oracle.compress(x, F16, 8.0, (2, 3, 4, 6, 8), 0.1, REL)
        c1 = oracle.compress(y, F16, 8.0 * 2.0 ** k, (2, 3, 4, 6, 8), 0.1, REL)
        # scaling up by a power of two is exact in fp16 as long as nothing overflows
        assert np.array_equal(np_widen(y, F16), (v * 2.0 ** k).astype(np.float32))
        assert np.array_equal(c0.bits, c1.bits)
        assert np.array_equal(c0.payload, c1.payload)
        assert np.array_equal(c0.row_ptr, c1.row_ptr)
        assert np.array_equal(c0.scale * np.float32(2.0 ** k), c1.scale)


# ------------------------------------------------------------------ packing

@pytest.mark.parametrize("b", [2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("H", [1, 31, 32, 33, 200])
def test_pack_matches_numpy_packbits(oracle, b, H):
    g = np.random.Generator(np.random.PCG64(b * 1000 + H))
    Q = 2 ** (b - 1) - 1
    m = g.integers(0, Q + 1, H).astype(np.int32)
    neg = (g.integers(0, 2, H).astype(np.uint8)) & (m > 0)
    got = oracle.pack_row(m, neg, b)
    code = (neg.astype(np.uint32) << (b - 1)) | m.astype(np.uint32)
    bitmat = ((code[:, None] >> np.arange(b)[None, :]) & 1).astype(np.uint8)   # LSB first
    ref = np.packbits(bitmat.reshape(-1), bitorder="little")
    assert got.size == 4 * ((H * b + 31) // 32)
    assert np.array_equal(got[:ref.size], ref) and not got[ref.size:].any()
    if b == 8:
        assert np.array_equal(got[:H], ((neg << 7) | m).astype(np.uint8))
    m2, neg2 = oracle.unpack_row(got, H, b)
    assert np.array_equal(m2, m) and np.array_equal(neg2, neg)


# ------------------------------------------------------------------ Eq. (dequnt) and the whole tensor

@pytest.mark.parametrize("name,dt,tau,bs", [("C1", F16, 6.0, (2, 4, 8)),
                                            ("C2", F16, 8.0, (2, 3, 4, 6, 8)),
                                            ("C4", BF16, 10.0, (2, 3, 4, 5, 6, 8))])
@pytest.mark.parametrize("eps", [0.05, 0.2])
def test_round_trip_against_independent_decode(oracle, name, dt, tau, bs, eps):
    import torch
    x = synth.make(name) if name == "C1" else (synth.make_c2(48) if name == "C2" else synth.make_c4(40))
    T, H = x.shape
    c = oracle.compress(x, dt, tau, bs, eps, REL)
    y = oracle.decompress(c)
    v = np_widen(x, dt)
    is_out = ~(np.abs(v) < np.float32(tau))
    assert c.nnz == int(is_out.sum())
    assert np.array_equal(y[is_out], x[is_out])                     # outliers: bit-exact
    # independent decode: numpy unpackbits + fp32 multiply + library narrowing
    for t in range(T):
        b = int(c.bits[t])
        assert b in bs
        row = c.payload[int(c.pay_off[t]): int(c.pay_off[t + 1])]
        bitsm = np.unpackbits(row, bitorder="little")[: H * b].reshape(H, b).astype(np.uint32)
        code = (bitsm << np.arange(b, dtype=np.uint32)[None, :]).sum(axis=1)
        mag = (code & (2 ** (b - 1) - 1)).astype(np.float32)
        sgn = np.where(code >> (b - 1), np.float32(-1), np.float32(1))
        val = sgn * (mag * c.scale[t])
        if dt == F16:
            ref = val.astype(np.float16).view(np.uint16)
        else:
            ref = torch.from_numpy(val).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        inl = ~is_out[t]
        assert np.array_equal(y[t][inl], ref[inl])
        assert not code[is_out[t]].any()                            # outlier slots carry code 0
        # canonical zero: no negative zero codes
        assert not np.any((code >> (b - 1) == 1) & (code & (2 ** (b - 1) - 1) == 0))
        # inlier error: half a step, plus the rounding of the 16-bit store
        s = float(c.scale[t])
        yv = np_widen(y[t], dt).astype(np.float64)
        ulp_out = np.abs(yv) * (2.0 ** -11 if dt == F16 else 2.0 ** -8)
        assert np.all(np.abs(v[t].astype(np.float64) - yv)[inl] <= (0.5 + 1e-4) * s + ulp_out[inl])
        # sign of every non-zero decoded inlier equals the input's sign
        nz = inl & (yv != 0)
        assert np.array_equal(np.signbit(yv[nz]), np.signbit(v[t][nz]))
    assert oracle.compressed_bytes(c) == (128 + 5 * T + 16 * (T + 1)
                                          + sum(4 * ((H * int(b) + 31) // 32) for b in c.bits)
                                          + 4 * c.nnz)
    if H % 32 == 0:
        assert c.payload_bytes == sum(H * int(b) // 8 for b in c.bits)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_edge_rows_round_trip(oracle, dt):
    d = F16 if dt == "f16" else BF16
    tau = 6.0
    x = synth.edge_rows(264, dt, tau)
    for mode, bud in ((REL, 0.05), (LSB, 0.2), (REL, 0.5)):
        c = oracle.compress(x, d, tau, (2, 4, 5, 8), bud, mode)
        y = oracle.decompress(c)
        v = np_widen(x, d)
        is_out = ~(np.abs(v) < np.float32(tau))
        assert np.array_equal(np.diff(c.row_ptr).astype(np.int64), is_out.sum(axis=1))
        assert np.array_equal(y[is_out], x[is_out])                 # incl. NaN payloads, +-Inf
        assert c.info["cnt"][1] == 264 and c.scale[1] == 0          # all-outlier row
        assert not y[0].any() and c.bits[0] == 2                    # all-zero row -> min B, +0
        assert c.info["cnt"][2] == len(range(0, 264, 7)) + len([j for j in range(3, 264, 11) if j % 7])
        assert c.info["cnt"][3] == 0                                # one ulp below tau stays inside
        yv = np_widen(y, d)
        assert not np.any(np.signbit(yv) & (yv == 0) & ~is_out)     # -0.0 decodes to +0.0


def test_determinism_and_thread_count(oracle):
    x = synth.make_c4(64)
    a = oracle.compress(x, BF16, 10.0, (2, 3, 4, 5, 6, 8), 0.2, REL, nthreads=1)
    b = oracle.compress(x, BF16, 10.0, (2, 3, 4, 5, 6, 8), 0.2, REL, nthreads=4)
    for f in ("bits", "scale", "pay_off", "row_ptr", "payload", "out_col", "out_val"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    assert np.array_equal(oracle.decompress(a, 1), oracle.decompress(b, 3))


def test_side_stream_share_shrinks_with_threshold(oracle):
    # qualitative statement of the paper's size-ratio figure: the lossless side
    # stream is a large share at a small threshold and negligible at a large one
    x = synth.make_c2(tokens=64)
    share = []
    for tau in (1.0, 5.0, 10.0):
        c = oracle.compress(x, F16, tau, (2, 4, 8), 0.05, REL)
        share.append(4 * c.nnz / oracle.compressed_bytes(c))
    assert share[0] > 0.3 and share[0] > share[1] > share[2] and share[2] < 0.05
