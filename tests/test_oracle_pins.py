"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each one checks the oracle
against something that is not the oracle: published known answers, numpy/torch
library routines, closed forms, invariants, higher-precision re-derivations and
brute force on tiny inputs.
"""
import itertools
import math
import os
import subprocess

import numpy as np
import pytest
import torch

import cvlc_synth as syn
from oracle import cvlc_oracle as orc


def _keys(U):
    return U.view(np.uint32) & np.uint32(0x7FFFFFFF)


def _read_kv(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[line[0]] = line[1:]
    return out


# --------------------------------------------------------------------------- Philox
def test_philox_known_answers(golden_dir):
    n = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            assert orc.philox4x32_10(v[0:4], v[4:6]) == tuple(v[6:10])
            n += 1
    assert n == 3


def test_u24_is_word0_top_bits_and_uniform():
    seed = 0x0123456789ABCDEF
    assert orc.u24(seed, 7, 11) == orc.philox4x32_10([11, 7, 0, 0], [0x89ABCDEF, 0x01234567])[0] >> 8
    draws = np.array([orc.u24(2402, 3, i) for i in range(1 << 15)])
    assert draws.max() < (1 << 24)
    counts = np.bincount(draws >> 18, minlength=64)
    expected = draws.size / 64
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert chi2 < 130  # 63 dof, p ~ 1e-6
    # different clients and seeds give different streams
    assert orc.u24(2402, 4, 0) != orc.u24(2402, 3, 0)
    assert orc.u24(2403, 3, 0) != orc.u24(2402, 3, 0)


# --------------------------------------------------------------------------- sizes the paper states
def test_position_id_width(golden_dir):
    const = _read_kv(os.path.join(golden_dir, "paper_constants.txt"))
    assert orc.s_bits(10_000_000) == int(const["s_bits_at_10M_params"][0])
    for d in [1, 2, 3, 4, 5, 255, 256, 257, 65_536, 65_537, 1_200_000, 11_200_000, 25_600_000, 2**31 - 1]:
        assert orc.s_bits(d) == max(1, math.ceil(math.log2(d)))
    assert [orc.s_bits(d) for d in (65_536, 1_200_000, 11_200_000, 25_600_000)] == [16, 21, 24, 25]


def test_kmax_of_a_1500_byte_packet(golden_dir):
    """k_max = R(b-H)/(s+1): at one bit per update a 1500-byte packet of a 10M
    model holds fewer than 480 updates; with our 128-bit H it holds 474."""
    const = _read_kv(os.path.join(golden_dir, "paper_constants.txt"))
    b = int(const["packet_bytes"][0]) * 8
    for R in (1, 3, 10):
        p = orc.plan_budget(10_000_000, 256 + R * b, [1] * R)
        assert p.counts() == [(b - 128) // 25] * R
        assert p.k < int(const["kmax_per_packet_bound"][0]) * R
        assert p.k >= R * int(const["kmin_per_packet"][0])


def test_config_plans_match_closed_forms(golden_dir):
    g = _read_kv(os.path.join(golden_dir, "config_sizes.txt"))
    p1 = orc.plan_for(syn.WORKLOADS[1])
    assert p1.counts() == [int(v) for v in g["cfg1_counts"]]
    assert p1.total_bits == 8 * int(g["cfg1_stream_bytes"][0])
    p4 = orc.plan_for(syn.WORKLOADS[4])
    assert p4.counts() == [int(v) for v in g["cfg4_counts"]]
    assert p4.total_bits == int(g["cfg4_total_bits"][0])
    assert p4.total_bits <= syn.WORKLOADS[4].budget_bits()


def _total_bits_closed_form(d, counts, code_len):
    s = max(1, math.ceil(math.log2(d)))
    return 32 * (8 + 4 * len(counts) + sum(-(-P * (s + y) // 32) for P, y in zip(counts, code_len)))


def test_budget_accounting_and_maximality():
    rng = np.random.default_rng(5)
    for _ in range(200):
        d = int(rng.integers(64, 5_000_000))
        R = int(rng.integers(1, 12))
        y = sorted(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 32], size=R).tolist(), reverse=True)
        budget = int(d * rng.uniform(0.05, 3.0)) + 256 + 160 * R
        p = orc.plan_budget(d, budget, y)
        s = orc.s_bits(d)
        assert p.total_bits == _total_bits_closed_form(d, p.counts(), y)
        assert p.total_bits <= budget
        b = 32 * ((budget - 256) // (32 * R))
        left = d
        for P, yr in zip(p.counts(), y):
            assert 32 * (-(-P * (s + yr) // 32)) + 128 <= b      # Eq. (3) per group
            assert (P + 1) * (s + yr) + 128 > b or P == left      # one more record would not fit
            left -= P
    with pytest.raises(orc.OracleError) as e:
        orc.plan_budget(1000, 256 + 3 * 128, [4, 2, 1])           # no room for a single record
    assert e.value.code == orc.ERR_BUDGET


def test_stream_length_equals_plan_bits():
    U = syn.update_vector(1, 0, d=5000)
    for y, frac in [((8, 4, 2), (0.1, 0.15, 0.25)), ((16,), (1.0,)), ((32, 3), (0.01, 0.2)), ((5, 5, 1), (0.0, 0.3, 0.0))]:
        p = orc.plan_fractions(5000, y, frac)
        enc = orc.encode(U, p, 1, 0)
        assert enc.words.size * 32 == p.total_bits == _total_bits_closed_form(5000, p.counts(), y)
        assert int(enc.words[7]) == enc.words.size
    with pytest.raises(orc.OracleError) as e:
        orc.encode(U, p, 1, 0, cap_words=p.total_words - 1)
    assert e.value.code == orc.ERR_CAPACITY


# --------------------------------------------------------------------------- ranking and grouping
TIE_KINDS = ["all_equal", "all_equal_mixed_sign", "two_valued", "few_levels", "zeros_and_denormals", "all_zero"]


@pytest.mark.parametrize("kind", TIE_KINDS)
def test_rank_matches_lexsort_on_tie_heavy_vectors(kind):
    for d in (1, 2, 63, 64, 65, 1000, 1 << 16):
        U = syn.tie_heavy_vector(kind, d, seed=d)
        key = _keys(U).astype(np.int64)
        ref = np.lexsort((np.arange(d), -key))      # magnitude descending, then index ascending
        assert np.array_equal(orc.rank(U), ref.astype(np.uint32))


def test_rank_distinct_magnitudes_matches_library_topk():
    U = syn.update_vector(1, 3, d=20_000)
    key = _keys(U)
    assert np.unique(key).size == key.size or True
    order = orc.rank(U)
    for k in (1, 17, 2000, 19_999):
        top = torch.topk(torch.from_numpy(np.abs(U).astype(np.float64)), k).indices.numpy()
        kth = np.sort(key)[::-1][k - 1]
        if (key == kth).sum() == 1:                      # boundary not tied: the set is unique
            assert set(order[:k].tolist()) == set(top.tolist())
    mags = np.abs(U[order].astype(np.float64))
    assert np.all(mags[:-1] >= mags[1:])


@pytest.mark.parametrize("kind", TIE_KINDS + ["laplace"])
def test_segments_partition_by_rank(kind):
    d = 4096
    U = syn.update_vector(1, 1, d=d) if kind == "laplace" else syn.tie_heavy_vector(kind, d, seed=1)
    p = orc.plan_manual(d, [8, 4, 4, 1], [100, 0, 1500, 901])
    seg = orc.segments(U, p)
    key = _keys(U).astype(np.int64)
    ref_order = np.lexsort((np.arange(d), -key))
    ref = np.zeros(d, dtype=np.uint32)
    Z = np.cumsum([0] + p.counts())
    for r in range(p.R):
        ref[ref_order[Z[r]:Z[r + 1]]] = r + 1
    assert np.array_equal(seg, ref)
    assert [int((seg == r + 1).sum()) for r in range(p.R)] == p.counts()
    present = [r for r in range(1, p.R + 1) if (seg == r).any()] + ([0] if (seg == 0).any() else [])
    for a, b in zip(present[:-1], present[1:]):          # larger magnitudes in earlier groups
        assert key[seg == a].min() >= key[seg == b].max()


# --------------------------------------------------------------------------- the two special cases of Sec. I
def test_one_group_of_raw_values_plus_zero_tail_is_topk():
    U = syn.update_vector(2, 0, d=30_000)
    for k in (1, 10, 3000):
        p = orc.plan_manual(U.size, [32], [k])
        out = orc.decode_aggregate([orc.encode(U, p, 9, 0).words], U.size)
        idx = torch.topk(torch.from_numpy(np.abs(U)), k).indices.numpy()
        ref = np.zeros_like(U)
        ref[idx] = U[idx]
        assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))
    # quantised top-k: same support, values within one centroid spacing
    p = orc.plan_manual(U.size, [6], [3000])
    enc = orc.encode(U, p, 9, 0)
    out = orc.decode_aggregate([enc.words], U.size)
    idx = torch.topk(torch.from_numpy(np.abs(U)), 3000).indices.numpy()
    mask = np.zeros(U.size, bool)
    mask[idx] = True
    assert np.all(out[~mask] == 0)
    step = (enc.stats[0].max - enc.stats[0].min) / 63
    assert np.abs(out[mask] - U[mask]).max() <= step * (1 + 1e-5)


@pytest.mark.parametrize("y", [1, 2, 5, 8, 12, 16])
def test_single_code_length_is_plain_stochastic_quantisation(y):
    """One group holding every coordinate: the CIDs are those of a textbook
    stochastic uniform quantiser, evaluated here in float64 from the same
    uniforms.  fp32 rounding may move a value across a decision boundary, so
    the two may differ by one level on a tiny fraction of coordinates."""
    U = syn.update_vector(1, 2, d=20_000)
    d = U.size
    p = orc.plan_manual(d, [y], [d])
    enc = orc.encode(U, p, 77, 5, debug=True)
    assert np.all(enc.seg == 1)
    L1 = (1 << y) - 1
    x = U.astype(np.float64)
    m, M = x.min(), x.max()
    t = (x - m) / (M - m) * L1
    lower = np.floor(t)
    u = np.array([orc.u24(77, 5, i) for i in range(d)], dtype=np.float64) / 2.0**24
    ref = np.minimum(lower + (u < (t - lower)), L1).astype(np.int64)
    diff = enc.cid.astype(np.int64) - ref
    assert np.abs(diff).max() <= 1
    assert (diff != 0).mean() < 2e-3
    assert enc.stats[0].min == U.min() and enc.stats[0].max == U.max()


# --------------------------------------------------------------------------- quantiser
def test_quantiser_deterministic_invariants():
    rng = np.random.default_rng(3)
    for y in (1, 2, 3, 7, 8, 15, 16):
        L1 = (1 << y) - 1
        for _ in range(300):
            m, M = np.sort(rng.normal(0, 1, 2).astype(np.float32))
            x = np.float32(rng.uniform(m, M))
            u = int(rng.integers(0, 1 << 24))
            cid = orc.quantise(float(x), float(m), float(M), y, u)
            assert 0 <= cid <= L1
            step = (float(M) - float(m)) / L1
            assert abs(orc.dequantise(cid, float(m), float(M), y) - float(x)) <= step * (1 + 1e-4) + 1e-12
            assert orc.quantise(float(m), float(m), float(M), y, u) == 0
            assert orc.quantise(float(M), float(m), float(M), y, u) == L1
            # the two candidate centroids bracket x
            lo = orc.quantise(float(x), float(m), float(M), y, (1 << 24) - 1)
            hi = orc.quantise(float(x), float(m), float(M), y, 0)
            assert hi - lo in (0, 1) and cid in (lo, hi)
    # a single-valued group has one centroid and decodes exactly
    assert orc.quantise(0.3, 0.3, 0.3, 4, 0) == 0
    assert orc.dequantise(0, np.float32(0.3), np.float32(0.3), 4) == float(np.float32(0.3))
    # raw 32-bit code keeps the bits
    v = np.float32(-1.2345e-7)
    assert orc.quantise(float(v), 0.0, 0.0, 32, 5) == int(v.view(np.uint32))


def test_quantiser_unbiased_mse_closed_form_and_lemma1():
    """E[x~] = x (Sec. IV-B), E||x~-x||^2 = sum step^2 p(1-p) <= P/(2^y-1)^2 ||x||^2 (PQ bound,
    Appendix case study), and the decomposition (a) in the proof of Lemma 1."""
    d, y, n_seeds, B = 48, 3, 6000, 2.0
    U = syn.update_vector(1, 9, d=d)
    p = orc.plan_manual(d, [y], [d])
    L1 = (1 << y) - 1
    x = U.astype(np.float64)
    m, M = x.min(), x.max()
    step = (M - m) / L1
    t = (x - m) / step
    frac = t - np.floor(t)
    dec = np.empty((n_seeds, d))
    for seed in range(n_seeds):
        dec[seed] = orc.decode_aggregate([orc.encode(U, p, seed, 0).words], d)
    mean = dec.mean(axis=0)
    sd = step * np.sqrt(frac * (1 - frac) / n_seeds)
    assert np.all(np.abs(mean - x) <= 5 * sd + 1e-9)
    mse = ((dec - x) ** 2).sum(axis=1).mean()
    closed = (step**2 * frac * (1 - frac)).sum()
    assert abs(mse - closed) <= 0.05 * closed
    assert mse <= d / L1**2 * (x**2).sum()
    lhs = ((dec / B - x) ** 2).sum(axis=1).mean()
    rhs = mse / B**2 + (1 - 1 / B) ** 2 * (x**2).sum()
    assert abs(lhs - rhs) <= 0.02 * rhs
    assert lhs <= (d / L1**2 + (B - 1) ** 2) / B**2 * (x**2).sum()


# --------------------------------------------------------------------------- bit layout
def _bits_of(words):
    return np.unpackbits(words.astype("<u4").view(np.uint8), bitorder="little")


def _field(bits, pos, n):
    return int(sum(int(b) << i for i, b in enumerate(bits[pos:pos + n])))


def test_bit_layout_by_independent_field_extraction():
    d = 3000
    U = syn.update_vector(1, 4, d=d)
    code_len, counts = [16, 7, 3, 1], [5, 333, 0, 1001]
    p = orc.plan_manual(d, code_len, counts, B=1.5)
    enc = orc.encode(U, p, 123, 42, debug=True)
    w, bits, s = enc.words, _bits_of(enc.words), 12
    assert w[0] == 0x434C5643 and w[0].tobytes() == b"CVLC"
    assert (w[1], w[2], w[3], w[4], w[6], w[7]) == (1, d, 4, s, 42, w.size)
    assert w[5] == np.float32(1.5).view(np.uint32)
    pos = 32 * (8 + 4 * 4)
    used = np.zeros(bits.size, bool)
    used[:pos] = True
    for r, (y, P) in enumerate(zip(code_len, counts)):
        hdr = w[8 + 4 * r: 12 + 4 * r]
        members = np.flatnonzero(enc.seg == r + 1)
        assert hdr[0] == y and hdr[1] == P == members.size
        if P:
            assert hdr[2] == U[members].min().view(np.uint32) and hdr[3] == U[members].max().view(np.uint32)
        else:
            assert hdr[2] == 0 and hdr[3] == 0
        W = s + y
        for e in range(P):
            assert _field(bits, pos + e * W, s) == members[e]              # ascending position IDs
            assert _field(bits, pos + e * W + s, y) == enc.cid[members[e]]
        used[pos: pos + P * W] = True
        pos += 32 * (-(-P * W // 32))
    assert pos == bits.size
    assert not bits[~used].any()                                           # padding is zero


def test_signed_zero_extremes_do_not_depend_on_order():
    for U in (np.array([0.0, -0.0, 0.0], np.float32), np.array([-0.0, 0.0, -0.0], np.float32)):
        enc = orc.encode(U, orc.plan_manual(3, [4], [3]), 1, 0)
        assert enc.words[10] == 0x80000000 and enc.words[11] == 0      # min = -0, max = +0
        assert np.array_equal(orc.decode_aggregate([enc.words], 3), np.zeros(3, np.float32))


def test_tiny_vectors_brute_force_roundtrip():
    rng = np.random.default_rng(11)
    for d in (1, 2, 3, 5, 8, 12):
        for R in (1, 2, 3):
            for counts in itertools.product(range(0, d + 1), repeat=R):
                if sum(counts) > d or rng.random() > 0.25:
                    continue
                y = sorted(rng.choice([1, 2, 3, 8, 16, 32], size=R).tolist(), reverse=True)
                U = rng.normal(0, 1, d).astype(np.float32)
                if d > 2:
                    U[1] = -U[0]                                    # a tie across signs
                p = orc.plan_manual(d, y, list(counts))
                enc = orc.encode(U, p, int(rng.integers(1 << 40)), 1, debug=True)
                pid, cid, seg = orc.unpack(enc.words, d)
                order = np.lexsort((np.arange(d), -_keys(U).astype(np.int64)))
                Z = np.cumsum((0,) + counts)
                exp_pid = np.concatenate([np.sort(order[Z[r]:Z[r + 1]]) for r in range(R)] + [np.empty(0, np.int64)])
                assert np.array_equal(pid, exp_pid.astype(np.uint32))
                assert np.array_equal(cid, enc.cid[pid]) and np.array_equal(seg, enc.seg[pid])
                out = orc.decode_aggregate([enc.words], d)
                kept = np.zeros(d, bool)
                kept[pid] = True
                assert np.all(out[~kept] == 0)
                for r in range(R):
                    mem = pid[seg == r + 1]
                    if mem.size == 0:
                        continue
                    if y[r] == 32:
                        assert np.array_equal(out[mem], U[mem])
                    else:
                        step = (float(U[mem].max()) - float(U[mem].min())) / ((1 << y[r]) - 1)
                        assert np.abs(out[mem].astype(np.float64) - U[mem]).max() <= step * (1 + 1e-4) + 1e-12


# --------------------------------------------------------------------------- decode / aggregate
def test_decode_aggregate_is_the_weighted_sum_of_single_decodes():
    d, n = 6000, 5
    streams, singles, Bs = [], [], [1.0, 2.0, 1.0, 4.0, 1.25]
    for c in range(n):
        U = syn.update_vector(2, c, d=d)
        p = orc.plan_fractions(d, [8, 4, 2], [0.02 * (c + 1), 0.05, 0.1], B=Bs[c])
        enc = orc.encode(U, p, 31337, c)
        streams.append(enc.words)
        singles.append(orc.decode_aggregate([enc.words], d, weights=[1.0]).astype(np.float64))
    ref = sum(s / (n * B) for s, B in zip(singles, Bs))                 # average of U~/B
    out = orc.decode_aggregate(streams, d)
    assert np.allclose(out, ref, rtol=1e-6, atol=0)
    wts = [0.5, -1.0, 2.0, 0.25, 3.0]
    ref = sum(np.float32(w).astype(np.float64) * s for w, s in zip(wts, singles))
    out = orc.decode_aggregate(streams, d, weights=wts)
    assert np.array_equal(out, ref.astype(np.float32))
    # streamed aggregation in two batches equals one call when the partial sum is exact in fp32
    a = orc.decode_aggregate(streams[:1], d, weights=wts[:1])
    b = orc.decode_aggregate(streams[1:], d, weights=wts[1:], out=a.copy())
    assert np.allclose(b, out, rtol=1e-6, atol=1e-12)
    # disjoint supports: nothing to add up, values pass through exactly
    U = syn.update_vector(1, 0, d=d)
    U1, U2 = U.copy(), U.copy()
    U1[d // 2:] = 0
    U2[: d // 2] = 0
    p = orc.plan_manual(d, [32], [d // 4])
    out = orc.decode_aggregate([orc.encode(U1, p, 1, 0).words, orc.encode(U2, p, 1, 1).words], d, weights=[1.0, 1.0])
    both = orc.decode_aggregate([orc.encode(U1, p, 1, 0).words], d, weights=[1.0]) + \
        orc.decode_aggregate([orc.encode(U2, p, 1, 1).words], d, weights=[1.0])
    assert np.array_equal(out, both)
    assert np.array_equal(orc.decode_aggregate([], d), np.zeros(d, np.float32))


def test_malformed_input_is_rejected():
    d = 500
    U = syn.update_vector(1, 0, d=d)
    p = orc.plan_fractions(d, [4], [0.2])
    for bad in (np.nan, np.inf, -np.inf):
        V = U.copy()
        V[17] = bad
        with pytest.raises(orc.OracleError) as e:
            orc.encode(V, p, 1, 0)
        assert e.value.code == orc.ERR_NONFINITE
    good = orc.encode(U, p, 1, 0).words
    cases = []
    w = good.copy(); w[0] ^= 1; cases.append(w)                      # magic
    w = good.copy(); w[2] = d + 1; cases.append(w)                   # other model size
    w = good.copy(); w[8] = 17; cases.append(w)                      # unsupported code length
    w = good.copy(); w[9] += 1; cases.append(w)                      # count does not match the length
    cases.append(good[:-1].copy())                                   # truncated
    w = good.copy(); w[12] |= (1 << 9) - 1; cases.append(w)          # first PID = 511 >= d
    w = good.copy(); w[12:14] = good[20:22]; cases.append(w)         # positions no longer ascending
    for w in cases:
        with pytest.raises(orc.OracleError) as e:
            orc.decode_aggregate([w], d)
        assert e.value.code == orc.ERR_STREAM
    for counts, y in (([d + 1], [4]), ([10, 10], [2, 4]), ([10], [17]), ([10], [0])):
        with pytest.raises(orc.OracleError) as e:
            orc.plan_manual(d, y, counts)
        assert e.value.code == orc.ERR_PLAN


# --------------------------------------------------------------------------- planner (Proposition 2, Algorithm 1)
def _gamma_eq5(d, counts, code_len, alpha, B=1.0, qsgd=False):
    """Eq. (5) typed from the paper, in Python floats; Q from the appendix case study."""
    beta = 2 * alpha + 1
    pw = lambda z: max(z, 1.0) ** beta
    k = sum(counts)
    g = (pw(d) - pw(k + 1)) / (pw(d) - 1)
    Z = 0
    for P, y in zip(counts, code_len):
        if P:
            levels = 2.0 ** (y - 1) - 1 if qsgd else 2.0**y - 1
            Q = min(P / levels**2, math.sqrt(P) / levels) if qsgd else P / levels**2
            g += (Q / B**2 + (1 - 1 / B) ** 2) * (pw(Z + P) - pw(Z)) / (pw(d) - 1)
        Z += P
    return g


def test_gamma_matches_equation_5():
    for alpha in (-0.9, -0.55, -0.2):
        for B in (1.0, 3.0):
            p = orc.plan_manual(100_000, [10, 6, 2], [100, 1000, 20_000], B=B)
            assert math.isclose(orc.gamma(p, alpha), _gamma_eq5(100_000, p.counts(), p.code_len(), alpha, B), rel_tol=1e-10)
    # beta = 2 alpha + 1 = 0 is the logarithmic limit of the same expression
    p = orc.plan_manual(100_000, [10, 6, 2], [100, 1000, 20_000])
    assert math.isclose(orc.gamma(p, -0.5), _gamma_eq5(100_000, p.counts(), p.code_len(), -0.5 + 1e-7), rel_tol=1e-5)
    # keeping everything at 32 raw bits leaves (almost) no error and never a negative one (with k = d no rank
    # is sparsified: the first term is 0, not minus the share of a rank d + 1); dropping everything leaves all of it
    assert 0.0 <= orc.gamma(orc.plan_manual(1000, [32], [1000]), -0.5) < 1e-12
    assert 0.0 <= orc.gamma(orc.plan_manual(1000, [32], [1000]), -0.2) < 1e-12
    assert math.isclose(orc.gamma(orc.plan_manual(1000, [], []), -0.5), 1.0, rel_tol=1e-12)


@pytest.mark.parametrize("alpha", [-0.9, -0.6, -0.3])
def test_algorithm1_plan_is_feasible_monotone_and_near_the_integer_optimum(alpha):
    d, budget = 200_000, 150_000
    s = orc.s_bits(d)
    for R in (1, 2, 3):
        p = orc.plan_alg1(d, budget, R, alpha)
        assert p.total_bits <= budget
        y, P = p.code_len(), p.counts()
        assert all(a >= b for a, b in zip(y[:-1], y[1:]))           # Eq. (4): P_1 <= ... <= P_R
        assert all(a <= b for a, b in zip(P[:-1], P[1:]))
        u = 32 * ((budget - 256) // (32 * R)) - 128
        assert all(Pr == u // (s + yr) for Pr, yr in zip(P, y))      # Eq. (3) tight
        best = min(_gamma_eq5(d, [u // (s + yr) for yr in ys], ys, alpha)
                   for ys in itertools.combinations_with_replacement(range(16, 0, -1), R))
        got = _gamma_eq5(d, P, y, alpha)
        assert got <= best * 1.05 + 1e-12
        if R == 1:                                                   # the P_y Top_k family of Sec. V: picks its best y
            assert math.isclose(got, best, rel_tol=1e-9)


@pytest.mark.parametrize("alpha", [-0.8, -0.4])
def test_algorithm1_with_the_qsgd_error_model(alpha):
    """The same sweep priced with QSGD's Q(P_r) = min(P/s^2, sqrt(P)/s): feasible, monotone, Eq. (3)
    tight, no code shorter than sign + one level bit, and near the best integer assignment."""
    d, budget = 200_000, 150_000
    s = orc.s_bits(d)
    for R in (1, 2, 3):
        p = orc.plan_alg1(d, budget, R, alpha, quant=orc.QSGD)
        assert p.quant == orc.QSGD and p.total_bits <= budget
        y, P = p.code_len(), p.counts()
        assert min(y) >= 2 and all(a >= b for a, b in zip(y[:-1], y[1:]))
        u = 32 * ((budget - 256) // (32 * R)) - 128
        assert all(Pr == u // (s + yr) for Pr, yr in zip(P, y))
        assert math.isclose(orc.gamma(p, alpha), _gamma_eq5(d, P, y, alpha, qsgd=True), rel_tol=1e-10)
        best = min(_gamma_eq5(d, [u // (s + yr) for yr in ys], ys, alpha, qsgd=True)
                   for ys in itertools.combinations_with_replacement(range(16, 1, -1), R))
        got = _gamma_eq5(d, P, y, alpha, qsgd=True)
        assert got <= best * 1.05 + 1e-12
        if R == 1:
            assert math.isclose(got, best, rel_tol=1e-9)


def _gamma_eq5_many(d, s, u, ys, alpha):
    """Eq. (5) for many code-length vectors at once (rows of `ys`), PQ, B = 1, Eq. (3) tight:
    P_r = floor(u / (s + y_r)).  numpy, typed from the equation as _gamma_eq5 is."""
    beta = 2 * alpha + 1
    ys = np.asarray(ys, dtype=np.float64)
    P = np.floor(u / (s + ys))
    Z = np.cumsum(P, axis=1)
    Zp = np.maximum(Z - P, 1.0)
    Q = P / (2.0**ys - 1.0) ** 2
    den = float(d) ** beta - 1.0
    tail = (float(d) ** beta - (Z[:, -1] + 1.0) ** beta) / den
    g = tail + (Q * (np.maximum(Z, 1.0) ** beta - Zp**beta)).sum(axis=1) / den
    g[Z[:, -1] > d] = np.inf
    return g


@pytest.mark.parametrize("alpha", [-0.9, -0.6, -0.3])
@pytest.mark.parametrize("d,budget", [(200_000, 150_000), (1_200_000, 1_800_000)])
def test_algorithm1_plan_against_every_integer_plan_up_to_six_groups(d, budget, alpha):
    """Sec. IV-C problem P2 by exhaustion: all non-increasing integer code-length vectors (54 264 of
    them at R = 6), each with Eq. (3) tight.  The sweep works on real-valued P_r and rounds at the
    end, so it may miss the integer optimum by one step of one code length; in gamma that is below
    one part in a thousand."""
    s = orc.s_bits(d)
    for R in (4, 5, 6):
        p = orc.plan_alg1(d, budget, R, alpha)
        u = 32 * ((budget - 256) // (32 * R)) - 128
        ys = np.array(list(itertools.combinations_with_replacement(range(16, 0, -1), R)))
        g = _gamma_eq5_many(d, s, u, ys, alpha)
        best = float(g.min())
        assert math.isclose(best, _gamma_eq5(d, [u // (s + int(y)) for y in ys[g.argmin()]], ys[g.argmin()].tolist(), alpha),
                            rel_tol=1e-9)                              # the vectorised form agrees with the scalar one
        got = _gamma_eq5(d, p.counts(), p.code_len(), alpha)
        assert best * (1 - 1e-12) <= got <= best * 1.001, (R, p.code_len(), ys[g.argmin()].tolist())


def _gamma_real(P, d, u, s, alpha, B=1.0):
    """Eq. (5) for real-valued group sizes with y_r = u / P_r - s (PQ)."""
    beta = 2 * alpha + 1
    pw = lambda z: max(z, 1.0) ** beta
    g = (pw(d) - pw(sum(P) + 1)) / (pw(d) - 1)
    Z = 0.0
    for Pr in P:
        Q = Pr / (2.0 ** (u / Pr - s) - 1.0) ** 2
        g += (Q / B**2 + (1 - 1 / B) ** 2) * (pw(Z + Pr) - pw(Z)) / (pw(d) - 1)
        Z += Pr
    return g


@pytest.mark.parametrize("d,budget,R", [(200_000, 150_000, 4), (1_200_000, 1_800_000, 7),
                                        (11_200_000, 11_200_000, 15), (25_600_000, 30_000_000, 31)])
def test_sweep_of_atomic_operations_reaches_the_minimiser_of_gamma(d, budget, R):
    """Theorem 1: for fixed k the point at which every pair (P_{r-1}, P_r) minimises Eq. (6) minimises
    gamma of Eq. (5) and has P_1 <= ... <= P_R.  Checked against a general constrained minimiser
    (SLSQP over all P_r at once, sum P_r = k) that knows nothing of pairs, at the group counts of the
    workloads, for k in the part of [k_min, k_max] where the best plans lie."""
    from scipy.optimize import minimize

    s = orc.s_bits(d)
    u = 32 * ((budget - 256) // (32 * R)) - 128
    kmax = R * u / (s + 1)
    for alpha in (-0.9, -0.6, -0.3):
        for frac in (0.3, 0.6):
            k = R + (kmax - R) * frac
            P, g = orc.alg1_sweep(d, budget, R, alpha, k)
            assert math.isclose(sum(P), k, rel_tol=1e-9)
            assert all(a <= b * (1 + 1e-9) for a, b in zip(P[:-1], P[1:]))          # Eq. (4)
            assert math.isclose(g, _gamma_real(P, d, u, s, alpha), rel_tol=1e-9)
            res = minimize(lambda x: math.log(_gamma_real(list(x), d, u, s, alpha)), np.full(R, k / R), method="SLSQP",
                           constraints=[{"type": "eq", "fun": lambda x: x.sum() - k}], bounds=[(1.0, u / (s + 1))] * R,
                           options={"maxiter": 500, "ftol": 1e-14})
            assert g <= _gamma_real(list(res.x), d, u, s, alpha) * (1 + 2e-5), (alpha, frac)
            # and no transfer between two neighbouring groups lowers gamma (stationarity, step of 1 update and of 1 %)
            for r in range(1, R):
                for step in (1.0, 0.01 * P[r - 1]):
                    for sign in (-1.0, 1.0):
                        Q = list(P)
                        Q[r - 1] -= sign * step
                        Q[r] += sign * step
                        if min(Q[r - 1], Q[r]) >= 1.0 and max(Q[r - 1], Q[r]) <= u / (s + 1):
                            assert _gamma_real(Q, d, u, s, alpha) >= g * (1 - 1e-6), (alpha, frac, r, step, sign)


@pytest.mark.parametrize("cfg,R", [(2, 7), (3, 15), (5, 31)])
def test_algorithm1_plans_of_the_workloads_are_locally_optimal_and_beat_fixed_length_plans(cfg, R):
    """At the workloads' sizes and group counts (exhaustion is out of reach): Eq. (3) tight and Eq. (4)
    in every plan; Theorem 1's ordering; no single code length moved by one bit (sizes refilled by
    Eq. (3), order kept) lowers gamma by more than the rounding of the real-valued solution can
    cost (5e-4 relative); and gamma is below that of every plan with one code length for all
    groups, the P_y Top_k family the paper compares with (Sec. V)."""
    w = syn.WORKLOADS[cfg]
    d, s = w.d, orc.s_bits(w.d)
    for client in (0, 1) if cfg == 5 else (0,):                      # cfg 5: two of the per-client budgets
        budget = w.budget_bits(client)
        u = 32 * ((budget - 256) // (32 * R)) - 128
        for alpha in ((-0.9, -0.55) if cfg == 5 else (-0.9, -0.7, -0.55, -0.3)):   # a 31-group plan takes seconds
            p = orc.plan_alg1(d, budget, R, alpha)
            y, P = p.code_len(), p.counts()
            assert p.total_bits <= budget and p.R == R
            assert all(a >= b for a, b in zip(y[:-1], y[1:])) and all(a <= b for a, b in zip(P[:-1], P[1:]))
            assert all(Pr == u // (s + yr) for Pr, yr in zip(P, y))
            g0 = _gamma_eq5(d, P, y, alpha)
            assert math.isclose(orc.gamma(p, alpha), g0, rel_tol=1e-10)
            for r in range(R):
                for step in (-1, 1):
                    y2 = list(y)
                    y2[r] += step
                    if not 1 <= y2[r] <= 16 or any(a < b for a, b in zip(y2[:-1], y2[1:])):
                        continue
                    P2 = [u // (s + yy) for yy in y2]
                    if sum(P2) <= d:
                        assert _gamma_eq5(d, P2, y2, alpha) >= g0 * (1 - 5e-4), (alpha, r, step)
            for yy in range(1, 17):
                if R * (u // (s + yy)) <= d:
                    assert g0 <= _gamma_eq5(d, [u // (s + yy)] * R, [yy] * R, alpha) * (1 + 1e-12), (alpha, yy)


def test_alpha_fit_recovers_a_power_law():
    d = 1 << 15
    for alpha in (-0.4, -0.8):
        mags = (np.arange(1, d + 1, dtype=np.float64) ** alpha).astype(np.float32)
        rng = np.random.default_rng(1)
        U = (mags * rng.choice([-1.0, 1.0], d)).astype(np.float32)[rng.permutation(d)]
        assert abs(orc.fit_alpha(U) - alpha) < 1e-3


def test_fit_points_are_order_statistics_at_doubling_ranks():
    """Definition 1 speaks of the l-th largest magnitude: the points of the fit are a
    library sort's entries at l = 1, 2, 4, ... and l = d, whatever d's residue."""
    rng = np.random.default_rng(7)
    for d in (1, 2, 3, 5, 64, 1000, 4097, 65536):
        U = (rng.standard_t(3, d) * 10.0 ** rng.uniform(-5, -2, d)).astype(np.float32)
        U[rng.integers(0, d, d // 7)] = 0.0                       # zeros and ties are ordinary input
        U[rng.integers(0, d, d // 9)] = np.float32(1e-3)
        ranks, keys = orc.fit_points(U)
        want = [1 << j for j in range(32) if (1 << j) < d] + [d]
        assert ranks.tolist() == want
        desc = np.sort(np.abs(U).view(np.uint32))[::-1]
        assert keys.tolist() == [int(desc[l - 1]) for l in want]


def test_alpha_fit_special_cases():
    """Closed forms: a constant vector has slope 0; two usable points give the slope
    between them; fewer than two usable points give the stated default -1."""
    assert orc.fit_alpha(np.full(1000, -2.5, dtype=np.float32)) == pytest.approx(0.0, abs=1e-15)
    U = np.array([8.0, -2.0], dtype=np.float32)                   # ranks 1 and 2
    assert orc.fit_alpha(U) == pytest.approx(math.log(2.0 / 8.0) / math.log(2.0), rel=1e-14)
    assert orc.fit_alpha(np.array([3.0], dtype=np.float32)) == -1.0
    assert orc.fit_alpha(np.zeros(100, dtype=np.float32)) == -1.0
    U = np.zeros(100, dtype=np.float32)
    U[17] = 4.0; U[3] = -1.0                                      # ranks 1, 2 usable, 4 ... 100 are zeros
    assert orc.fit_alpha(U) == pytest.approx(-2.0, rel=1e-14)


def _records(U, plan, enc):
    """(group index 0-based, position, reconstructed value) of every record of an encoded
    stream, through the parser and the single-value dequantiser."""
    pid, cid, seg = orc.unpack(enc.words, plan.d)
    xhat = np.array([orc.dequantise(int(c), enc.stats[int(g) - 1].min, enc.stats[int(g) - 1].max,
                                    plan.code_len()[int(g) - 1]) for c, g in zip(cid, seg)], dtype=np.float32)
    return seg.astype(np.int64) - 1, pid.astype(np.int64), xhat


@pytest.mark.parametrize("B", [1.0, 2.5])
def test_error_energy_is_the_squared_distance_to_the_scaled_reconstruction(B):
    """Sec. IV-B: Uhat = Utilde / B.  The error energy the encoder reports per group equals
    the squared distance between the group's values and their reconstructions read back
    from the stream; the tail is dropped whole."""
    d = 6000
    U = syn.update_vector(3, 1, d=d)
    plan = orc.plan_manual(d, [32, 9, 3, 1], [40, 300, 900, 1500], B=B)
    enc = orc.encode(U, plan, 77, 5)
    grp, pid, xhat = _records(U, plan, enc)
    x = U.astype(np.float64)
    for r in range(plan.R):
        sel = grp == r
        want = float(np.sum((xhat[sel].astype(np.float64) / B - x[pid[sel]]) ** 2))
        assert enc.stats[r].errsq == pytest.approx(want, rel=1e-12, abs=1e-300), r
    assert enc.stats[0].errsq == pytest.approx((1.0 - 1.0 / B) ** 2 * enc.stats[0].sumsq, rel=1e-12)  # raw group
    kept = np.zeros(d, dtype=bool)
    kept[pid] = True
    assert enc.stats[plan.R].errsq == enc.stats[plan.R].sumsq == pytest.approx(float(np.sum(x[~kept] ** 2)), rel=1e-12)


def test_empirical_gamma_is_the_relative_error_of_the_decoded_vector():
    """The left side of Propositions 1 and 2: ||Uhat - U||^2 / ||U||^2, with Uhat the
    parameter server's reconstruction (B = 1, one client: the decoder returns it exactly)."""
    for cfg, d in ((1, 5000), (3, 20000)):
        U = syn.update_vector(cfg, 2, d=d)
        plan = orc.plan_alg1(d, 2 * d, 4, -0.6)
        enc = orc.encode(U, plan, 3, 2)
        Uhat = orc.decode_aggregate([enc.words], d).astype(np.float64)
        x = U.astype(np.float64)
        want = float(np.sum((Uhat - x) ** 2) / np.sum(x ** 2))
        assert orc.empirical_gamma(enc.stats, plan.R) == pytest.approx(want, rel=1e-10)
        assert 0.0 < want < 1.0
    zeros = np.zeros(100, dtype=np.float32)
    enc = orc.encode(zeros, orc.plan_manual(100, [4], [10]), 1, 0)
    assert orc.empirical_gamma(enc.stats, 1) == 0.0


def test_error_energy_obeys_lemma_1():
    """Lemma 1 per group: E||Uhat - Ubar||^2 <= (Q + (B-1)^2) / B^2 ||Ubar||^2 with PQ's
    Q(P, y) = P / (2^y - 1)^2, and step (a) of its proof: the expectation splits into the
    quantisation error over B^2 plus (1 - 1/B)^2 ||Ubar||^2 (the rounding is unbiased)."""
    d, B, seeds = 3000, 3.0, 300
    U = syn.update_vector(1, 0, d=d)
    ys, Ps = [6, 3, 1], [200, 500, 800]
    scaled = orc.plan_manual(d, ys, Ps, B=B)
    plain = orc.plan_manual(d, ys, Ps, B=1.0)
    err_b = np.zeros((seeds, 3))
    err_1 = np.zeros((seeds, 3))
    for s in range(seeds):
        eb, e1 = orc.encode(U, scaled, 1000 + s, 0), orc.encode(U, plain, 1000 + s, 0)
        err_b[s] = [eb.stats[r].errsq for r in range(3)]
        err_1[s] = [e1.stats[r].errsq for r in range(3)]
    energy = np.array([eb.stats[r].sumsq for r in range(3)])
    for r in range(3):
        Q = Ps[r] / (2 ** ys[r] - 1) ** 2
        assert err_b[:, r].max() <= (Q + (B - 1) ** 2) / B ** 2 * energy[r]
        split = err_1[:, r].mean() / B ** 2 + (1 - 1 / B) ** 2 * energy[r]
        spread = err_b[:, r].std() / math.sqrt(seeds)
        assert abs(err_b[:, r].mean() - split) <= 5 * spread + 1e-9 * split


def test_next_round_scale_factor():
    """Footnote to Proposition 1: B = max_r Q(P_r, y_r) + 1, with PQ's Q of the appendix."""
    p = orc.plan_manual(11_200_000, [16, 8, 6, 4, 3, 2, 1], [19995, 24994, 26660, 28564, 29622, 30761, 31992])
    assert orc.next_scale(p) == pytest.approx(31992 / 1.0 + 1.0, rel=1e-15)          # the 1-bit group dominates
    p = orc.plan_manual(100_000, [8, 4], [100, 28564])
    assert orc.next_scale(p) == pytest.approx(28564 / 225.0 + 1.0, rel=1e-15)
    assert orc.next_scale(orc.plan_manual(1000, [32], [100])) == 1.0                  # raw values: no quantisation error
    assert orc.next_scale(orc.plan_manual(1000, [8, 2], [0, 0])) == 1.0
    for R in (1, 5):                                                                  # Proposition 1's condition B > (Q+1)/2
        q = orc.plan_alg1(500_000, 400_000, R, -0.7)
        Bn = orc.next_scale(q)
        assert all(Bn > (P / (2 ** y - 1) ** 2 + 1) / 2 for P, y in zip(q.counts(), q.code_len()) if y != 32)


# --------------------------------------------------------------------------- QSGD, the second quantiser of Sec. IV-D
def _f32_below(v):
    return float(np.nextafter(np.float32(v), np.float32(-np.inf)))


def test_qsgd_norm_is_the_smallest_fp32_whose_square_reaches_the_exact_sum():
    """The header's l2-norm must not depend on the order of a floating-point sum: it is defined
    on the exact sum of squares (rational arithmetic here)."""
    from fractions import Fraction
    rng = np.random.default_rng(19)
    cases = [rng.standard_normal(1000).astype(np.float32),
             (rng.standard_normal(500) * 10.0 ** rng.uniform(-44, 18, 500)).astype(np.float32),   # denormals to 1e18
             np.array([3.0, 4.0], dtype=np.float32),
             np.array([-7.25e-12], dtype=np.float32),
             np.array([1e-45, 1e-45, 1e-45], dtype=np.float32),
             np.full(4096, 0.1, dtype=np.float32),
             np.zeros(17, dtype=np.float32),
             np.array([3.0e38], dtype=np.float32)]
    for x in cases:
        n = orc.qsgd_norm(x)
        S = sum(Fraction(float(v)) ** 2 for v in x)
        assert Fraction(n) ** 2 >= S
        if n > 0.0:
            assert Fraction(_f32_below(n)) ** 2 < S
        assert n >= float(np.abs(x).max())                      # no entry exceeds the norm
        assert n == orc.qsgd_norm(x[::-1].copy())
        assert n == pytest.approx(math.sqrt(math.fsum(float(v) ** 2 for v in x)), rel=2e-7, abs=1e-45)
    assert orc.qsgd_norm(np.array([3.0, 4.0], dtype=np.float32)) == 5.0
    assert orc.qsgd_norm(np.array([-7.25e-12], dtype=np.float32)) == float(np.float32(7.25e-12))
    with pytest.raises(orc.OracleError):                        # the norm itself overflows fp32
        orc.qsgd_norm(np.array([3.0e38, 3.0e38], dtype=np.float32))


def test_qsgd_quantiser_invariants_and_textbook_rule():
    """QSGD's rule (Alistarh et al.): |x|/norm is rounded to a neighbouring level l/s or (l+1)/s,
    up with probability equal to the fractional position; the sign travels beside the level."""
    rng = np.random.default_rng(29)
    for y in (2, 3, 5, 8, 12, 16):
        s = (1 << (y - 1)) - 1
        x = (rng.standard_normal(400) * 10.0 ** rng.uniform(-3, 0, 400)).astype(np.float32)
        norm = orc.qsgd_norm(x)
        u = rng.integers(0, 1 << 24, x.size)
        cid = np.array([orc.quantise_qsgd(float(v), norm, y, int(uu)) for v, uu in zip(x, u)])
        level, sign = cid & s, cid >> (y - 1)
        assert np.all(cid < (1 << y)) and np.all(level <= s)
        assert np.array_equal(sign == 1, np.signbit(x))
        t = np.abs(x.astype(np.float64)) / norm * s
        ref = np.minimum(np.floor(t) + (u / 2.0**24 < t - np.floor(t)), s)
        assert np.abs(level - ref).max() <= 1 and (level != ref).mean() < 0.01      # fp32 vs fp64 at a boundary
        xt = np.array([orc.dequantise_qsgd(int(c), norm, y) for c in cid], dtype=np.float64)
        assert np.all(np.abs(xt - x) <= norm / s * (1 + 1e-5))
        assert np.all(np.signbit(xt) == np.signbit(x))
        lo = np.array([orc.quantise_qsgd(float(v), norm, y, (1 << 24) - 1) for v in x]) & s
        hi = np.array([orc.quantise_qsgd(float(v), norm, y, 0) for v in x]) & s
        assert np.all((hi - lo >= 0) & (hi - lo <= 1)) and np.all((level == lo) | (level == hi))
    one = np.array([-0.75], dtype=np.float32)                    # a single entry sits on the top level exactly
    assert orc.quantise_qsgd(-0.75, orc.qsgd_norm(one), 4, 123) == 7 | 8
    assert orc.dequantise_qsgd(7 | 8, 0.75, 4) == -0.75
    assert orc.quantise_qsgd(0.0, 0.0, 4, 5) == 0 and orc.dequantise_qsgd(3, 0.0, 4) == 0.0   # all-zero group
    v = np.float32(-1.2345e-7)
    assert orc.quantise_qsgd(float(v), 1.0, 32, 5) == int(v.view(np.uint32))
    assert orc.dequantise_qsgd(int(v.view(np.uint32)), 1.0, 32) == float(v)


def test_qsgd_stream_is_unbiased_within_the_published_variance_bound():
    """Through the whole encoder and decoder: E[x~] = x, and E||x~ - x||^2 <= min(P/s^2, sqrt(P)/s) ||x||^2
    (Lemma 3.1 of the QSGD paper; the Q(P_r) of the appendix case study)."""
    d, y, n_seeds = 60, 4, 4000
    U = syn.update_vector(1, 11, d=d)
    p = orc.plan_manual(d, [y], [d], quant=orc.QSGD)
    s = (1 << (y - 1)) - 1
    x = U.astype(np.float64)
    norm = orc.qsgd_norm(U)
    t = np.abs(x) / norm * s
    frac = t - np.floor(t)
    dec = np.empty((n_seeds, d))
    for seed in range(n_seeds):
        dec[seed] = orc.decode_aggregate([orc.encode(U, p, seed, 0).words], d)
    sd = norm / s * np.sqrt(frac * (1 - frac) / n_seeds)
    assert np.all(np.abs(dec.mean(axis=0) - x) <= 5 * sd + 1e-9)
    mse = ((dec - x) ** 2).sum(axis=1).mean()
    closed = ((norm / s) ** 2 * frac * (1 - frac)).sum()
    assert abs(mse - closed) <= 0.05 * closed
    assert mse <= min(d / s**2, math.sqrt(d) / s) * (x**2).sum()


def test_qsgd_stream_layout_and_plan_rules():
    """Header {y, P, norm, 0} per group, quantiser id in the version word, sign above the level;
    a 1-bit code cannot hold a sign and a level."""
    d = 5000
    U = syn.update_vector(3, 4, d=d)
    p = orc.plan_manual(d, [32, 9, 2], [30, 400, 1500], quant=orc.QSGD)
    pq = orc.plan_manual(d, [32, 9, 2], [30, 400, 1500])
    enc = orc.encode(U, p, 5, 1, debug=True)
    assert enc.words[1] >> 16 == 1 and p.total_bits == pq.total_bits
    assert np.array_equal(orc.segments(U, p), orc.segments(U, pq))          # the grouping does not depend on the quantiser
    pid, cid, seg = orc.unpack(enc.words, d)
    out = orc.decode_aggregate([enc.words], d)
    for r, y in enumerate([32, 9, 2]):
        sel = seg == r + 1
        hdr = enc.words[8 + 4 * r: 12 + 4 * r]
        norm = float(hdr[2:3].view(np.float32)[0])
        assert int(hdr[0]) == y and int(hdr[1]) == int(sel.sum()) and int(hdr[3]) == 0
        assert norm == orc.qsgd_norm(U[pid[sel]])
        want = np.array([orc.dequantise_qsgd(int(c), norm, y) for c in cid[sel]], dtype=np.float32)
        assert np.array_equal(out[pid[sel]], want)          # as values: the sum starts from +0, so -0 comes back as +0
        if y != 32:
            assert np.array_equal((cid[sel] >> (y - 1)) == 1, np.signbit(U[pid[sel]]))
    assert np.array_equal(out[pid[seg == 1]], U[pid[seg == 1]])             # raw group
    with pytest.raises(orc.OracleError):
        orc.plan_manual(d, [4, 1], [10, 10], quant=orc.QSGD)
    bad = enc.words.copy()
    bad[8 + 4 + 3] = 1                                                      # second header word of QSGD must be 0
    with pytest.raises(orc.OracleError):
        orc.decode_aggregate([bad], d)
    # the error model of the appendix: min(P/s^2, sqrt(P)/s) with s = 2^(y-1) - 1
    q = orc.plan_manual(100_000, [6, 3], [400, 10_000], quant=orc.QSGD)
    assert orc.next_scale(q) == pytest.approx(1.0 + min(10_000 / 9.0, 100.0 / 3.0), rel=1e-15)


# --------------------------------------------------------------------------- packets (Eq. (3), Sec. IV-D)
def test_packets_obey_the_size_constraint_and_carry_their_own_header():
    """Eq. (3): P (s + y_r) + H <= b for every packet, with the largest P that fits; one code length
    per packet; the fields the paper lists (s, y_r, centroid distribution) are in every packet, read
    here straight from the bits."""
    d = 40_000
    U = syn.update_vector(3, 6, d=d)
    for quant, ys in ((orc.PQ, [32, 9, 4, 1]), (orc.QSGD, [32, 9, 4, 2])):
        p = orc.plan_manual(d, ys, [300, 2500, 0, 9000], B=1.5, quant=quant)
        enc = orc.encode(U, p, 11, 7)
        for mtu in (1500, 256, 9000):
            pk, sizes = orc.packetize(enc.words, d, mtu)
            assert pk.shape[0] == orc.packet_count(p, mtu)
            b, H, s = 8 * mtu, 320, p.s
            pid, cid, seg = orc.unpack(enc.words, d)
            at = 0
            for r, (y, P) in enumerate(zip(ys, p.counts())):
                W = s + y
                cap = (b - H) // W
                assert cap * W + H <= b < (cap + 1) * W + H                   # maximal under Eq. (3)
                npk = max(1, -(-P // cap))
                rec_pid, rec_cid = pid[seg == r + 1], cid[seg == r + 1]
                for j in range(npk):
                    w = pk[at]
                    c = min(cap, P - j * cap)
                    assert int(sizes[at]) == 4 * (10 + -(-c * W // 32)) <= mtu
                    assert w[0] == 0x504C5643 and w[1] == enc.words[1] and w[2] == d and w[3] == 7
                    assert w[4] == enc.words[5]                                # B
                    assert w[5] == r | (4 << 8) | (y << 16) | (s << 24) and w[6] == P and w[7] == j * cap
                    assert w[8] == enc.words[8 + 4 * r + 2] and w[9] == enc.words[8 + 4 * r + 3]
                    bits = _bits_of(w[10:])
                    for e in (0, c // 2, c - 1) if c else ():
                        assert _field(bits, e * W, s) == int(rec_pid[j * cap + e])
                        assert _field(bits, e * W + s, y) == int(rec_cid[j * cap + e])
                    assert not bits[c * W:].any()                              # padding and the slot's tail are zero
                    at += 1
            assert at == pk.shape[0]


def test_packets_reassemble_in_any_order_and_reject_loss_and_tampering():
    d = 25_000
    U = syn.update_vector(1, 3, d=d)
    p = orc.plan_manual(d, [12, 6, 3], [700, 0, 5000])
    enc = orc.encode(U, p, 5, 2)
    pk, _ = orc.packetize(enc.words, d, 1500)
    assert np.array_equal(orc.depacketize(pk, d), enc.words)
    rng = np.random.default_rng(3)
    assert np.array_equal(orc.depacketize(pk[rng.permutation(pk.shape[0])], d), enc.words)
    with pytest.raises(orc.OracleError):
        orc.depacketize(pk[:-1], d)                                            # a packet is missing
    with pytest.raises(orc.OracleError):
        orc.depacketize(np.concatenate([pk, pk[3:4]]), d)                      # one arrives twice
    for word, value in ((0, 1), (2, d - 1), (5, int(pk[4][5]) ^ (1 << 16)), (6, int(pk[4][6]) + 1), (7, 1), (8, 0)):
        bad = pk.copy()
        bad[4][word] = value
        with pytest.raises(orc.OracleError):
            orc.depacketize(bad, d)
    # a stream that is nothing but headers still travels: one packet per (empty) group
    empty = orc.encode(U, orc.plan_manual(d, [8, 2], [0, 0]), 5, 2)
    pk, sizes = orc.packetize(empty.words, d, 1500)
    assert pk.shape[0] == 2 and sizes.tolist() == [40, 40]
    assert np.array_equal(orc.depacketize(pk, d), empty.words)


# --------------------------------------------------------------------------- memory errors and undefined arithmetic
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The oracle compiled with -fsanitize=address,undefined (any finding aborts) and driven through
    every entry point on small inputs: stream buffers of exactly the stream's size, truncated streams,
    lost packets, 31 groups, raw 32-bit and empty groups, both quantisers, the planner's three modes."""
    exe = tmp_path / "oracle_sanitize"
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_sanitize_main.c")
    subprocess.run(["gcc", "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-ffp-contract=off", "-Wall", "-Wextra", "-Werror", "-o", str(exe), src, "-lm"],
                   check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitizer run: ok" in run.stdout
