"""Pins for the oracle's random words, subset sampler and survivor reducer.

Each pin is something other than the oracle itself: published known-answer
vectors, exact combinatorics, brute-force enumeration, the paper's worked
examples (tests/golden/), or a second implementation written in another style.
"""
import math
import os

import numpy as np
import pytest

import oracle
from tests import pyref


# ------------------------------------------------------------------ Philox

def _kat_rows(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(golden_dir):
    rows = _kat_rows(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert list(oracle.philox4x32_10(ctr, key)) == want
        assert pyref.philox4x32_10(ctr, key) == want


def test_philox_matches_second_implementation_on_random_inputs():
    rng = np.random.default_rng(7)
    for _ in range(200):
        ctr = rng.integers(0, 2**32, size=4, dtype=np.uint64)
        key = rng.integers(0, 2**32, size=2, dtype=np.uint64)
        assert list(oracle.philox4x32_10(ctr, key)) == pyref.philox4x32_10(ctr, key)


def test_word_addressing():
    """word i = lane i mod 4 of the block with counter (s, i div 4, unit, stream), key = seed halves."""
    seed = 0x0123456789ABCDEF
    for (stream, unit, s, i) in [(0, 0, 0, 0), (3, 17, 4095, 5), (0xFFFFFFFF, 921599, 65535, 127), (1, 2, 3, 6)]:
        blk = pyref.philox4x32_10([s, i // 4, unit, stream], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.word(seed, stream, unit, s, i) == blk[i % 4]
    # distinct scenarios, units, streams and seeds give distinct words
    ws = {oracle.word(seed, 0, 0, s, 0) for s in range(64)} | {oracle.word(seed, 0, u, 0, 0) for u in range(1, 64)}
    assert len(ws) == 127
    assert oracle.word(seed, 0, 5, 9, 2) != oracle.word(seed, 1, 5, 9, 2)
    assert oracle.word(seed, 0, 5, 9, 2) != oracle.word(seed ^ (1 << 40), 0, 5, 9, 2)


# ------------------------------------------------------------------ subset sampler

@pytest.mark.parametrize("M,k", [(1, 0), (1, 1), (6, 2), (8, 5), (12, 6), (64, 1), (64, 63), (64, 40),
                                 (97, 33), (200, 150), (256, 128), (256, 255), (256, 256), (256, 0)])
def test_sampler_size_and_second_implementation(M, k):
    seed = 0xDEADBEEF12345678
    for s in range(24):
        v = oracle.sample_preempted(M, k, seed, 2, 11, s)
        assert v.shape == (M,) and set(np.unique(v)) <= {0, 1}
        assert int(v.sum()) == k
        assert np.array_equal(v, pyref.floyd_preempted(M, k, seed, 2, 11, s))


@pytest.mark.parametrize("M,k", [(5, 2), (6, 3), (7, 5), (8, 1), (9, 7), (10, 4)])
def test_sampler_uniform_over_all_subsets(M, k):
    """Every k-subset equally likely: chi-square over all C(M, k) subsets (also the complement branch)."""
    n_sub = math.comb(M, k)
    S = 2000 * n_sub
    counts = {}
    seed = 0x5EED0000 + 131 * M + k
    for s in range(S):
        key = oracle.sample_preempted(M, k, seed, 0, 3, s).tobytes()
        counts[key] = counts.get(key, 0) + 1
    assert len(counts) == n_sub
    expected = S / n_sub
    chi2 = sum((c - expected) ** 2 / expected for c in counts.values())
    dof = n_sub - 1
    # chi-square mean dof, variance 2 dof; 6 sigma
    assert chi2 < dof + 6.0 * math.sqrt(2.0 * dof) + 10.0


@pytest.mark.parametrize("M,k", [(64, 7), (64, 50), (256, 64), (130, 100)])
def test_sampler_marginals(M, k):
    """P(instance preempted) = k/M and P(pair preempted) = k(k-1)/(M(M-1))."""
    S = 20000
    acc = np.zeros(M, dtype=np.int64)
    pair = 0
    for s in range(S):
        v = oracle.sample_preempted(M, k, 99, 0, 1, s)
        acc += v
        pair += int(v[0] & v[M - 1]) + int(v[1] & v[M // 2])
    p = k / M
    sd = math.sqrt(p * (1 - p) / S)
    assert np.all(np.abs(acc / S - p) < 5.5 * sd)
    pp = k * (k - 1) / (M * (M - 1))
    sdp = math.sqrt(pp * (1 - pp) / (2 * S))
    assert abs(pair / (2 * S) - pp) < 5.5 * sdp


# ------------------------------------------------------------------ reducer and class rule

def test_reducer_against_array_definition():
    rng = np.random.default_rng(3)
    for D, P in [(1, 1), (2, 3), (3, 2), (3, 4), (7, 5), (16, 16), (4, 64), (256, 1), (1, 256), (13, 7), (5, 32)]:
        for _ in range(30):
            v = (rng.random(D * P) < rng.random()).astype(np.uint8)
            n_int, d_min, occ = oracle.reduce(D, P, v)
            assert (n_int, d_min) == pyref.survivors(D, P, v)
            assert np.array_equal(occ, D - v.reshape(D, P).sum(axis=0))
            assert n_int <= d_min <= (D * P - int(v.sum())) // P


def _read_rows(path):
    with open(path) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


def test_worked_example_six_instances(golden_dir):
    """Section 3.2: (2,3) wins on throughput, (3,2) wins under one or two preemptions."""
    rows = _read_rows(os.path.join(golden_dir, "liveput_example_six_instances.txt"))
    per_pipeline = {3: 50.0, 2: 30.0}
    got = {}
    for D, P, k, n_sub, none, intra, inter, rollback, lp0, lp1, lp2 in rows:
        D, P, k = int(D), int(P), int(k)
        M = D * P
        hi = np.zeros(D + 1, dtype=np.uint32)
        hm = np.zeros(D + 1, dtype=np.uint32)
        cls = {"none": 0, "intra": 0, "inter": 0, "rollback": 0}
        n = 0
        d_star = min(D, (M - k) // P)
        for _, v in pyref.all_subsets(M, k):
            a, b, _ = oracle.reduce(D, P, v)
            hi[a] += 1
            hm[b] += 1
            cls[pyref.migration_class(a, b, d_star)] += 1
            n += 1
        assert n == int(n_sub)
        assert [cls["none"], cls["intra"], cls["inter"], cls["rollback"]] == [int(none), int(intra), int(inter), int(rollback)]
        thr = np.arange(D + 1, dtype=np.float32) * np.float32(per_pipeline[P])
        tab = oracle.finalise(np.array([[D, P]], np.int32), np.array([0, D + 1], np.int32),
                              np.array([M, M - k], np.int32), thr, np.array([[2.0, 10.0, 40.0]], np.float32),
                              60.0, n, hi[None, :], hm[None, :])
        want = [float(lp0), float(lp1), float(lp2)]
        assert np.allclose(tab.liveput_d[:, 0, 0], want, rtol=1e-12)
        assert np.allclose(tab.liveput_f[:, 0, 0], want, rtol=1e-6)
        got[(D, P, k)] = tab.liveput_d[:, 0, 0]
    # what the paper prints: the ordering
    assert np.all(got[(2, 3, 0)] > got[(3, 2, 0)])
    for k in (1, 2):
        assert np.all(got[(3, 2, k)] > got[(2, 3, k)])


def test_migration_example_3x4(golden_dir):
    """Section 5.2: {a,f} needs intra-stage only, {b,f} needs inter-stage; both end with two pipelines."""
    rows = _read_rows(os.path.join(golden_dir, "migration_example_3x4.txt"))
    D, P = 3, 4
    letters = "abcdefghijkl"
    counts = {"none": 0, "intra": 0, "inter": 0, "rollback": 0}
    for _, v in pyref.all_subsets(12, 2):
        a, b, _ = oracle.reduce(D, P, v)
        counts[pyref.migration_class(a, b, (12 - 2) // P)] += 1
    for row in rows:
        if row[0] == "counts":
            assert [counts["none"], counts["intra"], counts["inter"], counts["rollback"]] == [int(x) for x in row[1:]]
            continue
        v = np.zeros(12, dtype=np.uint8)
        for ch in row[0].split(","):
            v[letters.index(ch)] = 1
        n_int, d_min, _ = oracle.reduce(D, P, v)
        pipelines = min(D, (12 - 2) // P)
        assert pipelines == int(row[2])
        assert pyref.migration_class(n_int, d_min, pipelines) == row[1]


def test_whole_stage_lost_means_rollback():
    """Section 7 (fault tolerance): if every instance of a stage is preempted neither migration recovers it."""
    for D, P, stage in [(2, 3, 1), (4, 4, 0), (3, 8, 7)]:
        v = np.zeros(D * P, dtype=np.uint8)
        v[stage::P] = 1
        n_int, d_min, occ = oracle.reduce(D, P, v)
        assert d_min == 0 and n_int == 0 and occ[stage] == 0
        assert pyref.migration_class(n_int, d_min, 1) == "rollback"


# ------------------------------------------------------------------ Monte-Carlo expectation vs exact enumeration

@pytest.mark.parametrize("D,P,k", [(2, 3, 2), (3, 2, 2), (3, 4, 2), (4, 4, 5), (2, 8, 3), (8, 2, 9), (5, 3, 11)])
def test_histograms_converge_to_exact_enumeration(D, P, k):
    M = D * P
    assert M <= 16
    hi_x, hm_x, n_sub = pyref.exact_histograms(D, P, k)
    S = 1 << 17
    cfg = np.array([[D, P]], np.int32)
    off = np.array([0, D + 1], np.int32)
    hi, hm = oracle.eval_hist(cfg, off, np.array([M, M - k], np.int32), 0xABCDEF, 0, 0, S, 2)
    assert hi.sum() == S and hm.sum() == S
    for got, exact in ((hi[0], hi_x), (hm[0], hm_x)):
        p = exact / n_sub
        sd = np.sqrt(p * (1 - p) / S)
        assert np.all(np.abs(got / S - p) <= 5.0 * sd + 1e-12)
        assert np.all(got[exact == 0] == 0)
    # the expectation itself: liveput at the no-migration and intra-stage levels
    thr = (np.arange(D + 1) * 7.5).astype(np.float32)
    tab = oracle.finalise(cfg, off, np.array([M, M - k], np.int32), thr, np.array([[2.0, 10.0, 40.0]], np.float32),
                          60.0, S, hi, hm)
    exact0 = float((hi_x * thr).sum() / n_sub)
    exact1 = float((hm_x * thr).sum() / n_sub)
    tol = 4.0 / math.sqrt(S) * float(thr[-1])
    assert abs(tab.liveput_d[0, 0, 0] - exact0) < tol
    assert abs(tab.liveput_d[1, 0, 0] - exact1) < tol


def test_scenario_prefix_is_independent_of_count():
    """Scenario s depends only on (seed, stream, unit, s): histograms over [0,a) + [a,b) = [0,b)."""
    cfg = np.array([[4, 4], [2, 8]], np.int32)
    off = np.array([0, 5, 8], np.int32)
    av = np.array([16, 11, 13], np.int32)
    a = oracle.eval_hist(cfg, off, av, 42, 1, 0, 300, 1)
    b = oracle.eval_hist(cfg, off, av, 42, 1, 300, 1000, 1)
    c = oracle.eval_hist(cfg, off, av, 42, 1, 0, 1000, 3)
    assert np.array_equal(a[0] + b[0], c[0]) and np.array_equal(a[1] + b[1], c[1])


def test_debug_sample_matches_sampler_and_reducer():
    D, P, a_next = 5, 8, 29
    masks, n_int, d_min = oracle.debug_sample(D, P, a_next, 77, 0, 9, 10, 50)
    for x in range(50):
        v = oracle.sample_preempted(D * P, D * P - a_next, 77, 0, 9, 10 + x)
        bits = np.unpackbits(masks[x].view(np.uint8), bitorder="little")[: D * P]
        assert np.array_equal(bits, v)
        assert (n_int[x], d_min[x]) == pyref.survivors(D, P, v)
