"""Pins for non-uniform preemption (section 5.1: the equal-probability assumption may be replaced by better
estimates; section 4.1: availability zones and instance types drive preemptions).

The oracle draws by zones and hazard weights; these tests check it against what successive weighted sampling
without replacement fixes mathematically: exact subset probabilities by enumeration of departure orders, the
exact distribution of per-zone counts of the urn process, exchangeability inside a zone, and the uniform
sampler as the one-zone special case.
"""
import math

import numpy as np
import pytest

import oracle
import parcae_inputs as pi
from tests import pyref


def _bits(masks, M):
    return np.unpackbits(masks.view(np.uint8), axis=1, bitorder="little")[:, :M]


def _chi2_ok(counts, probs, n):
    exp = probs * n
    keep = exp >= 5
    chi2 = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum() + 0.0
    dof = max(int(keep.sum()) - 1, 1)
    return chi2 < dof + 6 * math.sqrt(2 * dof) + 10, chi2, dof


@pytest.mark.parametrize("M,k", [(1, 0), (1, 1), (7, 3), (10, 9), (33, 5), (64, 40), (100, 50), (256, 3), (256, 255)])
def test_one_zone_is_the_uniform_sampler_bit_for_bit(M, k):
    for s in range(6):
        a = oracle.sample_preempted(M, k, 0xABCDEF12345, 3, 17, s)
        b = oracle.sample_preempted_zoned(M, k, np.zeros(M, np.uint8), [1 + 40 * s], 0xABCDEF12345, 3, 17, s)
        assert np.array_equal(a, b)


@pytest.mark.parametrize("M,k,Z", [(5, 0, 2), (5, 5, 2), (12, 4, 3), (64, 20, 4), (200, 150, 4), (256, 128, 3)])
def test_exactly_k_instances_go_and_zone_counts_respect_zone_sizes(M, k, Z):
    zone = (np.arange(M) * 7 % Z).astype(np.uint8)
    weight = [3, 1, 9, 2][:Z]
    for s in range(40):
        v = oracle.sample_preempted_zoned(M, k, zone, weight, 99, 0, 4, s)
        assert v.sum() == k and set(np.unique(v)) <= {0, 1}


@pytest.mark.parametrize("zone,weight,k", [
    ([0, 1, 2, 0, 1, 2], [1, 3, 7], 2),
    ([0, 0, 1, 1, 1, 2, 2], [5, 1, 2], 3),
    ([1, 0, 1, 0, 1, 0, 3], [2, 9, 1, 4], 4),      # a zone without members, k past the half
    ([0, 1, 0, 1, 1], [1, 200], 2),
])
def test_subset_frequencies_match_successive_weighted_sampling(zone, weight, k):
    M, S = len(zone), 200_000
    w_inst = [weight[z] for z in zone]
    exact = pyref.successive_sampling_subset_probs(w_inst, k)
    masks, _, _ = oracle.debug_sample(M, 1, M - k, 0x5EED, 1, 3, 0, S, zone=zone, weight=weight)
    code = masks[:, 0].astype(np.int64)
    subsets = sorted(exact)
    codes = np.asarray([sum(1 << j for j in sub) for sub in subsets])
    counts = np.asarray([(code == c).sum() for c in codes])
    assert counts.sum() == S                      # no other subset ever shows up
    ok, chi2, dof = _chi2_ok(counts, np.asarray([exact[sub] for sub in subsets]), S)
    assert ok, (chi2, dof)


def test_equal_weights_give_the_uniform_distribution_whatever_the_zones():
    zone, k, S = [0, 1, 2, 2, 1, 0, 1], 3, 150_000
    M = len(zone)
    masks, _, _ = oracle.debug_sample(M, 1, M - k, 0x77, 0, 0, 0, S, zone=zone, weight=[4, 4, 4])
    code = masks[:, 0].astype(np.int64)
    codes = [sum(1 << j for j in sub) for _, sub in zip(range(10**6), __import__("itertools").combinations(range(M), k))]
    counts = np.asarray([(code == c).sum() for c in codes])
    assert counts.sum() == S
    ok, chi2, dof = _chi2_ok(counts, np.full(len(codes), 1.0 / len(codes)), S)
    assert ok, (chi2, dof)


@pytest.mark.parametrize("M,k,weight", [(64, 20, [1, 4, 2]), (96, 70, [8, 1, 3, 5]), (256, 31, [2, 7])])
def test_zone_counts_follow_the_urn_process_and_members_of_a_zone_are_exchangeable(M, k, weight):
    Z, S = len(weight), 40_000
    rng = pi.SplitMix64(M * 1000 + k)
    zone = np.asarray([rng.randint(0, Z - 1) for _ in range(M)], dtype=np.uint8)
    sizes = [int((zone == z).sum()) for z in range(Z)]
    masks, _, _ = oracle.debug_sample(M, 1, M - k, 0xC0FFEE, 2, 9, 0, S, zone=zone, weight=weight)
    bits = _bits(masks, M)
    assert np.all(bits.sum(axis=1) == k)
    # marginal distribution of the count in every zone against the exact urn process
    dist = pyref.zone_count_distribution(sizes, weight, k)
    for z in range(Z):
        pmf = np.zeros(k + 1)
        for gone, p in dist.items():
            pmf[gone[z]] += p
        counts = np.bincount(bits[:, zone == z].sum(axis=1), minlength=k + 1)[: k + 1]
        ok, chi2, dof = _chi2_ok(counts, pmf, S)
        assert ok, (z, chi2, dof)
    # inside a zone every instance goes equally often
    for z in range(Z):
        hits = bits[:, zone == z].sum(axis=0).astype(float)
        if hits.size < 2:
            continue
        p = hits.sum() / (S * hits.size)
        sd = math.sqrt(S * p * (1 - p))
        assert np.all(np.abs(hits - S * p) <= 5 * sd + 1), (z, hits)
    # a zone with a larger weight loses a larger share of its instances
    share = [bits[:, zone == z].mean() for z in range(Z)]
    order = np.argsort(weight)
    assert all(share[order[i]] < share[order[i + 1]] for i in range(Z - 1) if weight[order[i]] < weight[order[i + 1]])


@pytest.mark.parametrize("D,P,k,zone,weight", [
    (2, 3, 2, [0, 0, 0, 1, 1, 1], [1, 6]),          # the second pipeline is the likely victim
    (3, 2, 3, [0, 1, 0, 1, 0, 1], [5, 1]),          # the first stage is the likely victim
    (2, 4, 3, [0, 1, 2, 0, 1, 2, 0, 1], [1, 2, 3]),
])
def test_histograms_converge_to_the_exact_weighted_expectation(D, P, k, zone, weight):
    M, S = D * P, 1 << 16
    exact = pyref.successive_sampling_subset_probs([weight[z] for z in zone], k)
    p_int, p_min = np.zeros(D + 1), np.zeros(D + 1)
    for sub, p in exact.items():
        v = np.zeros(M, np.uint8)
        v[list(sub)] = 1
        a, b = pyref.survivors(D, P, v)
        p_int[a] += p
        p_min[b] += p
    hi, hm = oracle.eval_unit(D, P, M - k, 0xFEED, 0, 0, 0, S, zone=zone, weight=weight)
    for got, p in ((hi, p_int), (hm, p_min)):
        sd = np.sqrt(p * (1 - p) / S)
        assert got.sum() == S
        assert np.all(np.abs(got / S - p) <= 5.0 * sd + 1e-12)
        assert np.all(got[p == 0] == 0)
    # and they differ from the uniform ones (the test would not notice ignored weights otherwise)
    hi_u, hm_u = oracle.eval_unit(D, P, M - k, 0xFEED, 0, 0, 0, S)
    assert not (np.array_equal(hi, hi_u) and np.array_equal(hm, hm_u))


def test_zone_words_come_from_their_own_sequences():
    """The zone draws use word sequence 0xFFFF, the subset of zone z sequence z: changing one zone's weight
    changes which zones lose instances but, for equal per-zone counts, not which members of a zone go."""
    assert oracle.word_at(5, 1, 2, 3, 0, 6) == oracle.word(5, 1, 2, 3, 6)
    assert oracle.word_at(5, 1, 2, 3, 1, 6) != oracle.word(5, 1, 2, 3, 6)
    M, k = 40, 10
    zone = np.asarray([0] * 20 + [1] * 20, dtype=np.uint8)
    seen = 0
    for s in range(400):
        a = oracle.sample_preempted_zoned(M, k, zone, [1, 1], 31, 0, 0, s)
        b = oracle.sample_preempted_zoned(M, k, zone, [1, 3], 31, 0, 0, s)
        if a[:20].sum() == b[:20].sum():
            assert np.array_equal(a, b)
            seen += 1
    assert seen > 10


def test_whole_query_with_zones_keeps_the_table_invariants():
    b = pi.workload("small").with_zones(3)
    S = 512
    r = oracle.run_query(b, 0, n_scenarios=S, n_threads=4)
    u = oracle.run_query(pi.workload("small"), 0, n_scenarios=S, n_threads=4)
    assert r.hist_int.sum() == u.hist_int.sum() == b.n_intervals * b.n_configs * S
    assert not np.array_equal(r.hist_min, u.hist_min)
    lp = r.tables.liveput_d
    assert np.all(lp[0] <= lp[1] + 1e-12) and np.all(lp[1] <= lp[2] + 1e-12)
    assert np.array_equal(lp[2], u.tables.liveput_d[2])      # the post-migration width depends on counts only
    assert np.all(r.tables.teff_d <= b.interval_sec + 1e-9)
    assert r.plan.feasible
