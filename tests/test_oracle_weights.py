"""Pins for preemption with a hazard weight per instance (section 5.1: the equal-probability assumption can be
replaced by more accurate estimations).

The oracle draws by successive weighted sampling without replacement.  These tests check it against what that
process fixes mathematically (exact subset probabilities by enumeration of the orders of departure; all weights
equal is the uniform law of section 5.1) and against a second, independent statement of the draw in Python
integers, bit for bit; the same second statement pins the zoned draw and the addressing of the word sequences.
"""
import math

import numpy as np
import pytest

import oracle
from tests import pyref


def _chi2_ok(counts, probs, n):
    exp = probs * n
    keep = exp >= 5
    chi2 = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum() + 0.0
    dof = max(int(keep.sum()) - 1, 1)
    return chi2 < dof + 6 * math.sqrt(2 * dof) + 10, chi2, dof


def _subset_counts(M, k, weight, S, seed=0xFEED, unit=5):
    masks, _, _ = oracle.debug_sample(M, 1, M - k, seed, 2, unit, 0, S, zone=weight, weight="instances")
    code = masks[:, 0].astype(np.int64)
    return code


@pytest.mark.parametrize("prefix", [0, 1, 3, 0xFFFE, 0xFFFF])
def test_word_sequences_are_addressed_by_block_index(prefix):
    """Word i of sequence `prefix`: counter word 1 = prefix * 2^16 + i / 4 (sequence 0 is the plain word)."""
    seed = 0x0123456789ABCDEF
    for s, unit, stream, i in [(0, 0, 0, 0), (7, 11, 3, 5), (0xFFFFFFFF, 899, 0xFFFFFFFF, 127), (4096, 17, 9, 64)]:
        assert oracle.word_at(seed, stream, unit, s, prefix, i) == pyref.word_at(seed, stream, unit, s, prefix, i)
    if prefix == 0:
        assert oracle.word_at(seed, 1, 2, 3, 0, 9) == oracle.word(seed, 1, 2, 3, 9)
    else:
        assert oracle.word_at(seed, 1, 2, 3, prefix, 9) != oracle.word(seed, 1, 2, 3, 9)


@pytest.mark.parametrize("weight,k", [
    ([1, 3, 7, 2, 9, 1], 2),
    ([5, 1, 1, 2, 8, 3, 1], 3),
    ([2, 9, 1, 4, 1, 6, 3], 5),        # past the half: there is no complement trick to get wrong
    ([1, 255, 1, 1, 30], 2),
    ([4, 4, 4, 4, 4, 4], 3),           # all equal
])
def test_subset_frequencies_match_successive_weighted_sampling(weight, k):
    M, S = len(weight), 200_000
    exact = pyref.successive_sampling_subset_probs(weight, k)
    code = _subset_counts(M, k, weight, S)
    subsets = sorted(exact)
    index = {sum(1 << j for j in sub): n for n, sub in enumerate(subsets)}
    counts = np.zeros(len(subsets))
    for c in code:
        counts[index[int(c)]] += 1                      # KeyError = a set of the wrong size
    ok, chi2, dof = _chi2_ok(counts, np.asarray([exact[sub] for sub in subsets]), S)
    assert ok, (chi2, dof)


@pytest.mark.parametrize("M,k,w", [(6, 2, 1), (7, 3, 9), (8, 4, 255), (8, 7, 2)])
def test_equal_weights_give_the_uniform_law(M, k, w):
    """Every k-subset equally likely (section 5.1), single-instance marginal k / M."""
    S = 150_000
    code = _subset_counts(M, k, [w] * M, S, seed=77, unit=2)
    n_sub = math.comb(M, k)
    values, counts = np.unique(code, return_counts=True)
    assert len(values) == n_sub and all(bin(int(v)).count("1") == k for v in values)
    ok, chi2, dof = _chi2_ok(counts.astype(float), np.full(n_sub, 1.0 / n_sub), S)
    assert ok, (chi2, dof)
    bits = (code[:, None] >> np.arange(M)[None, :]) & 1
    assert np.all(np.abs(bits.mean(axis=0) - k / M) < 4 * math.sqrt((k / M) * (1 - k / M) / S))


def test_a_heavy_instance_goes_first_in_proportion_to_its_weight():
    M, S = 40, 100_000
    weight = [1] * M
    weight[13] = 255
    v = np.stack([oracle.sample_preempted_weighted(M, 1, weight, 5, 0, 3, s) for s in range(0, S, 10)])
    p = 255 / (255 + M - 1)
    assert abs(v[:, 13].mean() - p) < 5 * math.sqrt(p * (1 - p) / len(v))
    assert np.all(v.sum(axis=1) == 1)


@pytest.mark.parametrize("M,k", [(1, 0), (1, 1), (9, 4), (33, 33), (64, 20), (100, 77), (256, 128), (256, 255)])
def test_draw_matches_a_second_statement_bit_for_bit(M, k):
    rng = np.random.default_rng(M * 1000 + k)
    weight = rng.integers(1, 256, size=M).astype(np.uint8)
    for s in (0, 1, 4095, 0xFFFFFFFF):
        got = oracle.sample_preempted_weighted(M, k, weight, 0xC0FFEE123456789, 7, 21, s)
        assert got.sum() == k
        assert np.array_equal(got, pyref.weighted_preempted(M, k, weight, 0xC0FFEE123456789, 7, 21, s))


@pytest.mark.parametrize("M,k,Z", [(1, 1, 1), (12, 5, 3), (40, 33, 4), (64, 10, 2), (200, 101, 4), (256, 250, 3)])
def test_zoned_draw_matches_a_second_statement_bit_for_bit(M, k, Z):
    rng = np.random.default_rng(M + 7 * k)
    zone = rng.integers(0, Z, size=M).astype(np.uint8)
    zw = rng.integers(1, 256, size=Z).astype(np.uint32)
    for s in (0, 3, 65535):
        got = oracle.sample_preempted_zoned(M, k, zone, zw, 0xABCDEF, 2, 9, s)
        assert np.array_equal(got, pyref.zoned_preempted(M, k, zone, zw, 0xABCDEF, 2, 9, s))


def test_weights_reach_the_histograms_and_idle_instances_take_their_share():
    """Whole-cluster pool: the grid is the first D * P instances; making the idle ones heavy protects the grid."""
    D, P, a_prev, a_next, S = 4, 4, 24, 16, 20_000
    light_grid = [1] * 16 + [200] * 8
    heavy_grid = [200] * 16 + [1] * 8
    hi_l, _ = oracle.eval_unit(D, P, a_next, 9, 0, 0, 0, S, a_prev=a_prev, zone=light_grid, weight="instances")
    hi_h, _ = oracle.eval_unit(D, P, a_next, 9, 0, 0, 0, S, a_prev=a_prev, zone=heavy_grid, weight="instances")
    assert hi_l.sum() == S and hi_h.sum() == S
    assert hi_l[D] > 0.7 * S          # most of the time all 8 preemptions fall on the 8 heavy idle instances
    assert hi_h[D] == 0 and hi_h[0] > 0.7 * S     # heavy grid: the preemptions fall on it, hardly a pipeline stays whole
    assert (hi_h * np.arange(D + 1)).sum() < 0.1 * (hi_l * np.arange(D + 1)).sum()
