"""Pins for the whole-cluster preemption pool (section 6.3: N- preemptions among all N_i available instances)."""
import math

import numpy as np
import pytest
from scipy import stats

import oracle
import parcae_inputs as pi
from tests import pyref


def test_mask_covers_the_available_instances_and_keeps_the_preemption_count():
    """The sampled vector has one entry per available instance and exactly N- ones (section 6.3)."""
    D, P, a_prev, a_next = 3, 4, 20, 13
    masks, n_int, d_min = oracle.debug_sample(D, P, a_next, 5, 0, 2, 0, 400, a_prev=a_prev)
    bits = np.unpackbits(masks.view(np.uint8), axis=1, bitorder="little")
    assert np.all(bits[:, a_prev:] == 0)
    assert np.all(bits.sum(axis=1) == a_prev - a_next)
    for x in range(400):
        assert (n_int[x], d_min[x]) == pyref.survivors(D, P, bits[x, : D * P])
    # some preemptions land on idle instances, some on the grid
    on_grid = bits[:, : D * P].sum(axis=1)
    assert on_grid.min() < a_prev - a_next and on_grid.max() > 0


@pytest.mark.parametrize("D,P,pool,k", [(2, 3, 9, 3), (3, 2, 10, 4), (2, 4, 12, 5), (4, 2, 11, 9), (1, 5, 9, 2), (5, 1, 8, 3)])
def test_histograms_converge_to_exact_enumeration_with_idle_instances(D, P, pool, k):
    hi_x, hm_x, n_sub = pyref.exact_histograms_pool(D, P, pool, k)
    assert n_sub == math.comb(pool, k)
    S = 1 << 16
    hi, hm = oracle.eval_unit(D, P, pool - k, 0xFEED, 0, 0, 0, S, a_prev=pool)
    for got, exact in ((hi, hi_x), (hm, hm_x)):
        p = exact / n_sub
        sd = np.sqrt(p * (1 - p) / S)
        assert got.sum() == S
        assert np.all(np.abs(got / S - p) <= 5.0 * sd + 1e-12)
        assert np.all(got[exact == 0] == 0)


def test_hits_on_the_grid_are_hypergeometric():
    D, P, pool, k = 4, 8, 50, 17
    S = 20000
    masks, _, _ = oracle.debug_sample(D, P, pool - k, 11, 3, 7, 0, S, a_prev=pool)
    bits = np.unpackbits(masks.view(np.uint8), axis=1, bitorder="little")
    hits = bits[:, : D * P].sum(axis=1)
    pmf = stats.hypergeom(pool, D * P, k).pmf(np.arange(k + 1))
    counts = np.bincount(hits, minlength=k + 1)[: k + 1]
    keep = pmf * S >= 5
    chi2 = ((counts[keep] - pmf[keep] * S) ** 2 / (pmf[keep] * S)).sum()
    dof = keep.sum() - 1
    assert chi2 < dof + 6 * math.sqrt(2 * dof) + 10


def test_pool_equal_to_the_grid_is_the_used_instance_pool():
    D, P, a_next = 4, 4, 11
    a = oracle.eval_unit(D, P, a_next, 77, 0, 5, 0, 3000, a_prev=D * P)
    b = oracle.eval_unit(D, P, a_next, 77, 0, 5, 0, 3000)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # a configuration that does not fit the available instances falls back to its own instances
    c = oracle.eval_unit(D, P, a_next, 77, 0, 5, 0, 3000, a_prev=12)
    assert np.array_equal(c[0], b[0]) and np.array_equal(c[1], b[1])


def test_whole_query_tables_and_plan():
    b = pi.workload("small")
    S = 512
    r = oracle.run_query(b, 0, n_scenarios=S, n_threads=4, pool_all=True)
    u = oracle.run_query(b, 0, n_scenarios=S, n_threads=4)
    cfg, av = b.configs, b.avail[0]
    for t in range(b.n_intervals):
        for c in range(b.n_configs):
            D, P = cfg[c]
            sl = slice(b.thr_off[c], b.thr_off[c + 1])
            assert r.hist_int[t, sl].sum() == S and r.hist_min[t, sl].sum() == S
            if av[t + 1] >= av[t] and D * P <= av[t]:    # no preemption predicted: liveput equals throughput
                assert r.hist_int[t, sl][D] == S
            d_star = min(D, av[t + 1] // P) if D * P <= av[t] else min(D, min(D * P, av[t + 1]) // P)
            assert r.tables.liveput_d[2, t, c] == b.thr[0, b.thr_off[c] + d_star]
    # the table invariants hold for this pool too
    full = b.thr[0, b.thr_off[1:] - 1].astype(np.float64)
    lp = r.tables.liveput_d
    assert np.all(lp <= full[None, None, :] * (1 + 1e-12))
    assert np.all(lp[0] <= lp[1] * (1 + 1e-12)) and np.all(lp[1] <= lp[2] * (1 + 1e-12))
    assert np.all(r.tables.teff_d <= b.interval_sec * (1 + 1e-12))
    # a small configuration is no longer safe just because it fits the next availability: preemptions fall
    # on it in proportion to its share of the cluster
    t = int(np.argmax(av[:-1] - av[1:]))
    c = int(np.argmax((cfg[:, 0] * cfg[:, 1] <= av[t + 1]) & (cfg[:, 0] * cfg[:, 1] >= 8)))
    D = cfg[c, 0]
    assert u.hist_int[t, b.thr_off[c] + D] == S and r.hist_int[t, b.thr_off[c] + D] < S
    assert r.plan.feasible and np.isfinite(r.plan.objective)
