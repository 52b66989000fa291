"""Pins for the oracle's liveput tables, transition weights and dynamic program."""
import itertools

import numpy as np
import pytest

import oracle
import parcae_inputs as pi
from tests import pyref


def _run(batch, q=0, S=None, threads=4):
    return oracle.run_query(batch, q, n_scenarios=S, n_threads=threads)


# ------------------------------------------------------------------ liveput tables

@pytest.mark.parametrize("name,S", [("tiny", 256), ("small", 512), ("medium", 128)])
def test_table_invariants(name, S):
    b = pi.workload(name)
    r = _run(b, S=S)
    C, T = b.n_configs, b.n_intervals
    full = b.thr[0, b.thr_off[1:] - 1].astype(np.float64)          # zero-preemption throughput per config
    lp = r.tables.liveput_d
    # liveput never exceeds the zero-preemption throughput; the three levels are ordered
    assert np.all(lp <= full[None, None, :] * (1 + 1e-12))
    assert np.all(lp[0] <= lp[1] * (1 + 1e-12)) and np.all(lp[1] <= lp[2] * (1 + 1e-12))
    assert np.all(r.tables.teff_d <= b.interval_sec * (1 + 1e-12)) and np.all(r.tables.teff_d >= 0)
    # histogram totals and the no-preemption case (section 3.2: liveput equals throughput)
    for t in range(T):
        for c in range(C):
            D, P = b.configs[c]
            sl = slice(b.thr_off[c], b.thr_off[c + 1])
            assert r.hist_int[t, sl].sum() == S and r.hist_min[t, sl].sum() == S
            k = max(0, D * P - b.avail[0, t + 1])
            if k == 0:
                assert r.hist_int[t, sl][D] == S and r.hist_min[t, sl][D] == S
                assert np.all(lp[:, t, c] == full[c])
                assert r.tables.teff_d[t, c] == b.interval_sec
                assert r.tables.gain_d[t, c] == full[c] * b.interval_sec
            if k == D * P:
                assert r.hist_int[t, sl][0] == S and r.hist_min[t, sl][0] == S
    # the float tables follow the double ones
    for f, d in ((r.tables.liveput_f, lp), (r.tables.teff_f, r.tables.teff_d), (r.tables.gain_f, r.tables.gain_d)):
        assert np.allclose(f, d, rtol=1e-5, atol=0)


def test_teff_by_class_counts_on_hand_built_histograms():
    """T_eff = T - T_mig averaged over scenarios by class (Eq. 4), on histograms written by hand."""
    D, P, S = 4, 2, 100
    cfg = np.array([[D, P]], np.int32)
    off = np.array([0, D + 1], np.int32)
    # k = 2 -> d_cap = 3.  n_int: 40x2, 60x3 ; d_min: 5x0, 15x2, 80x3
    hi = np.array([[0, 0, 40, 60, 0]], np.uint32)
    hm = np.array([[5, 0, 15, 80, 0]], np.uint32)
    thr = np.array([0, 10, 20, 30, 40], np.float32)
    cost = np.array([[2.0, 10.0, 70.0]], np.float32)     # re-partition longer than the interval -> clamped at 0
    tab = oracle.finalise(cfg, off, np.array([8, 6], np.int32), thr, cost, 60.0, S, hi, hm)
    # width 3: none = 60, intra = 80 - 60 = 20, rollback = 5, inter = 100 - 80 - 5 = 15
    teff = (60 * 60.0 + 20 * 58.0 + 15 * 50.0 + 5 * 0.0) / 100
    assert tab.teff_d[0, 0] == pytest.approx(teff, rel=1e-14)
    assert tab.gain_d[0, 0] == pytest.approx(30.0 * teff, rel=1e-14)
    assert tab.liveput_d[0, 0, 0] == pytest.approx((40 * 20 + 60 * 30) / 100)
    assert tab.liveput_d[1, 0, 0] == pytest.approx((15 * 20 + 80 * 30) / 100)
    assert tab.liveput_d[2, 0, 0] == 30.0


# ------------------------------------------------------------------ transition weights

def test_transition_special_cases():
    """Section 6.2: depth change => pipeline migration cost; same configuration and no preemption => no cost."""
    b = pi.workload("small")
    S = 256
    r = _run(b, S=S)
    C, T, tau = b.n_configs, b.n_intervals, b.interval_sec
    cfg, av = b.configs, b.avail[0]
    full = b.thr[0, b.thr_off[1:] - 1].astype(np.float64)
    cost = b.cost[0].astype(np.float64)
    used = cfg[:, 0] * cfg[:, 1]
    for t in range(T):
        prev_ok = (used <= av[t]) & (cfg[:, 1] >= b.p_min)
        if t == 0:
            prev_ok &= (np.arange(C) == b.cur_config[0])
        next_ok = (used <= av[t + 1]) & (cfg[:, 1] >= b.p_min)
        finite = np.isfinite(r.W_d[t])
        assert np.array_equal(finite, np.outer(prev_ok, next_ok))
        assert np.all(r.W_d[t][~finite] == -np.inf) and np.all(r.W_f[t][~finite] == -np.inf)
        for c, c2 in itertools.product(range(C), repeat=2):
            if not finite[c, c2]:
                continue
            w = r.W_d[t, c, c2]
            assert w <= full[c2] * tau * (1 + 1e-12)
            if cfg[c, 1] != cfg[c2, 1]:
                assert w == pytest.approx(full[c2] * max(0.0, tau - cost[c2, 2]), rel=1e-14)
            elif c == c2 and av[t + 1] >= used[c]:
                assert w == full[c] * tau
            elif cfg[c2, 0] > cfg[c, 0]:
                # growing the width: new instances load state, never cheaper than inter-stage
                assert w <= full[c2] * max(0.0, tau - cost[c2, 1]) * (1 + 1e-12)
            elif av[t + 1] >= used[c]:
                # narrowing with nothing preempted: surplus pipelines are just halted
                assert w == full[c2] * tau
    assert np.allclose(r.W_f[np.isfinite(r.W_f)], r.W_d[np.isfinite(r.W_d)], rtol=1e-5)


def test_transition_same_depth_matches_per_scenario_average():
    """W for a same-depth pair equals the plain per-scenario average of thr * (T - cost of that scenario's class)."""
    D, P, D2, S = 6, 4, 4, 400
    cfg = np.array([[D2, P], [D, P]], np.int32)
    off = pi.throughput_offsets(cfg)
    av = np.array([24, 19], np.int32)
    b = pi.custom_batch(24, cfg, [av], thr_per_pipeline=[3.0, 3.0],
                        cost=[[1.5, 9.0, 33.0], [2.5, 12.0, 50.0]], n_scenarios=S, seed=5)
    r = _run(b, S=S)
    unit = 0 * 2 + 1
    tot = 0.0
    for s in range(S):
        v = oracle.sample_preempted(D * P, D * P - 19, int(b.seed[0]), 0, unit, s)
        n_int, d_min = pyref.survivors(D, P, v)
        cls = pyref.migration_class(n_int, d_min, D2)
        c = {"none": 0.0, "intra": 1.5, "inter": 9.0, "rollback": 33.0}[cls]
        tot += 12.0 * (60.0 - c)
    assert r.W_d[0, 1, 0] == pytest.approx(tot / S, rel=1e-12)


# ------------------------------------------------------------------ dynamic program

def _random_W(rng, T, C, integer, p_inf=0.2):
    if integer:
        W = rng.integers(0, 4, size=(T, C, C)).astype(np.float32)
    else:
        W = rng.random((T, C, C)).astype(np.float32) * 100
    W[rng.random((T, C, C)) < p_inf] = -np.inf
    return W


@pytest.mark.parametrize("T,C,integer", [(1, 1, True), (2, 3, True), (4, 4, True), (5, 3, True), (3, 6, True),
                                         (4, 4, False), (5, 3, False), (3, 6, False)])
def test_dp_equals_exhaustive_enumeration(T, C, integer):
    """Eq. 6 finds an optimal sequence: compare with all C^(T+1) sequences."""
    rng = np.random.default_rng(100 * T + C + (7 if integer else 0))
    for trial in range(12):
        W = _random_W(rng, T, C, integer, p_inf=0.15 if trial % 3 else 0.5)
        p = oracle.dp_f32(W)
        best, seqs = pyref.brute_force_plans(W)
        if best == -np.inf:
            assert not p.feasible and p.objective == -np.inf and np.all(p.plan == -1) and p.start == -1
            continue
        assert p.feasible
        assert np.float32(p.objective) == best                      # left-to-right float sums: bit-equal
        assert p.objective == p.F[T].max()
        got = (p.start, *p.plan.tolist())
        assert got in seqs
        if integer:
            # ties: the plan is the smallest best sequence when compared from the last interval backwards
            assert got == min(seqs, key=lambda s: s[::-1])
        # back-pointers: smallest arg-max of every cell
        for t in range(T):
            col = p.F[t][:, None] + W[t]
            for c2 in range(C):
                m = col[:, c2].max()
                assert p.F[t + 1, c2] == m
                assert p.bp[t, c2] == (-1 if m == -np.inf else int(np.argmax(col[:, c2] == m)))
        # double-precision objective agrees with the double brute force
        bd, _ = pyref.brute_force_plans(W.astype(np.float64))
        assert oracle.dp_f64(W.astype(np.float64)) == pytest.approx(float(bd), rel=1e-12)


def test_dp_with_free_migrations_picks_max_throughput_each_interval():
    """Constant availability and zero migration costs: the best plan is the fastest fitting configuration throughout."""
    cfg = pi.candidate_list(16, (1, 2, 4, 8), 1)
    rates = {1: 1.0, 2: 2.3, 4: 3.9, 8: 7.0}            # per-pipeline rates: (D=5,P=2)... the best product wins
    b = pi.custom_batch(16, cfg, [[12] * 7], thr_per_pipeline=[rates[int(p)] for _, p in cfg],
                        cost=[[0.0, 0.0, 0.0]] * len(cfg), n_scenarios=64)
    r = _run(b, S=64)
    fits = cfg[:, 0] * cfg[:, 1] <= 12
    full = b.thr[0, b.thr_off[1:] - 1]
    best = int(np.argmax(np.where(fits, full, -1)))
    assert np.all(r.plan.plan == best)
    assert r.plan.objective == pytest.approx(6 * 60.0 * float(full[best]), rel=1e-6)


def test_dp_start_restriction_and_infeasible_query():
    cfg = pi.candidate_list(8, (1, 2, 4), 1)
    b = pi.custom_batch(8, cfg, [[8, 6, 7]], thr_per_pipeline=[1.0] * len(cfg), n_scenarios=32, cur_config=3)
    r = _run(b, S=32)
    assert r.plan.start == 3 and np.all(np.isfinite(r.W_f[0, 3, cfg[:, 0] * cfg[:, 1] <= 6]))
    assert np.all(r.W_f[0, np.arange(len(cfg)) != 3] == -np.inf)
    # availability below the memory floor in the middle of the horizon: training would be suspended (section 7)
    b2 = pi.custom_batch(8, cfg, [[8, 1, 7]], thr_per_pipeline=[1.0] * len(cfg), n_scenarios=32, p_min=2)
    r2 = _run(b2, S=32)
    assert not r2.plan.feasible and r2.plan.objective == -np.inf and np.all(r2.plan.plan == -1)


def test_plan_on_six_instance_example_has_closed_form_value():
    """Six instances falling to four (section 3.2's two configurations plus their narrower widths)."""
    cfg = np.array([[1, 2], [2, 2], [3, 2], [1, 3], [2, 3]], np.int32)   # 30 vs 50 samples/s per pipeline
    av = [[6, 6, 4, 4, 4, 4, 4, 4, 4]]
    b = pi.custom_batch(6, cfg, av, thr_per_pipeline=[30.0, 30.0, 30.0, 50.0, 50.0], cost=[[1.0, 8.0, 20.0]] * 5,
                        n_scenarios=4096, cur_config=4)
    r = _run(b, S=4096)
    # stay on (2,3) while six instances last: 100/s * 60 s; then re-partition to (2,2): 60/s * (60 - 20) s;
    # then six more intervals of (2,2) at 60/s * 60 s.  Depth 3 would keep one pipeline (50/s) at four instances.
    assert r.plan.start == 4 and r.plan.plan.tolist() == [4, 1, 1, 1, 1, 1, 1, 1]
    assert r.plan.objective == 6000.0 + 2400.0 + 6 * 3600.0
    assert r.objective_d == pytest.approx(30000.0, rel=1e-12)
    # leaving for (3,2) at once costs a re-partition now and still a migration at the drop: worse
    early = [4, 2, 1, 1, 1, 1, 1, 1, 1]
    assert sum(r.W_d[t, early[t], early[t + 1]] for t in range(8)) < r.objective_d


def test_workload_generator_shapes():
    """The synthetic workloads have the stated sizes."""
    want = {"tiny": (15, 65, 4, 256), "small": (30, 215, 12, 4096), "medium": (30, 215, 30, 16384),
            "large": (60, 770, 60, 65536)}
    for name, (C, L, T, S) in want.items():
        b = pi.workload(name)
        assert (b.n_configs, b.hist_len, b.n_intervals, b.n_scenarios) == (C, L, T, S)
        assert b.avail.min() >= pi.WORKLOADS[name].avail_floor and b.avail.max() <= b.n_instances
        assert np.all(b.thr[:, b.thr_off[:-1]] == 0)
        assert np.all(b.cost[..., 0] <= b.cost[..., 1]) and np.all(b.cost[..., 1] <= b.cost[..., 2])
    assert pi.workload("medium", dense=True).n_configs == 126
    assert pi.workload("large", dense=True).n_configs == 508
    sw = pi.workload("sweep", n_queries=8)
    assert sw.n_queries == 8 and sw.n_configs == 30 and len(set(sw.seed.tolist())) == 8


def test_cold_start_brings_up_the_first_configuration_at_the_repartition_cost():
    """cur_config = -2: nothing is running (training was suspended, section 7)."""
    cfg = pi.candidate_list(8, (1, 2, 4), 1)
    b = pi.custom_batch(8, cfg, [[1, 6, 7]], thr_per_pipeline=[1.0 + 0.5 * p for _, p in cfg], n_scenarios=64,
                        cur_config=-2, cost=[[1.0, 8.0, 25.0]] * len(cfg), p_min=2)
    r = _run(b, S=64)
    used = cfg[:, 0] * cfg[:, 1]
    full = b.thr[0, b.thr_off[1:] - 1]
    for c in range(len(cfg)):
        for c2 in range(len(cfg)):
            if c == c2 and used[c2] <= 6 and cfg[c2, 1] >= 2:
                assert r.W_f[0, c, c2] == np.float32(full[c2] * np.float32(35.0))
            else:
                assert r.W_f[0, c, c2] == -np.inf
    assert r.plan.feasible and r.plan.start == r.plan.plan[0]
    # the availability now (1 instance) does not matter for a cold start; a warm free start would be infeasible
    b.cur_config[0] = -1
    assert not _run(b, S=64).plan.feasible
