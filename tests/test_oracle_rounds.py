"""Pins for inter-stage migration costs that depend on the preemption scenario (section 8.4: the state-transfer
part of the cost varies with the preemptions and follows an alpha-beta model).

Reading under test: a stage with d_min survivors brings `width` instances to hold its state by doubling (every
holder passes the state on to one more instance per round), the stages work in parallel, the migration costs
inter + round_sec * (rounds - 1), never more than a re-partition.
"""
import numpy as np
import pytest

import oracle
import parcae_inputs as pi
from oracle import replay as rp


def _rounds_by_simulation(holders, width):
    """Rounds until `width` instances hold the state when every holder serves one new instance per round."""
    have, r = holders, 0
    while have < width:
        have += min(have, width - have)
        r += 1
    return r


def _scenario_cost(n_int, d_min, width, cost, round_sec):
    if width <= n_int:
        return 0.0
    if width <= d_min:
        return float(cost[0])
    if d_min == 0:
        return float(cost[2])
    r = _rounds_by_simulation(d_min, width)
    return min(float(cost[1]) + float(round_sec) * (r - 1), float(cost[2]))


def test_zero_round_cost_is_the_fixed_inter_stage_cost_bit_for_bit():
    b = pi.workload("small")
    base = oracle.run_query(b, 0, n_scenarios=700, n_threads=4)
    b.cost_round = np.zeros((1, b.n_configs), np.float32)
    same = oracle.run_query(b, 0, n_scenarios=700, n_threads=4)
    assert np.array_equal(base.W_f, same.W_f) and np.array_equal(base.W_d, same.W_d)
    assert np.array_equal(base.tables.teff_f, same.tables.teff_f) and np.array_equal(base.tables.gain_d, same.tables.gain_d)


def test_hand_computed_effective_seconds():
    """One unit, D = 4, P = 2, 16 scenarios: d_min bins (1, 2, 3, 4, 6), no pipeline untouched.  Target width 4
    with costs (2, 10, 40), 60 s intervals, 5 s per further round: six scenarios re-route (58 s left), d_min = 2
    or 3 needs one round (50 s, seven scenarios), d_min = 1 needs two (45 s, two scenarios), one rolls back
    (20 s): (6 * 58 + 7 * 50 + 2 * 45 + 20) / 16 = 50.5."""
    cfg = np.asarray([[4, 2]], np.int32)
    off = np.asarray([0, 5], np.int32)
    hi = np.asarray([[16, 0, 0, 0, 0]], np.uint32)
    hm = np.asarray([[1, 2, 3, 4, 6]], np.uint32)
    thr = np.arange(5, dtype=np.float32) * 10
    cost = np.asarray([[2.0, 10.0, 40.0]], np.float32)
    W_d, W_f = oracle.transition(cfg, off, [8, 8], thr, cost, 60.0, 16, 1, -1, hi, hm, cost_round=[5.0])
    assert W_d[0, 0, 0] == pytest.approx(40 * 50.5, rel=1e-12) and W_f[0, 0, 0] == np.float32(40 * 50.5)
    # capped by the re-partition cost: 30 s per round would make two rounds cost 40, not 10 + 30
    W_d, _ = oracle.transition(cfg, off, [8, 8], thr, cost, 60.0, 16, 1, -1, hi, hm, cost_round=[30.0])
    assert W_d[0, 0, 0] == pytest.approx(40 * (6 * 58 + 7 * 50 + 2 * 20 + 20) / 16, rel=1e-12)


@pytest.mark.parametrize("D,P,k,round_sec", [(8, 4, 9, 6.0), (16, 2, 11, 3.5), (5, 6, 12, 9.0), (32, 2, 40, 2.0),
                                               (6, 5, 4, 25.0)])
def test_tables_and_weights_equal_the_average_over_the_scenarios(D, P, k, round_sec):
    """effective seconds = mean over the sampled scenarios of max(0, tau - cost of that scenario), the cost worked
    out scenario by scenario from (n_int, d_min) with the rounds found by simulating the doubling."""
    S, tau = 3000, 60.0
    widths = sorted({1, 2, max(1, D // 2), D - 1, D})
    cfg = np.asarray([[w, P] for w in widths], np.int32)
    c_src = widths.index(D)
    off = pi.throughput_offsets(cfg)
    avail = np.asarray([D * P, D * P - k], np.int32)
    thr = np.concatenate([np.arange(w + 1, dtype=np.float32) * (1.0 + 0.1 * i) for i, w in enumerate(widths)])
    cost = np.asarray([[1.5 + 0.2 * i, 7.0 + i, 35.0 + 2 * i] for i in range(len(widths))], np.float32)
    rounds = np.asarray([round_sec * (1.0 + 0.3 * i) for i in range(len(widths))], np.float32)
    seed = 0xD00D
    hi, hm = oracle.eval_hist(cfg, off, avail, seed, 0, 0, S)
    _, n_int, d_min = oracle.debug_sample(D, P, D * P - k, seed, 0, c_src, 0, S)
    W_d, W_f = oracle.transition(cfg, off, avail, thr, cost, tau, S, 1, -1, hi, hm, cost_round=rounds)
    for c2, w in enumerate(widths):
        if w * P > avail[1]:
            assert W_d[0, c_src, c2] == -np.inf
            continue
        mean = np.mean([max(0.0, tau - _scenario_cost(int(a), int(m), w, cost[c2], rounds[c2]))
                        for a, m in zip(n_int, d_min)])
        want = float(thr[off[c2] + w]) * mean
        assert W_d[0, c_src, c2] == pytest.approx(want, rel=1e-12)
        assert abs(float(W_f[0, c_src, c2]) - want) <= 1e-5 * abs(want)
    tab = oracle.finalise(cfg, off, avail, thr, cost, tau, S, hi, hm, cost_round=rounds)
    d_star = min(D, (D * P - k) // P)
    mean = np.mean([max(0.0, tau - _scenario_cost(int(a), int(m), d_star, cost[c_src], rounds[c_src]))
                    for a, m in zip(n_int, d_min)])
    assert tab.teff_d[0, c_src] == pytest.approx(mean, rel=1e-12)
    assert tab.gain_d[0, c_src] == pytest.approx(float(thr[off[c_src] + d_star]) * mean, rel=1e-12)


def test_round_cost_only_ever_lowers_the_weights_and_saturates_at_the_repartition_cost():
    b = pi.workload("small")
    base = oracle.run_query(b, 0, n_scenarios=600, n_threads=4)
    prev = base.W_d
    for sec in (1.0, 5.0, 20.0, 1000.0):
        b.cost_round = np.full((1, b.n_configs), sec, np.float32)
        r = oracle.run_query(b, 0, n_scenarios=600, n_threads=4)
        fin = np.isfinite(prev)
        assert np.array_equal(np.isfinite(r.W_d), fin)
        assert np.all(r.W_d[fin] <= prev[fin] + 1e-9)
        assert np.array_equal(r.hist_min, base.hist_min)          # sampling is untouched
        prev = r.W_d
    # a prohibitive round cost: scenarios that need a second round pay the re-partition cost, no more
    floor = np.zeros_like(prev)
    for c2 in range(b.n_configs):
        full = b.thr[0, b.thr_off[c2] + b.configs[c2, 0]]
        floor[:, :, c2] = full * max(0.0, b.interval_sec - b.cost[0, c2, 2])
    fin = np.isfinite(prev)
    assert np.all(prev[fin] >= floor[fin] * (1 - 1e-6))


def test_replay_reward_follows_the_transition_weight_with_rounds():
    b = pi.custom_batch(16, [[1, 4], [2, 4], [3, 4], [4, 4]], [[16, 11]], thr_per_pipeline=[3.0] * 4,
                        cost=[[2.0, 9.0, 30.0]] * 4, n_scenarios=500, seed=3)
    b.cost_round = np.full((1, 4), 6.0, np.float32)
    hi, hm = oracle.eval_hist(b.configs, b.thr_off, b.avail[0], int(b.seed[0]), 0, 0, 500)
    W_d, W_f = oracle.transition(b.configs, b.thr_off, b.avail[0], b.thr[0], b.cost[0], 60.0, 500, 1, -1, hi, hm,
                                 cost_round=b.cost_round[0])
    cfgs = [(int(d), int(p)) for d, p in b.configs]
    for cur in range(4):
        for nxt in range(4):
            if not np.isfinite(W_d[0, cur, nxt]):
                continue
            sl = slice(b.thr_off[cur], b.thr_off[cur + 1])
            r_f, r_d = rp.transition_reward(cfgs, b.thr_off, b.thr[0], b.cost[0], 60.0, 500, cur, nxt, hi[0, sl],
                                            hm[0, sl], 6.0)
            assert r_f == W_f[0, cur, nxt] and r_d == pytest.approx(W_d[0, cur, nxt], rel=1e-12)
