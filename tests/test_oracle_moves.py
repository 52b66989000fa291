"""Pins for the migration cost that grows with the number of instances that must receive state (section 8.4: the
model-transfer part of the cost varies with the preemption scenario; alpha-beta model).

The oracle keeps a third statistic per unit, the stage-occupancy counts, and reads the expected cost of every target
width off it.  These tests pin the statistic against the array definition scenario by scenario, and the expected
effective seconds and transition weights against a plain average over the scenarios with the cost written out per
scenario (cap at the re-partition cost and clamp at zero included: they never bind for valid inputs).
"""
import numpy as np
import pytest

import oracle
import parcae_inputs as pi
from tests import pyref


def _bits(masks, M):
    return np.unpackbits(masks.view(np.uint8), axis=1, bitorder="little")[:, :M]


@pytest.mark.parametrize("D,P,a_next,a_prev", [(4, 4, 11, -1), (6, 3, 10, -1), (3, 8, 20, -1), (16, 2, 25, -1),
                                               (5, 7, 30, -1), (4, 4, 12, 22), (2, 16, 30, 40), (1, 9, 8, -1)])
def test_stage_occupancy_statistic_is_the_count_over_scenarios(D, P, a_next, a_prev):
    S = 700
    hi, hm, ho = oracle.eval_unit(D, P, a_next, 31, 1, 4, 0, S, a_prev=a_prev, with_occ=True)
    masks, n_int, d_min = oracle.debug_sample(D, P, a_next, 31, 1, 4, 0, S, a_prev=a_prev)
    pool = max(D * P, a_prev)
    want = np.zeros(D + 1, np.int64)
    for v in _bits(masks, pool):
        occ = pyref.stage_occupancy(D, P, v[: D * P])
        if occ.min() >= 1:
            for j in occ:
                want[j] += 1
    assert np.array_equal(ho, want)
    assert ho[0] == 0 and ho.sum() == P * (S - hm[0])
    # every width at once: the moves summed over the scenarios that lost no whole stage
    for width in range(1, D + 2):
        total = sum(pyref.moves_to_width(pyref.stage_occupancy(D, P, v[: D * P]), width)
                    for v in _bits(masks, pool) if pyref.stage_occupancy(D, P, v[: D * P]).min() >= 1)
        assert total == sum(int(ho[j]) * (width - j) for j in range(1, min(width, D + 1)))


def test_multi_gpu_instances_count_gpu_pipelines():
    D, P, g, S = 8, 3, 4, 400
    hi, hm, ho = oracle.eval_unit(D, P, 4, 3, 0, 0, 0, S, group=g, with_occ=True)
    assert np.all(np.nonzero(ho)[0] % g == 0) and ho.sum() == P * (S - hm[0])


def _per_scenario_teff(D, P, masks, pool, width, tau, co, beta):
    """Average over the scenarios of tau - cost of the scenario's migration class, the inter-stage cost being
    alpha + beta * moves, capped by the re-partition cost, nothing below zero."""
    acc = 0.0
    for v in _bits(masks, pool):
        n_int, d_min = pyref.survivors(D, P, v[: D * P])
        kind = pyref.migration_class(n_int, d_min, width)
        if kind == "none":
            cost = 0.0
        elif kind == "intra":
            cost = co[0]
        elif kind == "rollback":
            cost = co[2]
        else:
            cost = min(co[2], co[1] + beta * pyref.moves_to_width(pyref.stage_occupancy(D, P, v[: D * P]), width))
        acc += max(0.0, tau - cost)
    return acc / len(masks)


def test_effective_seconds_and_weights_equal_the_per_scenario_average():
    cfg = np.asarray([[2, 4], [3, 4], [4, 4], [6, 4], [2, 8], [3, 8]], np.int32)
    avail = [[24, 17, 20, 9, 24]]
    b = pi.custom_batch(24, cfg, avail, thr_per_pipeline=[1.0, 1.0, 1.0, 1.0, 2.1, 2.1],
                        cost=[[2.0, 10.0, 40.0]] * 6, n_scenarios=600, seed=5, cur_config=3).with_moves(seed=3)
    assert np.all(b.cost_move[0][[0, 1, 2, 3, 4, 5]] > 0)
    r = oracle.run_query(b, 0)
    S, tau, off = 600, 60.0, b.thr_off
    for t in range(4):
        for c in range(6):
            D, P = (int(x) for x in cfg[c])
            a_next = int(b.avail[0, t + 1])
            masks, _, _ = oracle.debug_sample(D, P, a_next, int(b.seed[0]), 0, t * 6 + c, 0, S)
            d_star = min(D, min(D * P, a_next) // P)
            co = [float(x) for x in b.cost[0, c]]
            want = _per_scenario_teff(D, P, masks, D * P, d_star, tau, co, float(b.cost_move[0, c]))
            assert abs(r.tables.teff_d[t, c] - want) <= 1e-11 * max(want, 1.0), (t, c)
            assert abs(float(r.tables.teff_f[t, c]) - want) <= 1e-5 * max(want, 1.0)
            for c2 in range(6):
                D2, P2 = (int(x) for x in cfg[c2])
                if P2 != P or not np.isfinite(r.W_d[t, c, c2]):
                    continue
                co2 = [float(x) for x in b.cost[0, c2]]
                te = _per_scenario_teff(D, P, masks, D * P, D2, tau, co2, float(b.cost_move[0, c2]))
                full = float(b.thr[0, off[c2] + D2])
                assert abs(r.W_d[t, c, c2] - full * te) <= 1e-11 * max(full * te, 1.0), (t, c, c2)
                assert abs(float(r.W_f[t, c, c2]) - full * te) <= 1e-5 * max(full * te, 1.0)


def test_three_by_two_grid_worked_by_hand():
    """3 x 2 grid (6 instances) falling to 4: two of the six go, 15 equally likely pairs, two pipelines can go on.
    Both in one stage (6 pairs): that stage keeps 1 of the 2 holders it needs, an inter-stage migration that moves
    one instance, 60 - 10 - 3 * 1 = 47 s.  One in each stage, same pipeline (3 pairs): two pipelines untouched,
    60 s.  One in each stage, different pipelines (6 pairs): re-routing inside the stages, 60 - 2 = 58 s.
    Expectation (6 * 47 + 3 * 60 + 6 * 58) / 15 = 54 s."""
    S = 60_000
    b = pi.custom_batch(6, [[2, 2], [3, 2]], [[6, 4]], thr_per_pipeline=[5.0, 5.0], cost=[[2.0, 10.0, 40.0]] * 2,
                        n_scenarios=S, cur_config=1)
    b.cost_move = np.asarray([[3.0, 3.0]], np.float32)
    r = oracle.run_query(b, 0, n_threads=4)
    ho = r.hist_occ[0, b.thr_off[1]: b.thr_off[2]].astype(np.int64)
    assert ho[0] == 0 and ho[1] == ho[3] and ho.sum() == 2 * S          # stages with 1 and with 3 survivors pair up
    assert abs(ho[1] / S - 6 / 15) < 4 * np.sqrt(0.4 * 0.6 / S)
    sigma = np.sqrt((6 * 47 ** 2 + 3 * 60 ** 2 + 6 * 58 ** 2) / 15 - 54 ** 2)
    assert abs(r.tables.teff_d[0, 1] - 54.0) < 4 * sigma / np.sqrt(S)    # the unit keeps D* = 2 pipelines
    assert abs(r.W_d[0, 1, 0] - 10.0 * r.tables.teff_d[0, 1]) < 1e-9    # (3,2) -> (2,2): the same expectation
    assert r.W_f[0, 1, 1] == -np.inf                                     # three pipelines no longer fit


def test_zero_move_cost_is_the_fixed_cost_bit_for_bit_and_the_cost_is_felt():
    b0 = pi.workload("small", n_scenarios=500)
    r0 = oracle.run_query(b0, 0, n_threads=4)
    bz = pi.workload("small", n_scenarios=500)
    bz.cost_move = np.zeros((1, bz.n_configs), np.float32)
    rz = oracle.run_query(bz, 0, n_threads=4)
    assert np.array_equal(r0.W_f, rz.W_f) and np.array_equal(r0.tables.teff_f, rz.tables.teff_f)
    assert np.array_equal(r0.plan.plan, rz.plan.plan)
    bm = pi.workload("small", n_scenarios=500).with_moves()
    rm = oracle.run_query(bm, 0, n_threads=4)
    fin = np.isfinite(r0.W_d)
    assert np.all(rm.W_d[fin] <= r0.W_d[fin] + 1e-9) and np.any(rm.W_d[fin] < r0.W_d[fin] - 1e-6)
    assert np.all(rm.W_d[fin] >= 0.0)
    # the generator keeps the dearest inter-stage migration within min(interval, re-partition cost)
    worst = (bm.configs[:, 0] - 1) * bm.configs[:, 1]
    dear = bm.cost[0, :, 1] + bm.cost_move[0] * worst
    assert np.all(dear <= np.minimum(bm.interval_sec, bm.cost[0, :, 2]) + 1e-4)
