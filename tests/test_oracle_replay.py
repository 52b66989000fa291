"""Pins for the oracle's receding-horizon replay (algorithm 1's loop, section 7 adaptation, reactive baseline)."""
import numpy as np
import pytest

import oracle
from oracle import replay as rp
import parcae_inputs as pi

CFG = [(1, 2), (2, 2), (3, 2), (4, 2), (1, 4), (2, 4), (1, 8)]


def test_adaptation_rules_of_section_7():
    # forecast right: the planned configuration stands
    assert rp.adapt(CFG, 2, 1, 2, 6, 6) == 2
    # more instances than forecast: pipelines are added at the same depth
    assert rp.adapt(CFG, 2, 1, 1, 8, 4) == 3
    assert rp.adapt(CFG, 2, 1, 4, 8, 5) == 5
    # fewer: pipelines are dropped at the same depth
    assert rp.adapt(CFG, 2, 1, 3, 5, 8) == 1
    assert rp.adapt(CFG, 2, 1, 5, 7, 8) == 4
    # not even one pipeline of that depth: fewer stages (deepest shallower depth that fits, widest of it)
    assert rp.adapt(CFG, 2, 1, 6, 7, 8) == 4
    assert rp.adapt(CFG, 2, 1, 5, 3, 8) == 0
    # fewer instances than the minimum depth: training is suspended
    assert rp.adapt(CFG, 2, 1, 5, 1, 8) == -1
    assert rp.adapt(CFG, 4, 1, 6, 3, 8) == -1
    # nothing planned stays nothing
    assert rp.adapt(CFG, 2, 1, -1, 8, 8) == -1
    # four-GPU instances: widths fit against four GPUs per instance
    assert rp.adapt([(4, 2), (8, 2), (4, 4)], 2, 4, 1, 3, 4) == 0


def test_reactive_choice_is_the_fastest_fitting_candidate():
    thr_full = np.array([30, 60, 90, 120, 50, 100, 70], np.float32)
    assert rp.reactive_choice(CFG, thr_full, 2, 1, 8) == 3
    assert rp.reactive_choice(CFG, thr_full, 2, 1, 6) == 2
    assert rp.reactive_choice(CFG, thr_full, 4, 1, 8) == 5
    assert rp.reactive_choice(CFG, thr_full, 2, 1, 1) == -1
    thr_tie = np.array([30, 60, 90, 100, 50, 100, 70], np.float32)
    assert rp.reactive_choice(CFG, thr_tie, 2, 1, 8) == 3          # smallest index on ties


def test_transition_reward_equals_the_transition_weight_of_the_oracle():
    """The Python statement of Eq. 4 used by the replay against the C oracle's weights, bit for bit."""
    b = pi.workload("small", n_scenarios=300)
    r = oracle.run_query(b, 0, n_threads=4)
    cfg = [(int(d), int(p)) for d, p in b.configs]
    t = 6
    n = 0
    for c in range(len(cfg)):
        for c2 in range(len(cfg)):
            if not np.isfinite(r.W_f[t, c, c2]):
                continue
            sl = slice(b.thr_off[c], b.thr_off[c + 1])
            f, d = rp.transition_reward(cfg, b.thr_off, b.thr[0], b.cost[0], b.interval_sec, 300, c, c2,
                                        r.hist_int[t, sl], r.hist_min[t, sl])
            assert f == r.W_f[t, c, c2] and d == pytest.approx(r.W_d[t, c, c2], rel=1e-13)
            n += 1
    assert n > 100
    # cold start pays the re-partition cost of the new configuration
    f, _ = rp.transition_reward(cfg, b.thr_off, b.thr[0], b.cost[0], b.interval_sec, 300, -1, 7, None, None)
    full = b.thr[0, b.thr_off[7] + cfg[7][0]]
    assert f == np.float32(full * np.float32(np.float32(b.interval_sec) - b.cost[0, 7, 2]))
    assert rp.transition_reward(cfg, b.thr_off, b.thr[0], b.cost[0], b.interval_sec, 300, 3, -1, None, None)[0] == 0


def _windows(true_avail, T, forecast=None):
    H = len(true_avail) - 1 - 0
    out = []
    for i in range(H):
        fut = [true_avail[min(i + 1 + t, len(true_avail) - 1)] for t in range(T)] if forecast is None else forecast[i]
        out.append([true_avail[i]] + list(fut))
    return np.asarray(out, np.int32)


def test_steady_availability_and_perfect_forecast():
    """Nothing is preempted: after the first move every interval commits throughput x interval length."""
    cfg = pi.candidate_list(16, (2, 4, 8), 2)
    rates = {2: 2.5, 4: 4.4, 8: 7.5}          # depth 2 is fastest, and it is the depth already running
    b = pi.custom_batch(16, cfg, [[12] * 5], thr_per_pipeline=[rates[int(p)] for _, p in cfg], n_scenarios=64,
                        p_min=2, cur_config=0)
    true = [12] * 9
    win = _windows(true, 4)
    fits = cfg[:, 0] * cfg[:, 1] <= 12
    full = b.thr[0, b.thr_off[1:] - 1]
    best = int(np.argmax(np.where(fits, full, -1)))
    for mode in (rp.PROACTIVE, rp.REACTIVE):
        r = rp.replay(b, 0, true, win, mode)
        assert np.all(r.chosen == best)
        assert np.all(r.reward[1:] == np.float32(full[best] * np.float32(60.0)))
        assert r.reward[0] < r.reward[1]                        # the first move pays a migration
        assert r.total == pytest.approx(r.total_d, rel=1e-6)


def test_wrong_forecast_triggers_adaptation_and_suspension():
    cfg = pi.candidate_list(8, (2, 4), 2)
    b = pi.custom_batch(8, cfg, [[8, 8, 8]], thr_per_pipeline=[1.0 + p for _, p in cfg], n_scenarios=128, p_min=2,
                        cur_config=len(cfg) - 1)
    true = [8, 3, 1, 6]
    forecast = [[8, 8], [8, 8], [8, 8]]                          # always optimistic
    r = rp.replay(b, 0, true, _windows(true, 2, forecast), rp.PROACTIVE)
    used = cfg[:, 0] * cfg[:, 1]
    assert r.chosen[0] >= 0 and used[r.chosen[0]] <= 3
    assert r.chosen[1] == -1 and r.reward[1] == 0                # one instance left: below the minimum depth
    assert r.chosen[2] >= 0 and used[r.chosen[2]] <= 6          # restart from nothing pays a re-partition
    c = r.chosen[2]
    assert r.reward[2] == np.float32(b.thr[0, b.thr_off[c] + cfg[c, 0]] * np.float32(np.float32(60.0) - b.cost[0, c, 2]))


def test_proactive_is_not_worse_than_reactive_on_average_with_a_perfect_forecast():
    b = pi.workload("sweep", n_queries=24, n_scenarios=256)
    H, T = 12, b.n_intervals
    tot = {rp.PROACTIVE: 0.0, rp.REACTIVE: 0.0}
    for q in range(24):
        true = b.avail[q, : H + T + 1]
        win = np.asarray([[true[i]] + [true[min(i + 1 + t, len(true) - 1)] for t in range(T)] for i in range(H)], np.int32)
        for mode in tot:
            tot[mode] += rp.replay(b, q, true[: H + 1], win, mode, n_threads=4).total_d
    assert tot[rp.PROACTIVE] >= 0.995 * tot[rp.REACTIVE]
