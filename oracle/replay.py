"""Receding-horizon replay of the planner along a true availability walk (test infrastructure, CPU oracle).

The paper's scheduler (algorithm 1) calls the liveput optimizer once per interval with a fresh forecast,
keeps the first configuration of the plan, adapts it when the forecast was wrong (section 7,
"parallelization adaptation") and pays the migration that the actual preemptions require.  The reactive
baseline it is compared with (section 9.4, "Proactive vs. Reactive") picks the fastest configuration for the
instances that are actually there, after the fact.  This module replays both on one query with plain Python
loops around the C oracle; it shares no code with the GPU library.

Step i (i = 0 .. H-1), state cur = configuration running in interval i (or -1 = none):
  1. proactive: plan on window i (window[0] = true availability now, window[1 + t] = forecast), random stream
     id + 2 i; target = first configuration of the plan (cur if the plan is infeasible); if nothing is
     running the plan starts cold (every first configuration pays its re-partition cost).
     reactive: no plan; target = fastest candidate that fits the actual next availability.
  2. a = true availability of interval i + 1.  Adaptation of the target (section 7): if a equals the
     forecast the target stands; otherwise pipelines are added or dropped at the target's depth (the widest
     candidate of that depth that fits a); if not even one pipeline of that depth fits, the deepest shallower
     depth that fits (widest candidate of it); if nothing fits, training is suspended (-1).
  3. reward = expected committed samples of the transition cur -> next under the actual drop from true[i] to a
     (Eq. 4 with the class rule), scenarios drawn with stream id + 2 i + 1; a cold start (cur = -1) or a change
     of depth pays the re-partition cost of the new configuration.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import batch_rounds, batch_zones, dp_f32, eval_hist, transition

PROACTIVE, REACTIVE = 0, 1
_F = np.float32


def fits(configs, c, a, group):
    return int(configs[c][0]) * int(configs[c][1]) <= group * a


def reactive_choice(configs, thr_full, p_min, group, a):
    """Fastest candidate that fits `a` instances (smallest index on ties), -1 if none."""
    best, arg = -1.0, -1
    for c in range(len(configs)):
        if configs[c][1] >= p_min and fits(configs, c, a, group) and float(thr_full[c]) > best:
            best, arg = float(thr_full[c]), c
    return arg


def widest_of_depth(configs, depth, a, group):
    """Widest candidate of the given depth that fits `a` instances, -1 if none."""
    arg = -1
    for c in range(len(configs)):
        if configs[c][1] == depth and fits(configs, c, a, group):
            if arg < 0 or configs[c][0] > configs[arg][0]:
                arg = c
    return arg


def adapt(configs, p_min, group, target, a, a_forecast):
    """Section 7: keep the depth and add or drop pipelines; fewer stages if no pipeline of that depth fits."""
    if target < 0:
        return -1
    if a == a_forecast and fits(configs, target, a, group):
        return target
    depth = int(configs[target][1])
    same = widest_of_depth(configs, depth, a, group)
    if same >= 0:
        return same
    for d in sorted({int(p) for _, p in configs if p_min <= p < depth}, reverse=True):
        c = widest_of_depth(configs, d, a, group)
        if c >= 0:
            return c
    return -1


def transition_reward(configs, thr_off, thr, cost, tau, S, cur, nxt, bins_int, bins_min, round_sec=0.0):
    """Expected committed samples of cur -> nxt in float (the library's operation order) and in double.

    round_sec > 0: an inter-stage migration with d_min survivors in its worst stage needs r rounds of state
    transfer (d_min * 2^r >= width) and costs inter + round_sec * (r - 1), at most the re-partition cost."""
    if nxt < 0:
        return _F(0.0), 0.0
    full = thr[thr_off[nxt] + configs[nxt][0]]
    e = [max(_F(0.0), _F(_F(tau) - cost[nxt][x])) for x in range(3)]
    e_d = [max(0.0, float(tau) - float(cost[nxt][x])) for x in range(3)]
    if cur < 0 or configs[cur][1] != configs[nxt][1]:
        return _F(full * e[2]), float(full) * e_d[2]
    D, w = int(configs[cur][0]), int(configs[nxt][0])
    n0 = int(bins_int[w:D + 1].sum()) if w <= D else 0
    n01 = int(bins_min[w:D + 1].sum()) if w <= D else 0
    n3 = int(bins_min[0])
    n1, n2 = n01 - n0, S - n01 - n3
    if float(round_sec) == 0.0:
        inter, inter_d = _F(_F(n2) * e[1]), n2 * e_d[1]
    else:
        by_rounds = [0] * 9
        for j in range(1, min(D, w - 1) + 1):
            r = 0
            while (j << r) < w:
                r += 1
            by_rounds[r] += int(bins_min[j])
        inter, inter_d = _F(0.0), 0.0
        for r in range(1, 9):
            c_f = min(_F(cost[nxt][1] + _F(_F(round_sec) * _F(r - 1))), cost[nxt][2])
            c_d = min(float(cost[nxt][1]) + float(round_sec) * (r - 1), float(cost[nxt][2]))
            inter = _F(inter + _F(_F(by_rounds[r]) * max(_F(0.0), _F(_F(tau) - c_f))))
            inter_d += by_rounds[r] * max(0.0, float(tau) - c_d)
    num = _F(_F(_F(n0) * _F(tau)) + _F(_F(n1) * e[0]))
    num = _F(num + inter)
    num = _F(num + _F(_F(n3) * e[2]))
    teff = _F(num / _F(S))
    teff_d = (n0 * float(tau) + n1 * e_d[0] + inter_d + n3 * e_d[2]) / S
    return _F(full * teff), float(full) * teff_d


@dataclass
class ReplayResult:
    chosen: np.ndarray      # [H] configuration of interval i + 1, -1 = suspended
    reward: np.ndarray      # [H] float32
    total: float            # float32 value, rewards added in step order
    total_d: float          # the same in double


def replay(batch, q, true_avail, windows, mode=PROACTIVE, n_threads=1, pool_all=False) -> ReplayResult:
    """Replay query q of `batch` (tables, seed, stream id, starting configuration) over H = len(windows) steps."""
    configs = [(int(d), int(p)) for d, p in batch.configs]
    C, T, S = len(configs), batch.n_intervals, batch.n_scenarios
    group = int(getattr(batch, "group_size", 1))
    thr, cost, off = batch.thr[q], batch.cost[q], batch.thr_off
    thr_full = thr[off[1:] - 1]
    seed, stream = int(batch.seed[q]), int(batch.stream_id[q])
    H = len(windows)
    zone, weight = batch_zones(batch, q)
    rounds = batch_rounds(batch, q)
    assert getattr(batch, "cost_move", None) is None, "the replay does not take a cost per moved instance"
    cur = int(batch.cur_config[q])
    chosen = np.zeros(H, np.int32)
    reward = np.zeros(H, np.float32)
    total, total_d = _F(0.0), 0.0
    for i in range(H):
        a_now, a = int(true_avail[i]), int(true_avail[i + 1])
        if mode == PROACTIVE:
            win = np.asarray(windows[i], np.int32)
            hi, hm = eval_hist(batch.configs, off, win, seed, (stream + 2 * i) & 0xFFFFFFFF, 0, S, n_threads, pool_all, group, zone, weight)
            _, W_f = transition(batch.configs, off, win, thr, cost, batch.interval_sec, S, batch.p_min,
                                cur if cur >= 0 else -2, hi, hm, group, rounds)   # nothing running: cold start
            plan = dp_f32(W_f)
            target = int(plan.plan[0]) if plan.feasible else cur
            forecast = int(win[1])
        else:
            target = reactive_choice(configs, thr_full, batch.p_min, group, a)
            forecast = a
        nxt = adapt(configs, batch.p_min, group, target, a, forecast)
        pair = np.asarray([a_now, a], np.int32)
        hi1, hm1 = eval_hist(batch.configs, off, pair, seed, (stream + 2 * i + 1) & 0xFFFFFFFF, 0, S, n_threads, pool_all,
                             group, zone, weight)
        if cur >= 0:
            sl = slice(off[cur], off[cur + 1])
            r_f, r_d = transition_reward(configs, off, thr, cost, batch.interval_sec, S, cur, nxt, hi1[0, sl], hm1[0, sl],
                                         0.0 if rounds is None or nxt < 0 else rounds[nxt])
        else:
            r_f, r_d = transition_reward(configs, off, thr, cost, batch.interval_sec, S, cur, nxt, None, None)
        chosen[i], reward[i] = nxt, r_f
        total = _F(total + r_f)
        total_d += r_d
        cur = nxt
    return ReplayResult(chosen, reward, float(total), total_d)
