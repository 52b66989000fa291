"""GPU library against the CPU oracle, element by element, through the C ABI.

Integers (masks, survivor counts, histograms, back-pointers, plans) must be bit-equal.  Float tables must be
bit-equal to the oracle's fixed-order float values and within 1e-5 relative of its double values.
"""
import numpy as np
import pytest

import oracle
import parcae_inputs as pi

pytestmark = pytest.mark.gpu

REL = 1e-5


@pytest.fixture(scope="module")
def pk():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2403_14097_amd as mod
    mod.load_library()
    return mod


def _np(t, dtype=None):
    a = t.detach().cpu().numpy()
    return a.view(dtype) if dtype is not None else a


def _sync():
    import torch
    torch.cuda.synchronize()


def _check_query_against_oracle(pk, batch, q, ev, pl, S, threads=8, check_W=None):
    """Full comparison of one query's outputs with the oracle run at S scenarios."""
    r = oracle.run_query(batch, q, n_scenarios=S, n_threads=threads)
    assert np.array_equal(_np(ev.hist_int[q], np.uint32), r.hist_int), "hist_int"
    assert np.array_equal(_np(ev.hist_min[q], np.uint32), r.hist_min), "hist_min"
    if ev.liveput is not None:
        for name, got, f, d in (("liveput", _np(ev.liveput[q]), r.tables.liveput_f, r.tables.liveput_d),
                                ("teff", _np(ev.teff[q]), r.tables.teff_f, r.tables.teff_d),
                                ("gain", _np(ev.gain[q]), r.tables.gain_f, r.tables.gain_d)):
            assert np.array_equal(got, f), name
            assert np.all(np.abs(got - d) <= REL * np.abs(d)), name
    if pl is not None:
        assert np.array_equal(_np(pl.bp[q]), r.plan.bp), "bp"
        assert np.array_equal(_np(pl.F[q]), r.plan.F), "F"        # -inf == -inf holds
        assert np.array_equal(_np(pl.plan[q]), r.plan.plan), "plan"
        assert int(pl.start[q]) == r.plan.start
        obj = float(pl.objective[q])
        assert obj == r.plan.objective
        if r.plan.feasible:
            assert abs(obj - r.objective_d) <= REL * abs(r.objective_d)
            assert int(pl.status[q]) == pk.PARCAE_OK
        else:
            assert int(pl.status[q]) == pk.PARCAE_EINFEASIBLE
    if check_W is not None:
        assert np.array_equal(_np(check_W[q]), r.W_f), "W"
        fin = np.isfinite(r.W_d)
        assert np.all(np.abs(_np(check_W[q])[fin] - r.W_d[fin]) <= REL * np.abs(r.W_d[fin]))
    return r


# ------------------------------------------------------------------ scenarios one by one

UNITS = [
    # D, P, a_next  (k = max(0, D*P - a_next))
    (1, 1, 0), (1, 1, 1), (4, 2, 5), (2, 4, 3), (3, 4, 10), (8, 1, 3), (2, 3, 4), (3, 2, 4),
    (16, 2, 20), (8, 4, 9), (4, 8, 30), (2, 16, 17), (1, 32, 20), (2, 32, 50), (16, 4, 40), (8, 8, 1),
    (5, 7, 20), (3, 13, 30), (9, 11, 60), (17, 15, 200), (64, 2, 100), (32, 4, 64), (16, 8, 100),
    (8, 16, 97), (4, 32, 96), (2, 64, 100), (1, 128, 77), (256, 1, 130), (128, 2, 3), (64, 4, 250),
    (32, 8, 128), (16, 16, 255), (8, 32, 129), (4, 64, 192), (2, 128, 128), (1, 256, 255), (1, 256, 0),
    (3, 64, 100), (1, 64, 40), (2, 96, 150), (7, 32, 100), (5, 40, 120), (12, 20, 100),
    # depths that are not powers of two, every mask width: 3..7, 9..31, above 32
    (10, 3, 20), (21, 3, 40), (42, 3, 100), (85, 3, 200), (6, 5, 21), (12, 5, 33), (25, 5, 90), (51, 5, 140),
    (5, 6, 19), (10, 6, 41), (21, 6, 100), (42, 6, 131), (4, 7, 20), (9, 7, 50), (18, 7, 77), (36, 7, 200),
    (3, 9, 20), (7, 9, 40), (14, 9, 100), (28, 9, 130), (2, 12, 15), (5, 12, 31), (10, 12, 75), (21, 12, 200),
    (2, 15, 22), (4, 15, 40), (8, 15, 70), (1, 23, 11), (2, 23, 30), (5, 23, 80), (11, 23, 150),
    (1, 31, 20), (2, 31, 40), (4, 31, 65), (8, 31, 200), (1, 33, 20), (3, 33, 60), (7, 33, 100),
    (1, 48, 30), (2, 48, 50), (5, 48, 129), (1, 63, 40), (4, 63, 150), (1, 65, 33), (3, 65, 111),
    (2, 100, 120), (1, 129, 100), (1, 200, 99), (1, 255, 128), (2, 127, 130),
]


def test_scenarios_match_oracle_one_by_one(pk):
    """Masks, n_int and d_min of individual scenarios: every mask width, both Floyd branches, any depth."""
    configs = sorted({(d, p) for d, p, _ in UNITS}, key=lambda x: (x[1], x[0]))
    cfg = np.asarray(configs, np.int32)
    avs = sorted({a for _, _, a in UNITS})
    # one query; interval t has availability avs[t]
    b = pi.custom_batch(256, cfg, [[256] + avs], thr_per_pipeline=[1.0] * len(cfg), n_scenarios=64, seed=1234)
    b.stream_id[:] = 5
    p = pk.upload(b)
    ns, s0 = 192, 1000
    for D, P, a in UNITS:
        c = configs.index((D, P))
        t = avs.index(a)
        masks, n_int, d_min = pk.parcae_debug_sample(p, 0, t, c, s0, ns)
        _sync()
        om, oi, od = oracle.debug_sample(D, P, a, int(b.seed[0]), 5, t * len(cfg) + c, s0, ns)
        assert np.array_equal(_np(masks, np.uint32), om), (D, P, a)
        assert np.array_equal(_np(n_int), oi), (D, P, a)
        assert np.array_equal(_np(d_min), od), (D, P, a)


# ------------------------------------------------------------------ whole path on the small workloads

@pytest.mark.parametrize("name", ["tiny", "small"])
def test_full_workload_parity(pk, name):
    b = pi.workload(name)
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    _check_query_against_oracle(pk, b, 0, ev, pl, b.n_scenarios, check_W=W)
    # the three ways to the plan agree: fused, from stored histograms, from stored weights
    pl2 = pk.parcae_plan_from_hist(p, ev.hist_int, ev.hist_min)
    pl3 = pk.parcae_dp_plan(W)
    _sync()
    for other in (pl2, pl3):
        for f in ("F", "bp", "plan", "start", "objective", "status"):
            assert np.array_equal(_np(getattr(other, f)), _np(getattr(pl, f))), f
    # eval alone gives the same tables and a per-query status
    ev2 = pk.parcae_liveput_eval(p)
    _sync()
    for f in ("hist_int", "hist_min", "liveput", "teff", "gain"):
        assert np.array_equal(_np(getattr(ev2, f)), _np(getattr(ev, f))), f
    assert int(ev2.status[0]) == pk.PARCAE_OK


@pytest.mark.parametrize("name,S,dense", [("medium", 1500, False), ("medium", 777, True), ("large", 640, False),
                                          ("large", 200, True), ("large", 4096, False)])
def test_prefix_parity_on_larger_workloads(pk, name, S, dense):
    """Scenario s does not depend on the scenario count, so a prefix of a big workload is a full parity case.
    S values are ragged (not multiples of the wave or block size)."""
    b = pi.workload(name, dense=dense, n_scenarios=S)
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    _check_query_against_oracle(pk, b, 0, ev, pl, S, check_W=W)


def test_batched_queries_parity(pk):
    """Several queries in one launch, each with its own walk, tables, seed and current configuration."""
    b = pi.workload("sweep", n_queries=6, n_scenarios=1000)
    b.stream_id[:] = np.arange(6, dtype=np.uint32) * 7
    b.cur_config[3] = -1
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    for q in range(6):
        _check_query_against_oracle(pk, b, q, ev, pl, 1000, check_W=W)


@pytest.mark.parametrize("name,nq,S", [("medium", 2, 300), ("medium", 3, 200), ("small", 5, 333), ("small", 6, 257)])
def test_batches_on_either_side_of_the_one_launch_staging(pk, name, nq, S):
    """Small batches are staged by a single workgroup (table, histogram rows, work list), larger ones by three
    kernels; 1800 and 1800 units take the first route (the second round of the workgroup's loop too), 2700 and 2160
    the other.  Everything the call writes is compared for every query."""
    b = pi.workload(name, n_queries=nq, n_scenarios=S)
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    for q in range(nq):
        _check_all_outputs(pk, b, q, ev, pl, W, S)
    # the evaluation alone takes the same staging and writes the same histograms and tables
    ev2 = pk.parcae_liveput_eval(p)
    _sync()
    for f in ("hist_int", "hist_min", "liveput", "teff", "gain"):
        assert np.array_equal(_np(getattr(ev, f)), _np(getattr(ev2, f))), f


@pytest.mark.parametrize("keep", ["liveput", "teff", "gain"])
def test_a_single_table_from_the_planning_call(pk, keep):
    """The planner's launch writes the liveput tables the caller asked for and leaves the others alone."""
    b = pi.workload("small", n_scenarios=500)
    p = pk.upload(b)
    full, _ = pk.parcae_liveput_plan(p)
    _sync()
    ev = pk.alloc_eval_out(p)
    for f in ("liveput", "teff", "gain"):
        if f != keep:
            setattr(ev, f, None)
    pl = pk.alloc_plan_out(p)
    pk.parcae_liveput_plan(p, ev, pl)
    _sync()
    assert np.array_equal(_np(getattr(ev, keep)), _np(getattr(full, keep)))
    r = oracle.run_query(b, 0, n_scenarios=500)
    assert np.array_equal(_np(pl.plan[0]), r.plan.plan)


def test_many_queries_take_the_per_query_planning_kernel(pk):
    """Forty queries: enough for the one-block-per-query planner (weights formed on the fly in LDS)."""
    b = pi.workload("sweep", n_queries=40, n_scenarios=300)
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    for q in (0, 7, 39):
        _check_query_against_oracle(pk, b, q, ev, pl, 300)
    # the same plans from weights in memory, with and without the optional outputs
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    pl2 = pk.parcae_dp_plan(W)
    lean = pk.alloc_plan_out(p, full=False)
    lean.bp = pl2.bp.clone()
    pk.parcae_dp_plan(W, lean)
    _sync()
    for f in ("F", "bp", "plan", "start", "objective", "status"):
        assert np.array_equal(_np(getattr(pl2, f)), _np(getattr(pl, f))), f
    assert np.array_equal(_np(lean.plan), _np(pl.plan)) and np.array_equal(_np(lean.objective), _np(pl.objective))
    # no back-pointer output at all: they fit in local memory here (2 * 30 * 30 bytes)
    bare = pk.alloc_plan_out(p, full=False)
    pk.parcae_dp_plan(W, bare)
    _sync()
    assert np.array_equal(_np(bare.plan), _np(pl.plan)) and np.array_equal(_np(bare.start), _np(pl.start))


def test_per_query_planning_kernel_with_rows_that_do_not_fit_in_lds_at_once(pk):
    """33 queries on 128 instances with every depth listed (296 candidates, 12 thousand histogram bins per
    step): the per-query planner has to bring the source rows in several chunks; many depths, cold start and a
    free start among the queries."""
    spec = pi.WorkloadSpec("wide", 33, 128, 5, 60.0, (1, 2, 3, 4, 8, 16, 32, 64), 1, 10, 32, 0.2, False, 4, 96)
    b = pi.make_batch(spec, seed=606)
    b.cur_config[3] = -1
    b.cur_config[4] = -2
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    for q in (0, 3, 4, 32):
        _check_query_against_oracle(pk, b, q, ev, pl, 96)


def test_dp_on_stored_weights_all_kernel_variants(pk):
    """Weights in memory: tiles staged in LDS (C <= 64), read in place (one block), and one launch per step."""
    for name, dense, S in (("small", False, 200), ("medium", True, 100), ("large", True, 64)):
        b = pi.workload(name, dense=dense, n_scenarios=S)
        p = pk.upload(b)
        ev = pk.parcae_liveput_eval(p)
        W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
        _sync()
        r = oracle.run_query(b, 0, n_scenarios=S, n_threads=8)
        assert np.array_equal(_np(W[0]), r.W_f)
        full = pk.parcae_dp_plan(W)                       # F wanted: stepwise launches when C is large
        lean = pk.alloc_plan_out(p, full=False)           # no F: one block per query
        lean.bp = full.bp.clone().zero_()
        pk.parcae_dp_plan(W, lean)
        _sync()
        assert np.array_equal(_np(full.F[0]), r.plan.F) and np.array_equal(_np(full.bp[0]), r.plan.bp)
        assert np.array_equal(_np(lean.bp[0]), r.plan.bp)
        for out in (full, lean):
            assert np.array_equal(_np(out.plan[0]), r.plan.plan) and int(out.start[0]) == r.plan.start
            assert float(out.objective[0]) == r.plan.objective


def test_multi_chunk_and_ragged_scenario_counts(pk):
    """Scenario counts around the block chunking (2048 per block) and the wave size."""
    base = pi.workload("small")
    for S in (1, 63, 65, 2047, 2049, 4097, 5000):
        b = base.with_scenarios(S)
        p = pk.upload(b)
        ev = pk.parcae_liveput_eval(p)
        _sync()
        hi, hm = oracle.eval_hist(b.configs, b.thr_off, b.avail[0], int(b.seed[0]), 0, 0, S, 8)
        assert np.array_equal(_np(ev.hist_int[0], np.uint32), hi), S
        assert np.array_equal(_np(ev.hist_min[0], np.uint32), hm), S


# ------------------------------------------------------------------ full sizes, sampled

def _sampled_unit_check(pk, b, ev, rng, n_samples, S):
    C, T = b.n_configs, b.n_intervals
    used = b.configs[:, 0] * b.configs[:, 1]
    hi_all = _np(ev.hist_int, np.uint32)
    hm_all = _np(ev.hist_min, np.uint32)
    # properties that hold at any size: every unit's bins sum to S; units without sampling have one bin
    sums_i = np.add.reduceat(hi_all, b.thr_off[:-1], axis=2)
    sums_m = np.add.reduceat(hm_all, b.thr_off[:-1], axis=2)
    assert np.all(sums_i == S) and np.all(sums_m == S)
    k = np.maximum(0, used[None, None, :] - b.avail[:, 1:, None])
    top = hi_all[:, :, b.thr_off[1:] - 1]
    assert np.all(top[k == 0] == S)
    # sampled non-trivial units, computed one by one by the oracle
    nz = np.argwhere((k > 0) & (k < used[None, None, :]))
    pick = nz[rng.choice(len(nz), size=min(n_samples, len(nz)), replace=False)]
    for q, t, c in pick:
        D, P = b.configs[c]
        hi, hm = oracle.eval_unit(int(D), int(P), int(b.avail[q, t + 1]), int(b.seed[q]), int(b.stream_id[q]),
                                  int(t * C + c), 0, S)
        sl = slice(b.thr_off[c], b.thr_off[c + 1])
        assert np.array_equal(hi_all[q, t, sl], hi), (q, t, c)
        assert np.array_equal(hm_all[q, t, sl], hm), (q, t, c)
    return len(pick)


def _plan_check_from_gpu_histograms(pk, b, q, ev, pl):
    """DP parity at full size: the oracle's tables and plan from the (already verified) integer histograms."""
    S = b.n_scenarios
    hi = _np(ev.hist_int[q], np.uint32)
    hm = _np(ev.hist_min[q], np.uint32)
    tab = oracle.finalise(b.configs, b.thr_off, b.avail[q], b.thr[q], b.cost[q], b.interval_sec, S, hi, hm)
    assert np.array_equal(_np(ev.liveput[q]), tab.liveput_f)
    assert np.array_equal(_np(ev.teff[q]), tab.teff_f) and np.array_equal(_np(ev.gain[q]), tab.gain_f)
    assert np.all(np.abs(_np(ev.gain[q]) - tab.gain_d) <= REL * np.abs(tab.gain_d))
    W_d, W_f = oracle.transition(b.configs, b.thr_off, b.avail[q], b.thr[q], b.cost[q], b.interval_sec, S, b.p_min,
                                 int(b.cur_config[q]), hi, hm)
    ref = oracle.dp_f32(W_f)
    assert np.array_equal(_np(pl.bp[q]), ref.bp) and np.array_equal(_np(pl.F[q]), ref.F)
    assert np.array_equal(_np(pl.plan[q]), ref.plan) and int(pl.start[q]) == ref.start
    assert float(pl.objective[q]) == ref.objective
    assert abs(ref.objective - oracle.dp_f64(W_d)) <= REL * abs(ref.objective)


@pytest.mark.parametrize("name", ["medium", "large"])
def test_full_size_single_query_sampled(pk, name):
    b = pi.workload(name)
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    n = _sampled_unit_check(pk, b, ev, np.random.default_rng(5), 24 if name == "large" else 60, b.n_scenarios)
    assert n > 0
    _plan_check_from_gpu_histograms(pk, b, 0, ev, pl)


def test_full_size_sweep_sampled(pk):
    """The 1024-query what-if sweep in the launch configuration the benchmark times."""
    b = pi.workload("sweep")
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    rng = np.random.default_rng(11)
    n = _sampled_unit_check(pk, b, ev, rng, 300, b.n_scenarios)
    assert n == 300
    assert np.all(_np(pl.status) == 0)
    for q in rng.choice(b.n_queries, size=24, replace=False):
        _plan_check_from_gpu_histograms(pk, b, int(q), ev, pl)
    for q in (0, 1023):
        _check_query_against_oracle(pk, b, q, ev, pl, b.n_scenarios)


@pytest.mark.parametrize("name,units,plans", [("medium", 120, 6), ("large", 24, 2)])
def test_full_size_batches_of_256_queries_sampled(pk, name, units, plans):
    """256 queries of the medium and of the large shape in one launch, at their full scenario counts: the launch
    configurations the benchmark reports beside the sweep.  Sampled units against the oracle, every status, and the
    tables and plans of a few queries from the histograms the GPU produced."""
    b = pi.workload(name, n_queries=256)
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    rng = np.random.default_rng(23)
    n = _sampled_unit_check(pk, b, ev, rng, units, b.n_scenarios)
    assert n == units
    assert np.all(_np(pl.status) == 0)
    for q in rng.choice(b.n_queries, size=plans, replace=False):
        _plan_check_from_gpu_histograms(pk, b, int(q), ev, pl)


def _closed_form_rows(b, q, k, S):
    """Histogram [T, L] of query q holding only the units whose scenarios are all alike by the definition of the
    draw: nothing preempted (k = 0: every pipeline intact, bin D) or everything preempted (k = M: bin 0)."""
    T, L = b.n_intervals, b.hist_len
    out = np.zeros((T, L), np.uint32)
    used = b.configs[:, 0] * b.configs[:, 1]
    for c in range(b.n_configs):
        none = k[q, :, c] == 0
        out[none, b.thr_off[c] + b.configs[c, 0]] = S
        out[k[q, :, c] == used[c], b.thr_off[c]] = S
    return out


def test_full_size_sweep_every_unit_of_every_query(pk):
    """The 1024-query sweep in the benchmark's launch configuration, whole: both histograms of every unit of every
    query against the oracle (units that the definition makes trivial, k = 0 or k = M by the oracle's own pool
    rule, against their single bin; every other unit sampled by the oracle, also those the library writes in
    closed form), then tables, value function, back-pointers and plan of every query."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    b = pi.workload("sweep")
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    S, nq = b.n_scenarios, b.n_queries
    hi_all, hm_all = _np(ev.hist_int, np.uint32), _np(ev.hist_min, np.uint32)
    used = b.configs[:, 0] * b.configs[:, 1]
    k = np.maximum(0, used[None, None, :] - b.avail[:, 1:, None])          # pool of used instances (section 4.2)
    want = ((k > 0) & (k < used[None, None, :])).astype(np.uint8)
    assert 0.3 < want.mean() < 0.5

    def check(q):
        oi, om = oracle.eval_hist(b.configs, b.thr_off, b.avail[q], int(b.seed[q]), int(b.stream_id[q]), 0, S, 1,
                                  want=want[q])
        easy = _closed_form_rows(b, q, k, S)
        return bool(np.array_equal(hi_all[q], oi + easy) and np.array_equal(hm_all[q], om + easy))

    workers = max(1, min(16, os.cpu_count() or 1))
    with ThreadPoolExecutor(workers) as pool:          # the C oracle runs outside the interpreter lock
        ok = list(pool.map(check, range(nq)))
    assert all(ok), [q for q, good in enumerate(ok) if not good][:10]
    assert np.all(_np(pl.status) == 0)

    def check_plan(q):
        _plan_check_from_gpu_histograms(pk, b, q, ev, pl)
        return True

    ev_np = type(ev)(*[None if t is None else t.cpu() for t in (ev.hist_int, ev.hist_min, ev.liveput, ev.teff, ev.gain, ev.status)])
    pl_np = type(pl)(*[None if t is None else t.cpu() for t in (pl.F, pl.bp, pl.plan, pl.start, pl.objective, pl.status)])
    ev, pl = ev_np, pl_np                               # host copies: the per-query checks slice them 1024 times
    with ThreadPoolExecutor(workers) as pool:
        assert all(pool.map(check_plan, range(nq)))


# ------------------------------------------------------------------ whole-cluster preemption pool

def test_pool_all_scenarios_one_by_one(pk):
    """Preemptions drawn among all available instances: masks cover the pool, the grid is its first D * P bits."""
    cases = [  # D, P, a_prev, a_next
        (3, 4, 20, 13), (2, 8, 30, 25), (4, 8, 64, 40), (2, 16, 64, 10), (1, 32, 50, 33), (16, 4, 100, 70),
        (8, 16, 200, 120), (2, 64, 256, 130), (32, 1, 40, 22), (1, 8, 20, 9), (5, 7, 60, 31), (4, 4, 16, 9), (4, 4, 12, 9),
        (3, 32, 256, 1), (6, 2, 12, 12), (6, 2, 40, 0),
    ]
    configs = sorted({(d, p) for d, p, _, _ in cases}, key=lambda x: (x[1], x[0]))
    cfg = np.asarray(configs, np.int32)
    b = pi.custom_batch(256, cfg, [[256, 256]], thr_per_pipeline=[1.0] * len(cfg), n_scenarios=64, seed=99)
    ns, s0 = 160, 7
    for D, P, a_prev, a_next in cases:
        b.avail[0, :] = (a_prev, a_next)
        p = pk.upload(b)
        p.flags = pk.PARCAE_POOL_ALL
        c = configs.index((D, P))
        masks, n_int, d_min = pk.parcae_debug_sample(p, 0, 0, c, s0, ns)
        _sync()
        om, oi, od = oracle.debug_sample(D, P, a_next, int(b.seed[0]), 0, c, s0, ns, a_prev=a_prev)
        assert np.array_equal(_np(masks, np.uint32), om), (D, P, a_prev, a_next)
        assert np.array_equal(_np(n_int), oi) and np.array_equal(_np(d_min), od), (D, P, a_prev, a_next)


@pytest.mark.parametrize("name,S,nq", [("tiny", 256, 1), ("small", 1000, 1), ("large", 300, 1), ("sweep", 500, 40)])
def test_pool_all_full_parity(pk, name, S, nq):
    b = pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None)
    p = pk.upload(b)
    p.flags = pk.PARCAE_POOL_ALL
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    for q in sorted({0, nq - 1}):
        r = oracle.run_query(b, q, n_scenarios=S, n_threads=8, pool_all=True)
        assert np.array_equal(_np(ev.hist_int[q], np.uint32), r.hist_int)
        assert np.array_equal(_np(ev.hist_min[q], np.uint32), r.hist_min)
        assert np.array_equal(_np(ev.liveput[q]), r.tables.liveput_f) and np.array_equal(_np(ev.gain[q]), r.tables.gain_f)
        assert np.array_equal(_np(ev.teff[q]), r.tables.teff_f)
        assert np.all(np.abs(_np(ev.gain[q]) - r.tables.gain_d) <= REL * np.abs(r.tables.gain_d))
        assert np.array_equal(_np(W[q]), r.W_f)
        assert np.array_equal(_np(pl.bp[q]), r.plan.bp) and np.array_equal(_np(pl.F[q]), r.plan.F)
        assert np.array_equal(_np(pl.plan[q]), r.plan.plan) and float(pl.objective[q]) == r.plan.objective


# ------------------------------------------------------------------ multi-GPU instances

def test_grouped_instances_scenarios_one_by_one(pk):
    cases = [  # D, P, g, a_prev (-1: used pool), a_next   -- availability in instances
        (8, 3, 4, -1, 5), (4, 2, 2, -1, 3), (16, 4, 4, -1, 9), (32, 8, 4, -1, 40), (64, 4, 8, -1, 20),
        (8, 16, 2, -1, 50), (12, 5, 3, -1, 13), (8, 4, 2, 30, 22), (16, 8, 4, 60, 33), (6, 7, 2, 40, 25),
        (8, 32, 8, -1, 20), (128, 2, 64, -1, 3),
    ]
    for D, P, g, a_prev, a_next in cases:
        cfg = np.asarray([[D, P]], np.int32)
        b = pi.custom_batch(256, cfg, [[max(a_prev, 0), a_next]], thr_per_pipeline=[1.0], n_scenarios=64, seed=5,
                            group_size=g)
        p = pk.upload(b)
        if a_prev >= 0:
            p.flags = pk.PARCAE_POOL_ALL
        masks, n_int, d_min = pk.parcae_debug_sample(p, 0, 0, 0, 3, 128)
        _sync()
        om, oi, od = oracle.debug_sample(D, P, a_next, int(b.seed[0]), 0, 0, 3, 128, a_prev=a_prev, group=g)
        assert np.array_equal(_np(masks, np.uint32), om), (D, P, g)
        assert np.array_equal(_np(n_int), oi) and np.array_equal(_np(d_min), od), (D, P, g)
        assert np.all(_np(n_int) % g == 0) and np.all(_np(d_min) % g == 0)


@pytest.mark.parametrize("pool_all", [False, True])
def test_grouped_instances_full_parity(pk, pool_all):
    """Four-GPU instances: 64 instances, candidates in blocks of four pipelines, 40 queries and 1 query."""
    for nq in (1, 40):
        spec = pi.WorkloadSpec("quad", nq, 64, 10, 60.0, (2, 4, 8, 16), 2, 6, 16, 0.1, False, 2, 700)
        b = pi.make_batch(spec, seed=21)
        # the walks of the drawn batch (in instances) on candidates counted in GPUs: D * P up to 4 * 64
        cfg = pi.candidate_list(256, (2, 4, 8, 16), 2)
        cfg = cfg[(cfg[:, 0] % 4 == 0) & (cfg[:, 0] * cfg[:, 1] <= 256) & (cfg[:, 0] <= 64)]
        g = pi.custom_batch(64, cfg, b.avail, thr_per_pipeline=[1.0 + 0.05 * p for _, p in cfg], n_scenarios=700,
                            p_min=2, group_size=4, seed=8)
        p = pk.upload(g)
        if pool_all:
            p.flags = pk.PARCAE_POOL_ALL
        ev, pl = pk.parcae_liveput_plan(p)
        W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
        _sync()
        for q in sorted({0, nq - 1}):
            r = oracle.run_query(g, q, n_threads=8, pool_all=pool_all)
            assert np.array_equal(_np(ev.hist_int[q], np.uint32), r.hist_int)
            assert np.array_equal(_np(ev.hist_min[q], np.uint32), r.hist_min)
            assert np.array_equal(_np(ev.liveput[q]), r.tables.liveput_f)
            assert np.array_equal(_np(ev.teff[q]), r.tables.teff_f) and np.array_equal(_np(ev.gain[q]), r.tables.gain_f)
            assert np.array_equal(_np(W[q]), r.W_f)
            assert np.array_equal(_np(pl.bp[q]), r.plan.bp) and np.array_equal(_np(pl.F[q]), r.plan.F)
            assert np.array_equal(_np(pl.plan[q]), r.plan.plan) and float(pl.objective[q]) == r.plan.objective


# ------------------------------------------------------------------ non-uniform preemption (zones)

def _with_zone_arrays(b, zone, weight):
    b.n_zones = len(weight)
    b.zone = np.ascontiguousarray(np.broadcast_to(np.asarray(zone, np.uint8), (b.n_queries, b.n_instances)))
    w = np.ones((b.n_queries, pi.MAX_ZONES), np.uint32)
    w[:, : len(weight)] = weight
    b.zone_weight = w
    return b


def test_zoned_scenarios_one_by_one(pk):
    """Weighted draws: every mask width, zones with no member in the pool, counts past the half, idle instances,
    multi-GPU instances."""
    rng = pi.SplitMix64(4242)
    cases = [  # D, P, group, a_prev (-1: used pool), a_next, weights
        (2, 3, 1, -1, 4, [1, 6]), (3, 4, 1, -1, 7, [5, 1, 2]), (8, 4, 1, -1, 20, [1, 2, 3, 4]), (4, 8, 1, -1, 6, [9, 1]),
        (16, 4, 1, -1, 33, [1, 255, 7]), (8, 8, 1, -1, 60, [3, 3, 3, 3]), (2, 32, 1, -1, 31, [2, 1, 8]),
        (16, 8, 1, -1, 100, [1, 4, 2, 9]), (4, 32, 1, -1, 20, [7, 2]), (32, 8, 1, -1, 128, [1, 3, 5, 7]),
        (2, 128, 1, -1, 250, [4, 1, 1, 6]), (1, 256, 1, -1, 3, [1, 200, 30]), (5, 7, 1, -1, 18, [2, 5, 1]),
        (11, 23, 1, -1, 140, [1, 9]), (3, 65, 1, -1, 111, [6, 1, 3]), (64, 1, 1, 80, 41, [1, 5]),
        (3, 4, 1, 20, 13, [8, 1, 3]), (8, 16, 1, 200, 120, [1, 2, 4, 8]), (16, 4, 4, -1, 9, [1, 7]),
        (8, 4, 2, 30, 22, [3, 1, 9]), (6, 2, 1, -1, 12, [1, 2]), (6, 2, 1, -1, 0, [1, 2]), (7, 9, 1, -1, 62, [1, 1, 1, 50]),
    ]
    for D, P, g, a_prev, a_next, weight in cases:
        cfg = np.asarray([[D, P]], np.int32)
        b = pi.custom_batch(256, cfg, [[max(a_prev, 0), a_next]], thr_per_pipeline=[1.0], n_scenarios=64, seed=17,
                            group_size=g)
        zone = [rng.randint(0, len(weight) - 1) for _ in range(256)]
        if len(weight) == 4:
            zone = [z if z != 2 or j > 40 else 0 for j, z in enumerate(zone)]   # zone 2 is empty in small pools
        _with_zone_arrays(b, zone, weight)
        b.stream_id[:] = 9
        p = pk.upload(b)
        if a_prev >= 0:
            p.flags = pk.PARCAE_POOL_ALL
        ns, s0 = 200, 31
        masks, n_int, d_min = pk.parcae_debug_sample(p, 0, 0, 0, s0, ns)
        _sync()
        om, oi, od = oracle.debug_sample(D, P, a_next, int(b.seed[0]), 9, 0, s0, ns, a_prev=a_prev, group=g,
                                         zone=b.zone[0], weight=weight)
        assert np.array_equal(_np(masks, np.uint32), om), (D, P, g, a_prev, a_next)
        assert np.array_equal(_np(n_int), oi) and np.array_equal(_np(d_min), od), (D, P, g, a_prev, a_next)


def test_one_zone_gives_the_uniform_results(pk):
    b = pi.workload("small", n_scenarios=600)
    ev_u, pl_u = pk.parcae_liveput_plan(pk.upload(b))
    z = _with_zone_arrays(pi.workload("small", n_scenarios=600), [0] * 32, [37])
    ev_z, pl_z = pk.parcae_liveput_plan(pk.upload(z))
    _sync()
    assert np.array_equal(_np(ev_u.hist_int), _np(ev_z.hist_int)) and np.array_equal(_np(ev_u.hist_min), _np(ev_z.hist_min))
    assert np.array_equal(_np(pl_u.plan), _np(pl_z.plan))


@pytest.mark.parametrize("name,S,nq,pool_all", [("tiny", 256, 1, False), ("small", 1000, 1, False),
                                                ("medium", 700, 1, True), ("large", 300, 1, False),
                                                ("sweep", 500, 40, False), ("sweep", 300, 36, True)])
def test_zoned_full_parity(pk, name, S, nq, pool_all):
    b = pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None).with_zones(3 if name != "large" else 4)
    p = pk.upload(b)
    if pool_all:
        p.flags = pk.PARCAE_POOL_ALL
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    for q in sorted({0, nq // 2, nq - 1}):
        r = oracle.run_query(b, q, n_scenarios=S, n_threads=8, pool_all=pool_all)
        assert np.array_equal(_np(ev.hist_int[q], np.uint32), r.hist_int)
        assert np.array_equal(_np(ev.hist_min[q], np.uint32), r.hist_min)
        assert np.array_equal(_np(ev.liveput[q]), r.tables.liveput_f) and np.array_equal(_np(ev.gain[q]), r.tables.gain_f)
        assert np.array_equal(_np(ev.teff[q]), r.tables.teff_f)
        assert np.all(np.abs(_np(ev.gain[q]) - r.tables.gain_d) <= REL * np.abs(r.tables.gain_d))
        assert np.array_equal(_np(W[q]), r.W_f)
        assert np.array_equal(_np(pl.bp[q]), r.plan.bp) and np.array_equal(_np(pl.F[q]), r.plan.F)
        assert np.array_equal(_np(pl.plan[q]), r.plan.plan) and float(pl.objective[q]) == r.plan.objective
    # the weights matter: the same batch without zones gives other histograms
    u = pk.upload(pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None))
    if pool_all:
        u.flags = pk.PARCAE_POOL_ALL
    ev_u = pk.parcae_liveput_eval(u)
    _sync()
    assert not np.array_equal(_np(ev_u.hist_min), _np(ev.hist_min))


def test_zoned_full_size_sweep_sampled(pk):
    """The 1024-query sweep at its full scenario count with three zones: sampled units against the oracle."""
    b = pi.workload("sweep").with_zones(3)
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    hi, hm = _np(ev.hist_int, np.uint32), _np(ev.hist_min, np.uint32)
    T, C, S = b.n_intervals, b.n_configs, b.n_scenarios
    assert np.all(hi.reshape(b.n_queries, T, -1).sum(axis=2) == C * S)
    rng = pi.SplitMix64(99)
    checked = 0
    while checked < 24:
        q, t, c = rng.randint(0, b.n_queries - 1), rng.randint(0, T - 1), rng.randint(0, C - 1)
        D, P = (int(x) for x in b.configs[c])
        k = max(0, D * P - int(b.avail[q, t + 1]))
        if k == 0 or k == D * P:
            continue
        zone, weight = oracle.batch_zones(b, q)
        oi, om = oracle.eval_unit(D, P, int(b.avail[q, t + 1]), int(b.seed[q]), int(b.stream_id[q]), t * C + c, 0, S,
                                  zone=zone, weight=weight)
        sl = slice(int(b.thr_off[c]), int(b.thr_off[c + 1]))
        assert np.array_equal(hi[q, t, sl], oi) and np.array_equal(hm[q, t, sl], om), (q, t, c)
        checked += 1
    assert np.all(_np(pl.status) == 0)


def test_invalid_zone_data_is_flagged_per_query(pk):
    b = pi.workload("sweep", n_scenarios=128, n_queries=6).with_zones(3)
    b.zone[1, 5] = 3            # zone index out of range
    b.zone_weight[2, 1] = 0     # weight below 1
    b.zone_weight[4, 0] = 256   # weight above 255
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    st = _np(pl.status)
    assert list(st) == [0, pk.PARCAE_EINVAL, pk.PARCAE_EINVAL, 0, pk.PARCAE_EINVAL, 0]
    r = oracle.run_query(b, 3, n_threads=4)
    assert np.array_equal(_np(ev.hist_int[3], np.uint32), r.hist_int) and np.array_equal(_np(pl.plan[3]), r.plan.plan)
    # host-visible errors
    p.n_zones = 5
    with pytest.raises(pk.ParcaeError):
        pk.parcae_liveput_plan(p)
    p.n_zones, p.zone = 3, None
    with pytest.raises(pk.ParcaeError):
        pk.parcae_liveput_plan(p)


# ------------------------------------------------------------------ inter-stage cost by transfer rounds

@pytest.mark.parametrize("name,S,nq,dense,extra", [("tiny", 256, 1, False, ""), ("small", 1000, 1, False, ""),
                                                    ("medium", 600, 1, True, ""), ("large", 300, 1, False, "pool"),
                                                    ("sweep", 500, 40, False, ""), ("sweep", 300, 33, False, "zones")])
def test_transfer_round_costs_full_parity(pk, name, S, nq, dense, extra):
    """Every planning kernel (weights in memory for few queries, on the fly for many) and the tables."""
    b = pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None, dense=dense).with_rounds()
    if extra == "zones":
        b = b.with_zones(3)
    b.cost_round[:, ::5] = 0.0                 # some candidates keep the fixed inter-stage cost
    b.cost_round[:, 1::7] = 45.0               # some hit the re-partition cap at once
    p = pk.upload(b)
    if extra == "pool":
        p.flags = pk.PARCAE_POOL_ALL
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    for q in sorted({0, nq // 2, nq - 1}):
        r = oracle.run_query(b, q, n_scenarios=S, n_threads=8, pool_all=(extra == "pool"))
        assert np.array_equal(_np(ev.hist_int[q], np.uint32), r.hist_int)
        assert np.array_equal(_np(ev.hist_min[q], np.uint32), r.hist_min)
        assert np.array_equal(_np(ev.teff[q]), r.tables.teff_f) and np.array_equal(_np(ev.gain[q]), r.tables.gain_f)
        assert np.all(np.abs(_np(ev.gain[q]) - r.tables.gain_d) <= REL * np.abs(r.tables.gain_d))
        assert np.array_equal(_np(W[q]), r.W_f)
        fin = np.isfinite(r.W_d)
        assert np.all(np.abs(_np(W[q])[fin] - r.W_d[fin]) <= REL * np.abs(r.W_d[fin]))
        assert np.array_equal(_np(pl.bp[q]), r.plan.bp) and np.array_equal(_np(pl.F[q]), r.plan.F)
        assert np.array_equal(_np(pl.plan[q]), r.plan.plan) and float(pl.objective[q]) == r.plan.objective
    # the round cost is felt: weights differ from the fixed-cost ones
    b0 = pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None, dense=dense)
    if extra == "zones":
        b0 = b0.with_zones(3)
    p0 = pk.upload(b0)
    if extra == "pool":
        p0.flags = pk.PARCAE_POOL_ALL
    W0 = pk.parcae_transition_weights(p0, ev.hist_int, ev.hist_min)
    _sync()
    w, w0 = _np(W[0]), _np(W0[0])
    fin = np.isfinite(w0)
    assert np.all(w[fin] <= w0[fin]) and np.any(w[fin] < w0[fin])


def test_transfer_round_costs_in_the_replay_and_bad_values(pk):
    import torch
    from oracle import replay as rp
    nq, H = 4, 6
    spec = pi.WorkloadSpec("replay", nq, 64, 16, 60.0, (2, 4, 8, 16, 32), 4, 6, 16, 0.12, False, 2, 300)
    b = pi.make_batch(spec, seed=77)
    b_plan = b.take(range(nq))
    b_plan.n_intervals = 8
    b_plan.avail = np.ascontiguousarray(b.avail[:, :9])
    b_plan = b_plan.with_rounds(4.0, 12.0)
    true, win = _replay_inputs(b, H, 9)
    win = np.ascontiguousarray(win[:, :, :9])
    p = pk.upload(b_plan)
    t_true, t_win = torch.from_numpy(true).cuda(), torch.from_numpy(win).cuda()
    for mode in (pk.PARCAE_REPLAY_PROACTIVE, pk.PARCAE_REPLAY_REACTIVE):
        chosen, reward, total = pk.parcae_replay(p, t_true, t_win if mode == pk.PARCAE_REPLAY_PROACTIVE else None, mode)
        _sync()
        for q in range(nq):
            r = rp.replay(b_plan, q, true[q], win[:, q, :], mode, n_threads=8)
            assert np.array_equal(_np(chosen[q]), r.chosen) and np.array_equal(_np(reward[q]), r.reward), (mode, q)
            assert float(total[q]) == r.total
    # bad values are flagged per query
    bad = pi.workload("sweep", n_scenarios=64, n_queries=4).with_rounds()
    bad.cost_round[1, 3] = -1.0
    bad.cost_round[2, 0] = np.inf
    _, pl = pk.parcae_liveput_plan(pk.upload(bad))
    _sync()
    assert list(_np(pl.status)) == [0, pk.PARCAE_EINVAL, pk.PARCAE_EINVAL, 0]


# ------------------------------------------------------------------ a hazard weight per instance

def test_weighted_scenarios_one_by_one(pk):
    """Successive weighted sampling instance by instance: every mask width, counts past the half (no complement
    here), idle instances, multi-GPU instances, extreme weights."""
    rng = pi.SplitMix64(777)
    cases = [  # D, P, group, a_prev (-1: used pool), a_next, largest weight
        (2, 3, 1, -1, 4, 9), (3, 4, 1, -1, 7, 255), (8, 4, 1, -1, 20, 3), (4, 8, 1, -1, 6, 16), (16, 4, 1, -1, 33, 255),
        (8, 8, 1, -1, 60, 2), (2, 32, 1, -1, 31, 40), (16, 8, 1, -1, 100, 7), (4, 32, 1, -1, 20, 255),
        (32, 8, 1, -1, 128, 5), (2, 128, 1, -1, 250, 100), (1, 256, 1, -1, 3, 255), (5, 7, 1, -1, 18, 12),
        (11, 23, 1, -1, 140, 30), (3, 65, 1, -1, 111, 8), (64, 1, 1, 80, 41, 6), (3, 4, 1, 20, 13, 255),
        (8, 16, 1, 200, 120, 9), (16, 4, 4, -1, 9, 20), (8, 4, 2, 30, 22, 200), (6, 2, 1, -1, 12, 4),
        (6, 2, 1, -1, 0, 4), (7, 9, 1, -1, 62, 1), (1, 1, 1, -1, 0, 77),
    ]
    for D, P, g, a_prev, a_next, wmax in cases:
        cfg = np.asarray([[D, P]], np.int32)
        b = pi.custom_batch(256, cfg, [[max(a_prev, 0), a_next]], thr_per_pipeline=[1.0], n_scenarios=64, seed=23,
                            group_size=g)
        b.inst_weight = np.asarray([[rng.randint(1, wmax) for _ in range(256)]], np.uint8)
        b.stream_id[:] = 4
        p = pk.upload(b)
        if a_prev >= 0:
            p.flags = pk.PARCAE_POOL_ALL
        ns, s0 = 200, 17
        masks, n_int, d_min = pk.parcae_debug_sample(p, 0, 0, 0, s0, ns)
        _sync()
        om, oi, od = oracle.debug_sample(D, P, a_next, int(b.seed[0]), 4, 0, s0, ns, a_prev=a_prev, group=g,
                                         zone=b.inst_weight[0], weight="instances")
        assert np.array_equal(_np(masks, np.uint32), om), (D, P, g, a_prev, a_next)
        assert np.array_equal(_np(n_int), oi) and np.array_equal(_np(d_min), od), (D, P, g, a_prev, a_next)


def _check_all_outputs(pk, b, q, ev, pl, W, S, pool_all=False):
    r = oracle.run_query(b, q, n_scenarios=S, n_threads=8, pool_all=pool_all)
    assert np.array_equal(_np(ev.hist_int[q], np.uint32), r.hist_int), "hist_int"
    assert np.array_equal(_np(ev.hist_min[q], np.uint32), r.hist_min), "hist_min"
    if r.hist_occ is not None:
        assert np.array_equal(_np(ev.hist_occ[q], np.uint32), r.hist_occ), "hist_occ"
    assert np.array_equal(_np(ev.liveput[q]), r.tables.liveput_f) and np.array_equal(_np(ev.gain[q]), r.tables.gain_f)
    assert np.array_equal(_np(ev.teff[q]), r.tables.teff_f)
    assert np.all(np.abs(_np(ev.gain[q]) - r.tables.gain_d) <= REL * np.abs(r.tables.gain_d))
    assert np.array_equal(_np(W[q]), r.W_f), "W"
    fin = np.isfinite(r.W_d)
    assert np.all(np.abs(_np(W[q])[fin] - r.W_d[fin]) <= REL * np.abs(r.W_d[fin]))
    assert np.array_equal(_np(pl.bp[q]), r.plan.bp) and np.array_equal(_np(pl.F[q]), r.plan.F)
    assert np.array_equal(_np(pl.plan[q]), r.plan.plan) and float(pl.objective[q]) == r.plan.objective
    assert int(pl.status[q]) == (pk.PARCAE_OK if r.plan.feasible else pk.PARCAE_EINFEASIBLE)
    return r


@pytest.mark.parametrize("name,S,nq,pool_all", [("tiny", 256, 1, False), ("small", 1000, 1, False),
                                                ("medium", 700, 1, True), ("large", 200, 1, False),
                                                ("sweep", 500, 40, False), ("sweep", 300, 36, True)])
def test_weighted_full_parity(pk, name, S, nq, pool_all):
    b = pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None).with_weights(max_weight=255 if nq == 36 else 8)
    p = pk.upload(b)
    if pool_all:
        p.flags = pk.PARCAE_POOL_ALL
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    for q in sorted({0, nq // 2, nq - 1}):
        _check_all_outputs(pk, b, q, ev, pl, W, S, pool_all)
    # the weights matter: the same batch drawn uniformly gives other histograms
    u = pk.upload(pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None))
    if pool_all:
        u.flags = pk.PARCAE_POOL_ALL
    ev_u = pk.parcae_liveput_eval(u)
    _sync()
    assert not np.array_equal(_np(ev_u.hist_min), _np(ev.hist_min))


def test_weighted_replay_and_bad_weights(pk):
    import torch
    from oracle import replay as rp
    nq, H = 3, 4
    spec = pi.WorkloadSpec("replay", nq, 48, 12, 60.0, (2, 4, 8, 16), 2, 5, 12, 0.1, False, 2, 200)
    b = pi.make_batch(spec, seed=91)
    b_plan = b.take(range(nq))
    b_plan.n_intervals = 6
    b_plan.avail = np.ascontiguousarray(b.avail[:, :7])
    b_plan = b_plan.with_weights(max_weight=20)
    true, win = _replay_inputs(b, H, 2)
    win = np.ascontiguousarray(win[:, :, :7])
    p = pk.upload(b_plan)
    for mode in (pk.PARCAE_REPLAY_PROACTIVE, pk.PARCAE_REPLAY_REACTIVE):
        chosen, reward, total = pk.parcae_replay(p, torch.from_numpy(true).cuda(),
                                                 torch.from_numpy(win).cuda() if mode == pk.PARCAE_REPLAY_PROACTIVE else None, mode)
        _sync()
        for q in range(nq):
            r = rp.replay(b_plan, q, true[q], win[:, q, :], mode, n_threads=8)
            assert np.array_equal(_np(chosen[q]), r.chosen) and np.array_equal(_np(reward[q]), r.reward), (mode, q)
    bad = pi.workload("sweep", n_scenarios=64, n_queries=4).with_weights()
    bad.inst_weight[2, 40] = 0
    _, pl = pk.parcae_liveput_plan(pk.upload(bad))
    _sync()
    assert list(_np(pl.status)) == [0, 0, pk.PARCAE_EINVAL, 0]


# ------------------------------------------------------------------ cost per instance that must receive state

@pytest.mark.parametrize("name,S,nq,dense,extra", [("tiny", 256, 1, False, ""), ("small", 1000, 1, False, ""),
                                                    ("medium", 600, 1, True, ""), ("large", 200, 1, False, "pool"),
                                                    ("sweep", 500, 40, False, ""), ("sweep", 300, 33, False, "zones"),
                                                    ("sweep", 300, 34, False, "weights"), ("small", 2500, 1, False, "pool")])
def test_cost_per_moved_instance_full_parity(pk, name, S, nq, dense, extra):
    """The third statistic (stage occupancies) from every sampling kernel variant, tables and weights with the move
    cost, plans through the weights in memory for few and for many queries."""
    b = pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None, dense=dense).with_moves()
    if extra == "zones":
        b = b.with_zones(3)
    if extra == "weights":
        b = b.with_weights()
    b.cost_move[:, ::5] = 0.0                  # some candidates keep the fixed inter-stage cost
    p = pk.upload(b)
    if extra == "pool":
        p.flags = pk.PARCAE_POOL_ALL
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    pl2 = pk.parcae_plan_from_hist(p, ev.hist_int, ev.hist_min)
    _sync()
    for q in sorted({0, nq // 2, nq - 1}):
        r = _check_all_outputs(pk, b, q, ev, pl, W, S, extra == "pool")
        assert r.hist_occ.sum() > 0
    for f in ("F", "bp", "plan", "start", "objective", "status"):
        assert np.array_equal(_np(getattr(pl2, f)), _np(getattr(pl, f))), f
    # the move cost is felt
    b0 = pi.workload(name, n_scenarios=S, n_queries=nq if nq > 1 else None, dense=dense)
    if extra == "zones":
        b0 = b0.with_zones(3)
    if extra == "weights":
        b0 = b0.with_weights()
    p0 = pk.upload(b0)
    if extra == "pool":
        p0.flags = pk.PARCAE_POOL_ALL
    W0 = pk.parcae_transition_weights(p0, ev.hist_int, ev.hist_min)
    _sync()
    w, w0 = _np(W[0]), _np(W0[0])
    fin = np.isfinite(w0)
    assert np.all(w[fin] <= w0[fin]) and np.any(w[fin] < w0[fin])


def test_cost_per_moved_instance_multi_gpu_instances_and_bad_values(pk):
    spec = pi.WorkloadSpec("quad", 3, 64, 6, 60.0, (2, 4, 8, 16), 2, 6, 16, 0.1, False, 2, 400)
    walk = pi.make_batch(spec, seed=21)
    cfg = pi.candidate_list(256, (2, 4, 8, 16), 2)
    cfg = cfg[(cfg[:, 0] % 4 == 0) & (cfg[:, 0] * cfg[:, 1] <= 256) & (cfg[:, 0] <= 64)]
    g = pi.custom_batch(64, cfg, walk.avail, thr_per_pipeline=[1.0 + 0.05 * p for _, p in cfg], n_scenarios=400, p_min=2,
                        group_size=4, seed=8).with_moves()
    p = pk.upload(g)
    ev, pl = pk.parcae_liveput_plan(p)
    W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
    _sync()
    for q in range(3):
        _check_all_outputs(pk, g, q, ev, pl, W, 400)
    bad = pi.workload("sweep", n_scenarios=64, n_queries=5).with_moves()
    bad.cost_move[1, 3] = -1.0
    bad.cost_move[2, 0] = np.inf
    c = int(np.argmax((bad.configs[:, 0] - 1) * bad.configs[:, 1]))
    bad.cost_move[3, c] = 100.0            # the dearest inter-stage migration would outlast the interval
    _, pl = pk.parcae_liveput_plan(pk.upload(bad))
    _sync()
    assert list(_np(pl.status)) == [0, pk.PARCAE_EINVAL, pk.PARCAE_EINVAL, pk.PARCAE_EINVAL, 0]


# ------------------------------------------------------------------ randomly drawn problems

def _random_problem(rng, with_moves=True):
    """A small problem with every option drawn at random: sizes, depth list, pool, instance size, zones, round
    costs, start state, scenario count (mostly not a power of two), queries on either side of the planner switch."""
    group = [1, 1, 1, 2, 4][rng.randint(0, 4)]
    n_inst = rng.randint(1, 256 if rng.randint(0, 3) == 0 else 48)
    depth_pool = [1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 13, 16, 23, 31, 32, 33, 48, 64, 65, 100, 128, 200, 256]
    depths = sorted({depth_pool[rng.randint(0, len(depth_pool) - 1)] for _ in range(rng.randint(1, 5))})
    depths = [p for p in depths if p <= n_inst] or [1]
    p_min = depths[rng.randint(0, len(depths) - 1)] if rng.randint(0, 2) == 0 else 1
    cfg = pi.candidate_list(n_inst, depths, p_min, feasible_only=rng.randint(0, 1) == 1)
    if len(cfg) == 0:
        cfg = pi.candidate_list(n_inst, depths, 1)
    if len(cfg) > 120:                                   # keep the oracle quick: a random subset, order preserved
        keep = sorted({rng.randint(0, len(cfg) - 1) for _ in range(120)})
        cfg = cfg[keep]
    cfg = cfg.copy()
    cfg[:, 0] *= group                                    # D counts GPUs: multiples of the instance size
    cfg = cfg[cfg[:, 0] <= 256]
    nq = [1, 2, 33][rng.randint(0, 2)]
    T = rng.randint(1, 5)
    S = [1, 63, 64, 65, 200, 256, 300][rng.randint(0, 6)]
    avail = [[rng.randint(0, n_inst) for _ in range(T + 1)] for _ in range(nq)]
    thr = [rng.uniform(0.5, 3.0) for _ in range(len(cfg))]
    cost = [[rng.uniform(0.0, 3.0), rng.uniform(3.0, 20.0), rng.uniform(20.0, 70.0)] for _ in range(len(cfg))]
    b = pi.custom_batch(n_inst, cfg, avail, thr_per_pipeline=thr, cost=cost, interval_sec=[30.0, 60.0][rng.randint(0, 1)],
                        p_min=p_min, n_scenarios=S, seed=rng.randint(1, 1 << 30), group_size=group)
    for q in range(nq):
        b.cur_config[q] = [-2, -1, rng.randint(0, len(cfg) - 1)][rng.randint(0, 2)]
        b.stream_id[q] = rng.randint(0, 1000)
    draw = rng.randint(0, 3)
    if draw == 0:
        b = b.with_zones(rng.randint(1, 4), seed=rng.randint(1, 999), max_weight=[3, 255][rng.randint(0, 1)])
    elif draw == 1:
        b = b.with_weights(seed=rng.randint(1, 999), max_weight=[2, 16][rng.randint(0, 1)])
    refine = rng.randint(0, 3)
    if refine == 0:
        b = b.with_rounds(0.0, 25.0, seed=rng.randint(1, 999))
    elif refine == 1 and with_moves:
        b = b.with_moves(seed=rng.randint(1, 999))
    return b, rng.randint(0, 1) == 1


def test_random_problems_match_the_oracle(pk):
    rng = pi.SplitMix64(0xF00D)
    for case in range(40):
        b, pool_all = _random_problem(rng)
        p = pk.upload(b)
        if pool_all:
            p.flags = pk.PARCAE_POOL_ALL
        ev, pl = pk.parcae_liveput_plan(p)
        W = pk.parcae_transition_weights(p, ev.hist_int, ev.hist_min)
        _sync()
        tag = (case, b.n_instances, b.n_configs, b.n_queries, b.n_intervals, b.n_scenarios, b.group_size, b.n_zones,
               b.cost_round is not None, b.inst_weight is not None, b.cost_move is not None, pool_all)
        for q in range(b.n_queries):
            r = oracle.run_query(b, q, n_threads=8, pool_all=pool_all)
            assert np.array_equal(_np(ev.hist_int[q], np.uint32), r.hist_int), tag
            assert np.array_equal(_np(ev.hist_min[q], np.uint32), r.hist_min), tag
            if r.hist_occ is not None:
                assert np.array_equal(_np(ev.hist_occ[q], np.uint32), r.hist_occ), tag
            assert np.array_equal(_np(ev.liveput[q]), r.tables.liveput_f), tag
            assert np.array_equal(_np(ev.teff[q]), r.tables.teff_f) and np.array_equal(_np(ev.gain[q]), r.tables.gain_f), tag
            assert np.array_equal(_np(W[q]), r.W_f), tag
            assert np.array_equal(_np(pl.bp[q]), r.plan.bp) and np.array_equal(_np(pl.F[q]), r.plan.F), tag
            assert np.array_equal(_np(pl.plan[q]), r.plan.plan) and int(pl.start[q]) == r.plan.start, tag
            assert float(pl.objective[q]) == r.plan.objective, tag
            assert int(pl.status[q]) == (pk.PARCAE_OK if r.plan.feasible else pk.PARCAE_EINFEASIBLE), tag


# ------------------------------------------------------------------ receding-horizon replay

def _replay_inputs(b, H, noise_seed):
    """True walks = the batch's own walks; forecasts = the truth plus a small seeded error, clipped."""
    T = b.n_intervals
    rng = np.random.default_rng(noise_seed)
    true = np.ascontiguousarray(b.avail[:, : H + 1])
    nq = b.n_queries
    win = np.zeros((H, nq, T + 1), np.int32)
    for i in range(H):
        for q in range(nq):
            fut = [b.avail[q, min(i + 1 + t, b.avail.shape[1] - 1)] for t in range(T)]
            err = rng.integers(-3, 4, size=T)
            win[i, q, 0] = true[q, i]
            win[i, q, 1:] = np.clip(np.asarray(fut) + err, 0, b.n_instances)
    return true, win


@pytest.mark.parametrize("nq,pool_all,zones", [(3, False, 0), (40, False, 0), (5, True, 0), (4, False, 3)])
def test_replay_matches_the_oracle_replay(pk, nq, pool_all, zones):
    import torch
    from oracle import replay as rp
    spec = pi.WorkloadSpec("replay", nq, 64, 18, 60.0, (2, 4, 8, 16, 32), 4, 6, 16, 0.12, False, 2, 300)
    b = pi.make_batch(spec, seed=404)
    H = 7
    b_plan = b.take(range(nq))
    b_plan.n_intervals = 10                                   # look-ahead of the planner inside the replay
    b_plan.avail = np.ascontiguousarray(b.avail[:, :11])
    b_plan.cur_config[1 % nq] = -1                            # one query starts with nothing running
    if zones:
        b_plan = b_plan.with_zones(zones)
    true, win = _replay_inputs(b, H, 5)
    win = np.ascontiguousarray(win[:, :, :11])
    p = pk.upload(b_plan)
    if pool_all:
        p.flags = pk.PARCAE_POOL_ALL
    t_true = torch.from_numpy(true).cuda()
    t_win = torch.from_numpy(win).cuda()
    for mode in (pk.PARCAE_REPLAY_PROACTIVE, pk.PARCAE_REPLAY_REACTIVE):
        chosen, reward, total = pk.parcae_replay(p, t_true, t_win if mode == pk.PARCAE_REPLAY_PROACTIVE else None, mode)
        _sync()
        for q in sorted({0, 1 % nq, nq - 1}):
            r = rp.replay(b_plan, q, true[q], win[:, q, :], mode, n_threads=8, pool_all=pool_all)
            assert np.array_equal(_np(chosen[q]), r.chosen), (mode, q)
            assert np.array_equal(_np(reward[q]), r.reward), (mode, q)
            assert float(total[q]) == r.total
            assert abs(float(total[q]) - r.total_d) <= REL * abs(r.total_d)


def test_replay_on_randomly_drawn_problems(pk):
    """Replay of both kinds on problems with every option drawn at random, walks and forecasts random too."""
    import torch
    from oracle import replay as rp
    rng = pi.SplitMix64(0xBEEF)
    for case in range(16):
        b, pool_all = _random_problem(rng, with_moves=False)       # the replay takes no cost per moved instance
        nq, T, N = b.n_queries, b.n_intervals, b.n_instances
        H = rng.randint(1, 5)
        true = np.asarray([[rng.randint(0, N) for _ in range(H + 1)] for _ in range(nq)], np.int32)
        win = np.zeros((H, nq, T + 1), np.int32)
        for i in range(H):
            for q in range(nq):
                win[i, q, 0] = true[q, i]
                for t in range(T):
                    win[i, q, 1 + t] = min(N, max(0, int(true[q, min(i + 1 + t, H)]) + rng.randint(-2, 2)))
        p = pk.upload(b)
        if pool_all:
            p.flags = pk.PARCAE_POOL_ALL
        t_true, t_win = torch.from_numpy(true).cuda(), torch.from_numpy(win).cuda()
        for mode in (pk.PARCAE_REPLAY_PROACTIVE, pk.PARCAE_REPLAY_REACTIVE):
            chosen, reward, total = pk.parcae_replay(p, t_true, t_win if mode == pk.PARCAE_REPLAY_PROACTIVE else None, mode)
            _sync()
            for q in sorted({0, nq - 1}):
                r = rp.replay(b, q, true[q], win[:, q, :], mode, n_threads=8, pool_all=pool_all)
                assert np.array_equal(_np(chosen[q]), r.chosen), (case, mode, q)
                assert np.array_equal(_np(reward[q]), r.reward) and float(total[q]) == r.total, (case, mode, q)


def test_replay_flags_bad_walks_windows_and_start_configurations(pk):
    """Bad DEVICE data in the replay inputs is reported per query and never used as an index: a starting
    configuration past the candidate list, a true-walk entry above N, a window entry below 0 in a late step."""
    import torch
    from oracle import replay as rp
    nq, H = 5, 4
    spec = pi.WorkloadSpec("replay", nq, 32, 12, 60.0, (2, 4, 8), 2, 4, 8, 0.1, False, 2, 128)
    b = pi.make_batch(spec, seed=31)
    b_plan = b.take(range(nq))
    b_plan.n_intervals = 6
    b_plan.avail = np.ascontiguousarray(b.avail[:, :7])
    true, win = _replay_inputs(b, H, 3)
    win = np.ascontiguousarray(win[:, :, :7])
    good_true, good_win = true.copy(), win.copy()
    b_plan.cur_config[1] = b_plan.n_configs + 5            # past the list
    true[2, 3] = 33                                         # above N
    win[3, 3, 5] = -1                                       # below 0, last step's window
    p = pk.upload(b_plan)
    for mode in (pk.PARCAE_REPLAY_PROACTIVE, pk.PARCAE_REPLAY_REACTIVE):
        chosen, reward, total, status = pk.parcae_replay(
            p, torch.from_numpy(true).cuda(), torch.from_numpy(win).cuda() if mode == pk.PARCAE_REPLAY_PROACTIVE else None,
            mode, with_status=True)
        _sync()
        want = [0, pk.PARCAE_EINVAL, pk.PARCAE_EINVAL, pk.PARCAE_EINVAL if mode == pk.PARCAE_REPLAY_PROACTIVE else 0, 0]
        assert _np(status).tolist() == want, mode
        for q in (0, 4):                                   # the clean queries are unaffected
            r = rp.replay(b_plan, q, good_true[q], good_win[:, q, :], mode, n_threads=4)
            assert np.array_equal(_np(chosen[q]), r.chosen) and np.array_equal(_np(reward[q]), r.reward), (mode, q)
        assert np.all(_np(chosen) >= -1) and np.all(_np(chosen) < b_plan.n_configs)


def test_replay_suspends_and_restarts(pk):
    """Availability falls below the memory floor and comes back: nothing runs, then a cold start."""
    import torch
    from oracle import replay as rp
    cfg = pi.candidate_list(8, (2, 4), 2)
    b = pi.custom_batch(8, cfg, [[8, 8, 8]], thr_per_pipeline=[1.0 + p for _, p in cfg], n_scenarios=128, p_min=2,
                        cur_config=len(cfg) - 1)
    true = np.asarray([[8, 3, 1, 6, 7]], np.int32)
    win = np.asarray([[[8, 8, 8]], [[3, 8, 8]], [[1, 8, 8]], [[6, 6, 6]]], np.int32)
    p = pk.upload(b)
    chosen, reward, total = pk.parcae_replay(p, torch.from_numpy(true).cuda(), torch.from_numpy(win).cuda())
    _sync()
    r = rp.replay(b, 0, true[0], win[:, 0, :], rp.PROACTIVE)
    assert r.chosen[1] == -1 and r.chosen[2] >= 0
    assert np.array_equal(_np(chosen[0]), r.chosen) and np.array_equal(_np(reward[0]), r.reward)
    assert float(total[0]) == r.total


# ------------------------------------------------------------------ edge cases

def test_degenerate_shapes(pk):
    # one instance, one candidate, one interval, one scenario
    b = pi.custom_batch(1, [[1, 1]], [[1, 0]], thr_per_pipeline=[3.0], n_scenarios=1, cur_config=0)
    ev, pl = pk.parcae_liveput_plan(pk.upload(b))
    _sync()
    _check_query_against_oracle(pk, b, 0, ev, pl, 1)
    # the largest pool: 256 instances in every shape, half of them preempted
    cfg = pi.candidate_list(256, (1, 2, 4, 8, 16, 32, 64, 128, 256), 1)
    cfg = cfg[cfg[:, 0] * cfg[:, 1] == 256]
    b = pi.custom_batch(256, cfg, [[256, 128, 255, 1, 0, 256]], thr_per_pipeline=[1.0] * len(cfg), n_scenarios=300)
    ev, pl = pk.parcae_liveput_plan(pk.upload(b))
    _sync()
    _check_query_against_oracle(pk, b, 0, ev, pl, 300)


def test_largest_scenario_count(pk):
    """S = 2^24, the largest count the float tables take exactly: one sampled unit, 16384 work items that meet
    in the same bins, counts and tables against the oracle."""
    S = pk.PARCAE_MAX_SCENARIOS
    b = pi.custom_batch(8, [[2, 4]], [[8, 5]], thr_per_pipeline=[7.0], cost=[[2.0, 10.0, 40.0]], n_scenarios=S, seed=12)
    ev, pl = pk.parcae_liveput_plan(pk.upload(b))
    _sync()
    hi, hm = _np(ev.hist_int[0], np.uint32), _np(ev.hist_min[0], np.uint32)
    assert hi.sum() == S and hm.sum() == S
    r = oracle.run_query(b, 0, n_threads=8)
    assert np.array_equal(hi, r.hist_int) and np.array_equal(hm, r.hist_min)
    assert np.array_equal(_np(ev.liveput[0]), r.tables.liveput_f) and np.array_equal(_np(ev.teff[0]), r.tables.teff_f)
    assert np.array_equal(_np(pl.plan[0]), r.plan.plan) and float(pl.objective[0]) == r.plan.objective
    # one more scenario is refused on the host
    p = pk.upload(b)
    p.n_scenarios = S + 1
    with pytest.raises(pk.ParcaeError):
        pk.parcae_liveput_plan(p)


def test_depths_that_are_not_powers_of_two(pk):
    cfg = pi.candidate_list(60, (3, 5, 7, 12, 13, 23), 3)
    b = pi.custom_batch(60, cfg, [[60, 41, 52, 33, 60, 20]], thr_per_pipeline=[float(p) ** 0.5 for _, p in cfg],
                        n_scenarios=500, p_min=3, seed=9)
    ev, pl = pk.parcae_liveput_plan(pk.upload(b))
    _sync()
    _check_query_against_oracle(pk, b, 0, ev, pl, 500)


def test_infeasible_and_invalid_queries_are_flagged_per_query(pk):
    cfg = pi.candidate_list(8, (2, 4), 2)
    av = [[8, 6, 7, 5], [8, 1, 7, 5], [8, 6, 7, 5], [8, 6, 9, 5]]   # q1: below the memory floor; q3: above N
    b = pi.custom_batch(8, cfg, av, thr_per_pipeline=[1.0] * len(cfg), n_scenarios=200, p_min=2)
    b.thr[2, 0] = 1.0                                                 # q2: thr[.][0] != 0
    p = pk.upload(b)
    ev, pl = pk.parcae_liveput_plan(p)
    _sync()
    st = _np(pl.status)
    assert st.tolist() == [pk.PARCAE_OK, pk.PARCAE_EINFEASIBLE, pk.PARCAE_EINVAL, pk.PARCAE_EINVAL]
    _check_query_against_oracle(pk, b, 0, ev, pl, 200)
    _check_query_against_oracle(pk, b, 1, ev, pl, 200)
    assert np.all(_np(pl.plan[1]) == -1) and float(pl.objective[1]) == -np.inf and int(pl.start[1]) == -1
    ev2 = pk.parcae_liveput_eval(p)
    _sync()
    assert _np(ev2.status).tolist() == [0, 0, pk.PARCAE_EINVAL, pk.PARCAE_EINVAL]


def test_optional_outputs_may_be_null(pk):
    b = pi.workload("tiny")
    p = pk.upload(b)
    ev = pk.alloc_eval_out(p, tables=False)
    ev.status = None
    pl = pk.alloc_plan_out(p, full=False)
    pl.start = None
    pl.objective = None
    pl.status = None
    pk.parcae_liveput_plan(p, ev, pl)
    _sync()
    r = oracle.run_query(b, 0)
    assert np.array_equal(_np(ev.hist_int[0], np.uint32), r.hist_int)
    assert np.array_equal(_np(pl.plan[0]), r.plan.plan)


def test_runs_on_a_side_stream_and_repeats_identically(pk):
    import torch
    b = pi.workload("small")
    p = pk.upload(b)
    ev0, pl0 = pk.parcae_liveput_plan(p)
    _sync()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ev1, pl1 = pk.parcae_liveput_plan(p)
    side.synchronize()
    for f in ("hist_int", "hist_min", "liveput", "teff", "gain"):
        assert np.array_equal(_np(getattr(ev0, f)), _np(getattr(ev1, f)))
    for f in ("F", "bp", "plan", "start", "objective"):
        assert np.array_equal(_np(getattr(pl0, f)), _np(getattr(pl1, f)))


def test_whole_call_can_be_captured_in_a_hip_graph_and_replayed(pk):
    """The calls enqueue kernels only (no memset or memcpy nodes), so a captured graph replays correctly; every
    replay is checked against the eager result, with eager work and synchronisations between replays."""
    import torch
    b = pi.workload("small", n_scenarios=2000)
    p = pk.upload(b)
    ev0, pl0 = pk.parcae_liveput_plan(p)
    _sync()
    ev, pl = pk.alloc_eval_out(p), pk.alloc_plan_out(p)
    p.workspace()                                   # allocate before capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pk.parcae_liveput_plan(p, ev, pl)           # warm-up on the capture stream
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pk.parcae_liveput_plan(p, ev, pl)
    for rep in range(4):
        for t in (ev.hist_int, ev.hist_min, ev.liveput, pl.F, pl.bp, pl.plan, pl.objective):
            t.fill_(-1 if t.dtype != torch.float32 else float("nan"))
        _sync()
        graph.replay()
        _sync()
        for f in ("hist_int", "hist_min", "liveput", "teff", "gain"):
            assert np.array_equal(_np(getattr(ev, f)), _np(getattr(ev0, f))), (rep, f)
        for f in ("F", "bp", "plan", "start", "objective", "status"):
            assert np.array_equal(_np(getattr(pl, f)), _np(getattr(pl0, f))), (rep, f)
        ev1 = pk.parcae_liveput_eval(p)             # eager work between the replays
        _sync()
        assert np.array_equal(_np(ev1.hist_int), _np(ev0.hist_int))
