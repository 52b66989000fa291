"""Extreme shapes through every oracle entry point: the largest pool, the largest multi-GPU grid, a single scenario,
a single interval, a single candidate.  Plain invariants only; the point of the module is to walk the buffers to
their ends (it also runs under AddressSanitizer and UndefinedBehaviorSanitizer, see test_sanitizers.py)."""
import numpy as np
import pytest

import oracle
import parcae_inputs as pi


@pytest.mark.parametrize("D,P,k", [(1, 256, 255), (256, 1, 128), (16, 16, 1), (4, 64, 256), (2, 128, 0), (255, 1, 254)])
def test_largest_pool(D, P, k):
    M = D * P
    v = oracle.sample_preempted(M, k, 0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF)
    assert v.shape == (M,) and v.sum() == k
    n_int, d_min, occ = oracle.reduce(D, P, v)
    assert 0 <= n_int <= d_min <= D and occ.sum() == M - k
    masks, ni, dm = oracle.debug_sample(D, P, M - k, 1, 2, 3, 0xFFFFFFF0, 16)
    assert np.all(ni <= dm) and np.all(dm <= D)


@pytest.mark.parametrize("D,P,g,a_next", [(256, 64, 64, 100), (64, 256, 64, 255), (256, 4, 4, 3), (128, 2, 64, 1)])
def test_largest_grid_of_multi_gpu_instances(D, P, g, a_next):
    """D x P counts GPUs (up to 256 pipelines of 64 stages on 64-GPU instances: 16384 GPUs), the pool counts
    instances (at most 256)."""
    M = D * P // g
    assert M <= 256
    hi, hm = oracle.eval_unit(D, P, a_next, 7, 0, 0, 0, 64, group=g)
    assert hi.sum() == 64 and hm.sum() == 64 and hi.shape == (D + 1,)
    nz = np.nonzero(hi)[0]
    assert np.all(nz % g == 0)
    inst = oracle.sample_preempted(M, max(0, M - a_next), 7, 0, 0, 0)
    assert inst.sum() == max(0, M - a_next)


def test_whole_cluster_pool_and_zones_at_the_size_limit():
    zone = (np.arange(256) % 4).astype(np.uint8)
    for k_left in (0, 1, 128, 255, 256):
        v = oracle.sample_preempted_zoned(256, 256 - k_left, zone, [1, 255, 3, 200], 5, 6, 7, 8)
        assert v.sum() == 256 - k_left
    hi, hm = oracle.eval_unit(3, 32, 1, 9, 0, 5, 0, 32, a_prev=256)          # 96 GPUs used, 160 idle, one survivor
    assert hi.sum() == 32 and hi[0] == 32
    hi, hm = oracle.eval_unit(8, 32, 130, 9, 0, 5, 0, 32, a_prev=256, zone=zone, weight=[9, 1, 1, 1])
    assert hi.sum() == 32 and hm.sum() == 32


@pytest.mark.parametrize("S,T", [(1, 1), (1, 3), (3, 1)])
def test_one_scenario_one_interval_one_candidate(S, T):
    for cfg in ([[1, 1]], [[256, 1]], [[1, 256]], [[2, 3], [3, 3], [1, 7]]):
        N = max(d * p for d, p in cfg)
        avail = [[N] + [max(0, N - 1 - t) for t in range(T)]]
        b = pi.custom_batch(N, cfg, avail, thr_per_pipeline=[1.5] * len(cfg), n_scenarios=S, cur_config=0)
        r = oracle.run_query(b, 0)
        assert r.hist_int.sum() == S * T * len(cfg) and r.plan.F.shape == (T + 1, len(cfg))
        assert np.all(r.tables.liveput_f[0] <= r.tables.liveput_f[2] + 1e-6)
        b2 = b.with_rounds(0.0, 30.0)
        r2 = oracle.run_query(b2, 0, pool_all=True)
        assert r2.hist_min.sum() == S * T * len(cfg)


def test_long_candidate_list_through_tables_weights_and_plan():
    cfg = pi.candidate_list(256, (1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233, 256), 1)
    b = pi.custom_batch(256, cfg, [[256, 200, 17, 256, 0, 255]], thr_per_pipeline=[1.0 + 0.01 * p for _, p in cfg],
                        n_scenarios=3, p_min=2, cur_config=-2)
    r = oracle.run_query(b, 0, n_threads=4)
    C = len(cfg)
    assert r.W_f.shape == (5, C, C) and r.plan.bp.shape == (5, C)
    assert not r.plan.feasible          # an interval with no instance at all: nothing can run through it
