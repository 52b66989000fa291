"""Pins for multi-GPU instances (section 9.2, "Multi-GPU instances"): the GPUs of an instance go together."""
import itertools
import math

import numpy as np
import pytest

import oracle
import parcae_inputs as pi
from tests import pyref


def _expand(D, P, g, node_bits):
    """GPU-level preemption vector from an instance-level one, by repeating rows of the instance grid."""
    nodes = np.asarray(node_bits[: D * P // g], dtype=np.uint8).reshape(D // g, P)
    return np.repeat(nodes, g, axis=0).reshape(-1)


def test_group_layout():
    """Instance G holds stage G mod P of g neighbouring pipelines."""
    lib = oracle.lib()
    import ctypes as ct
    D, P, g = 4, 2, 2
    want = {0: [0, 2], 1: [1, 3], 2: [4, 6], 3: [5, 7]}
    for G, idx in want.items():
        node = np.zeros(4, np.uint8)
        node[G] = 1
        gpu = np.zeros(D * P, np.uint8)
        lib.orc_expand_groups(ct.c_int(D), ct.c_int(P), ct.c_int(g), node.ctypes.data_as(ct.POINTER(ct.c_uint8)),
                              gpu.ctypes.data_as(ct.POINTER(ct.c_uint8)))
        assert np.flatnonzero(gpu).tolist() == idx
        assert np.array_equal(gpu, _expand(D, P, g, node))


def test_one_four_gpu_instance_interrupts_four_pipelines():
    """The sentence of section 9.2: preempting one 4-GPU instance interrupts 4 pipelines."""
    D, P, g = 8, 3, 4                      # 24 GPUs on 6 instances
    hi, hm = oracle.eval_unit(D, P, 5, 123, 0, 0, 0, 500, group=g)     # 6 instances used, 5 left
    assert hi[D - 4] == 500 and hi.sum() == 500
    assert hm[D - 4] == 500                # the stage of that instance keeps 4 of its 8 replicas
    # single-GPU instances losing one GPU interrupt one pipeline
    hi1, _ = oracle.eval_unit(D, P, 23, 123, 0, 0, 0, 500)
    assert hi1[D - 1] == 500


@pytest.mark.parametrize("D,P,g,k", [(4, 3, 2, 2), (6, 2, 3, 2), (8, 2, 4, 1), (8, 4, 2, 5), (4, 5, 4, 3)])
def test_histograms_against_exact_enumeration_of_instance_subsets(D, P, g, k):
    nodes = D * P // g
    exact_i = np.zeros(D + 1)
    exact_m = np.zeros(D + 1)
    n_sub = 0
    for comb in itertools.combinations(range(nodes), k):
        v = np.zeros(nodes, np.uint8)
        v[list(comb)] = 1
        a, b = pyref.survivors(D, P, _expand(D, P, g, v))
        exact_i[a] += 1
        exact_m[b] += 1
        n_sub += 1
    assert n_sub == math.comb(nodes, k)
    S = 1 << 15
    hi, hm = oracle.eval_unit(D, P, nodes - k, 9, 0, 4, 0, S, group=g)
    for got, ex in ((hi, exact_i), (hm, exact_m)):
        p = ex / n_sub
        assert np.all(np.abs(got / S - p) <= 5 * np.sqrt(p * (1 - p) / S) + 1e-12)
        assert np.all(got[ex == 0] == 0)
        assert np.all(got[np.arange(D + 1) % g != 0] == 0)         # pipelines go and stay in blocks of g


def test_same_as_the_instance_grid_scaled_by_the_group_size():
    """A D x P grid of g-GPU instances behaves like a (D / g) x P grid of instances, counts times g."""
    # the last two grids hold more than 256 GPUs (1024 and 16384): D * P counts GPUs, only instances are capped
    for D, P, g, a_next, a_prev in [(8, 4, 2, 11, -1), (12, 2, 4, 4, -1), (8, 8, 2, 20, 40), (16, 4, 4, 9, 30),
                                    (128, 8, 4, 200, -1), (256, 64, 64, 100, 256)]:
        big = oracle.eval_unit(D, P, a_next, 31, 2, 17, 0, 2000, a_prev=a_prev, group=g)
        small = oracle.eval_unit(D // g, P, a_next, 31, 2, 17, 0, 2000, a_prev=a_prev)
        for b_, s_ in zip(big, small):
            assert np.array_equal(b_[::g], s_) and b_.sum() == 2000


def test_tables_and_plan_with_four_gpu_instances():
    cfg = pi.candidate_list(32, (2, 4, 8), 2)
    cfg = cfg[cfg[:, 0] % 4 == 0]                                     # widths in blocks of four pipelines
    av = [[8, 7, 8, 5, 6, 6, 3, 4]]                                   # instances of 4 GPUs each
    b = pi.custom_batch(8, cfg, av, thr_per_pipeline=[1.0 + 0.1 * p for _, p in cfg], n_scenarios=600,
                        p_min=2, group_size=4, seed=3)
    r = oracle.run_query(b, 0, n_threads=2)
    used = cfg[:, 0] * cfg[:, 1]
    for t in range(7):
        fin = np.isfinite(r.W_d[t])
        assert np.array_equal(fin.any(axis=0), used <= 4 * b.avail[0, t + 1])      # GPUs against instances x 4
        for c, (D, P) in enumerate(cfg):
            nodes = D * P // 4
            k = max(0, nodes - b.avail[0, t + 1])
            d_star = min(D, 4 * ((nodes - k) // P))
            assert r.tables.liveput_d[2, t, c] == b.thr[0, b.thr_off[c] + d_star]
    assert r.plan.feasible
    assert all(cfg[c, 0] * cfg[c, 1] <= 4 * b.avail[0, t + 1] for t, c in enumerate(r.plan.plan))
