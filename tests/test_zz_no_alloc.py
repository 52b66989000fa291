"""The entry point that allocates nothing (workspace inside the library) against parcae_liveput_plan,
through the C ABI, on the GPU: two calls in a row, the second on a smaller problem, every output bit for bit."""
import numpy as np
import pytest

import parcae_inputs as pi

pytestmark = pytest.mark.gpu

EVAL_FIELDS = ("hist_int", "hist_min", "liveput", "teff", "gain")
PLAN_FIELDS = ("F", "bp", "plan", "start", "objective", "status")


@pytest.fixture(scope="module")
def pk():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2403_14097_amd as mod
    mod.load_library()
    return mod


def _np(t):
    return t.detach().cpu().numpy()


def _poison(*outs):
    import torch
    for out in outs:
        for t in vars(out).values():
            if t is not None:
                t.fill_(float("nan") if t.dtype == torch.float32 else -7)


def test_static_entry_matches_the_workspace_entry_on_two_calls_in_a_row(pk):
    import torch
    cases = [
        pi.workload("sweep", n_queries=48, n_scenarios=1500),   # per-query planner, sampled units split into items
        pi.workload("small", n_scenarios=700),                  # smaller: one query, weights through the workspace
    ]
    assert cases[1].n_queries * cases[1].n_intervals * cases[1].hist_len < cases[0].n_queries * cases[0].n_intervals * cases[0].hist_len
    for b in cases:
        p = pk.upload(b)
        assert pk.parcae_workspace_bytes(p) <= pk.PARCAE_STATIC_WORKSPACE_BYTES
        ev0, pl0 = pk.parcae_liveput_plan(p)
        torch.cuda.synchronize()
        ev1, pl1 = pk.alloc_eval_out(p), pk.alloc_plan_out(p)
        _poison(ev1, pl1)
        torch.cuda.synchronize()
        pk.parcae_liveput_plan_static(p, ev1, pl1)
        torch.cuda.synchronize()
        for f in EVAL_FIELDS:
            assert np.array_equal(_np(getattr(ev1, f)), _np(getattr(ev0, f))), (b.name, f)     # NaN-free: plain equality
        for f in PLAN_FIELDS:
            assert np.array_equal(_np(getattr(pl1, f)), _np(getattr(pl0, f))), (b.name, f)
        assert np.all(_np(pl1.status) == 0) and np.all(_np(pl1.plan) >= 0)


def test_static_entry_refuses_what_its_array_cannot_hold(pk):
    b = pi.workload("large", dense=True, n_scenarios=64)         # 62 MB of transition weights: beyond the 16 MiB array
    p = pk.upload(b)
    assert pk.parcae_workspace_bytes(p) > pk.PARCAE_STATIC_WORKSPACE_BYTES
    ev, pl = pk.alloc_eval_out(p, tables=False), pk.alloc_plan_out(p, full=False)
    with pytest.raises(pk.ParcaeError) as err:
        pk.parcae_liveput_plan_static(p, ev, pl)
    assert err.value.code == pk.PARCAE_EWORKSPACE
