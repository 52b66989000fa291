"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header declares,
and turns bad shapes into error codes before anything is launched."""
import ctypes as ct
import os
import re

import pytest

import paper_2403_14097_amd as pk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "parcae.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(parcae_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = pk.load_library()
    declared = _declared_symbols()
    assert set(declared) == set(pk.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_strerror():
    assert pk.parcae_version() >= 200
    assert pk.strerror(0) == "ok"
    for code in (pk.PARCAE_EINVAL, pk.PARCAE_EWORKSPACE, pk.PARCAE_EHIP, pk.PARCAE_EINFEASIBLE, -99):
        assert isinstance(pk.strerror(code), str) and pk.strerror(code)


def test_hist_len():
    assert pk.parcae_hist_len([(1, 2), (2, 2), (3, 2)]) == 9
    assert pk.parcae_hist_len([(256, 1)]) == 257
    assert pk.load_library().parcae_hist_len(None, 3) == pk.PARCAE_EINVAL


def _problem(configs, nq=1, N=8, T=4, S=16, tau=60.0, p_min=1, flags=0, fake_ptr=0x1000, group=0):
    arr = (pk.parcae_config * len(configs))()
    for i, (d, p) in enumerate(configs):
        arr[i].D, arr[i].P = d, p
    prob = pk.parcae_problem(ct.sizeof(pk.parcae_problem), nq, N, T, len(configs), S, p_min, tau, flags,
                             ct.cast(arr, ct.POINTER(pk.parcae_config)),
                             fake_ptr, fake_ptr, fake_ptr, fake_ptr, None, None, group)
    return prob, arr


def test_workspace_bytes_and_shape_errors():
    lib = pk.load_library()
    out = ct.c_size_t(0)
    good, keep = _problem([(1, 1), (2, 1), (1, 2), (2, 4)])
    assert lib.parcae_workspace_bytes(ct.byref(good), ct.byref(out)) == pk.PARCAE_OK
    assert out.value >= 4 * 16 + 4 + 4 * 4 * 4 and out.value % 256 == 0
    grouped, keep2 = _problem([(4, 4), (8, 4)], group=4)      # 32 GPUs on 8 four-GPU instances
    assert lib.parcae_workspace_bytes(ct.byref(grouped), ct.byref(out)) == pk.PARCAE_OK
    assert lib.parcae_workspace_bytes(ct.byref(good), None) == pk.PARCAE_EINVAL
    assert lib.parcae_workspace_bytes(None, ct.byref(out)) == pk.PARCAE_EINVAL
    bad_cases = [
        _problem([(2, 1), (1, 1)]),              # not sorted
        _problem([(1, 1), (1, 1)]),              # duplicate
        _problem([(1, 2), (1, 1)]),              # P descending
        _problem([(3, 4)]),                      # D * P > N
        _problem([(0, 1)]), _problem([(1, 0)]),
        _problem([(1, 1)], N=257), _problem([(1, 1)], N=0),
        _problem([(1, 1)], T=0), _problem([(1, 1)], nq=0),
        _problem([(1, 1)], S=0), _problem([(1, 1)], S=(1 << 24) + 1),
        _problem([(1, 1)], tau=0.0), _problem([(1, 1)], tau=float("inf")), _problem([(1, 1)], tau=float("nan")),
        _problem([(1, 1)], flags=2), _problem([(1, 1)], flags=0x80000001),
        _problem([(1, 1)], fake_ptr=None),       # NULL device tables
        _problem([(3, 2)], group=2), _problem([(2, 2)], group=-1), _problem([(2, 2)], group=65),
        _problem([(20, 2)], group=4),            # 10 instances needed, 8 exist
    ]
    for prob, _keep in bad_cases:
        assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL


def test_structure_size_field():
    """The problem structure carries its own size: an older (shorter) caller is accepted as long as it has the
    members of the first release, a newer (longer) one is read up to what this build knows."""
    lib = pk.load_library()
    out = ct.c_size_t(0)
    prob, keep = _problem([(1, 1), (2, 1)])
    full = ct.sizeof(pk.parcae_problem)
    assert prob.struct_size == full
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_OK
    prob.struct_size = pk.parcae_problem.profile.offset      # a caller built before the profiling hooks existed
    prob.profile = ct.cast(0xdead0000, ct.POINTER(pk.parcae_profile))   # must not be read
    prob.cost_move = 0x1000                                   # nor this (without its histogram it would be refused)
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_OK
    prob.profile = None
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_OK
    prob.struct_size = full
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL   # cost_move without hist_occ
    prob.cost_move = None
    prob.struct_size = full + 64                              # a newer caller
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_OK
    for bad in (0, 4, pk.parcae_problem.cost_round.offset):
        prob.struct_size = bad
        assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL


def test_entry_points_reject_bad_arguments_before_any_launch():
    """NULL outputs, a missing or misaligned or short workspace: an error code and nothing is enqueued."""
    lib = pk.load_library()
    prob, keep = _problem([(1, 1), (2, 1), (1, 2)])
    need = ct.c_size_t(0)
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(need)) == 0
    fake = 0x10000
    # required outputs missing
    assert lib.parcae_liveput_eval(ct.byref(prob), None, fake, None, None, None, None, fake, need.value, None) == pk.PARCAE_EINVAL
    assert lib.parcae_plan_from_hist(ct.byref(prob), fake, fake, None, None, None, None, None, None, fake, need.value,
                                     None) == pk.PARCAE_EINVAL
    assert lib.parcae_transition_weights(ct.byref(prob), fake, fake, None, fake, need.value, None) == pk.PARCAE_EINVAL
    assert lib.parcae_dp_plan(None, 1, 1, 1, None, fake, fake, None, None, None, None) == pk.PARCAE_EINVAL
    assert lib.parcae_dp_plan(fake, 1, 1, 5000, None, fake, fake, None, None, None, None) == pk.PARCAE_EINVAL
    # no back-pointer output: only while they fit in the workgroup's local memory (2 * T * C <= 16384 bytes)
    assert lib.parcae_dp_plan(fake, 1, 100, 100, None, None, fake, None, None, None, None) == pk.PARCAE_EINVAL
    # workspace problems
    for ws, nbytes in ((None, need.value), (fake + 4, need.value), (fake, need.value - 1)):
        assert lib.parcae_liveput_eval(ct.byref(prob), fake, fake, None, None, None, None, ws, nbytes, None) == pk.PARCAE_EWORKSPACE
        assert lib.parcae_liveput_plan(ct.byref(prob), fake, fake, None, None, None, None, None, fake, None, None, None,
                                       ws, nbytes, None) == pk.PARCAE_EWORKSPACE
    # unit indices out of range
    assert lib.parcae_debug_sample(ct.byref(prob), 0, 4, 0, 0, 8, fake, fake, fake, fake, need.value, None) == pk.PARCAE_EINVAL
    assert lib.parcae_debug_sample(ct.byref(prob), 0, 0, 3, 0, 8, fake, fake, fake, fake, need.value, None) == pk.PARCAE_EINVAL
    assert lib.parcae_debug_sample(ct.byref(prob), 1, 0, 0, 0, 8, fake, fake, fake, fake, need.value, None) == pk.PARCAE_EINVAL


def test_zone_and_candidate_limits_are_checked_on_the_host():
    lib = pk.load_library()
    out = ct.c_size_t(0)
    fake = 0x1000
    prob, keep = _problem([(1, 1), (2, 1)])
    prob.n_zones = 5                                   # more zones than the library has
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL
    prob.n_zones = -1
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL
    prob.n_zones = 2                                   # zones without their tables
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL
    prob.zone, prob.zone_weight = fake, fake
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_OK
    # every (D, P) with D * P <= 256: about 1500 candidates, more than the planning kernels hold
    many = [(d, p) for p in range(1, 257) for d in range(1, 256 // p + 1)]
    assert len(many) > 1200
    big, keep2 = _problem(many, N=256, T=2)
    assert lib.parcae_workspace_bytes(ct.byref(big), ct.byref(out)) == pk.PARCAE_OK
    ws = 0x100000
    assert lib.parcae_plan_from_hist(ct.byref(big), fake, fake, None, None, fake, None, None, None, ws, out.value,
                                     None) == pk.PARCAE_EINVAL
    assert lib.parcae_liveput_plan(ct.byref(big), fake, fake, None, None, None, None, None, fake, None, None, None,
                                   ws, out.value, None) == pk.PARCAE_EINVAL


def test_weights_per_instance_and_cost_per_move_are_checked_on_the_host():
    lib = pk.load_library()
    out = ct.c_size_t(0)
    fake = 0x1000
    prob, keep = _problem([(1, 2), (2, 2), (1, 4)], nq=40)
    plain = ct.c_size_t(0)
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(plain)) == pk.PARCAE_OK
    prob.inst_weight = fake
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_OK
    prob.n_zones, prob.zone, prob.zone_weight = 2, fake, fake          # zones and instance weights exclude each other
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL
    prob.n_zones = 0
    prob.cost_move = fake                                               # needs its histogram
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL
    prob.hist_occ = fake
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_OK
    assert out.value > plain.value                                      # the weights go through the workspace
    prob.cost_round = fake                                              # two refinements of the same cost
    assert lib.parcae_workspace_bytes(ct.byref(prob), ct.byref(out)) == pk.PARCAE_EINVAL
    prob.cost_round = None
    need = ct.c_size_t(0)
    assert lib.parcae_replay_workspace_bytes(ct.byref(prob), 3, pk.PARCAE_REPLAY_PROACTIVE, ct.byref(need)) == pk.PARCAE_OK
    assert lib.parcae_replay(ct.byref(prob), 3, fake, fake, pk.PARCAE_REPLAY_PROACTIVE, fake, fake, fake, None, 0x100000,
                             need.value, None) == pk.PARCAE_EINVAL      # the replay takes no cost per moved instance
    deep, keep2 = _problem([(1, 256)], N=256, S=1 << 24)
    deep.cost_move, deep.hist_occ = fake, fake                          # S * P would overflow a 32-bit bin
    assert lib.parcae_workspace_bytes(ct.byref(deep), ct.byref(out)) == pk.PARCAE_EINVAL


def test_reactive_replay_needs_no_planner():
    """The reactive baseline never plans: no candidate limit, no planner part in its workspace."""
    lib = pk.load_library()
    many = [(d, p) for p in range(1, 257) for d in range(1, 256 // p + 1)]
    big, keep = _problem(many, N=256, T=3)
    pro, rea = ct.c_size_t(0), ct.c_size_t(0)
    assert lib.parcae_replay_workspace_bytes(ct.byref(big), 4, pk.PARCAE_REPLAY_PROACTIVE, ct.byref(pro)) == pk.PARCAE_OK
    assert lib.parcae_replay_workspace_bytes(ct.byref(big), 4, pk.PARCAE_REPLAY_REACTIVE, ct.byref(rea)) == pk.PARCAE_OK
    assert rea.value < pro.value
    assert lib.parcae_replay_workspace_bytes(ct.byref(big), 4, 7, ct.byref(rea)) == pk.PARCAE_EINVAL
    fake, ws = 0x1000, 0x100000
    # proactive: the candidate list does not fit the planning kernels; refused before anything is enqueued
    assert lib.parcae_replay(ct.byref(big), 4, fake, fake, pk.PARCAE_REPLAY_PROACTIVE, fake, fake, fake, None, ws,
                             pro.value, None) == pk.PARCAE_EINVAL
    # a short workspace is refused for either mode
    assert lib.parcae_replay(ct.byref(big), 4, fake, None, pk.PARCAE_REPLAY_REACTIVE, fake, fake, fake, None, ws,
                             rea.value - 1, None) == pk.PARCAE_EWORKSPACE


def test_static_entry_point_limits_are_checked_before_anything_else():
    """The entry point with the built-in workspace refuses problems beyond its stated limits on the host."""
    lib = pk.load_library()
    fake = 0x1000
    out = ct.c_size_t(0)
    # 1024 queries of a long horizon: the workspace would exceed the built-in array
    big, keep = _problem([(d, 4) for d in range(1, 17)], nq=4096, N=64, T=64)
    assert lib.parcae_workspace_bytes(ct.byref(big), ct.byref(out)) == pk.PARCAE_OK
    assert out.value > pk.PARCAE_STATIC_WORKSPACE_BYTES
    assert lib.parcae_liveput_plan_static(ct.byref(big), fake, fake, None, None, None, None, None, fake, None, None,
                                          None, None) == pk.PARCAE_EWORKSPACE
    # more candidates than its fixed table holds
    many = [(d, p) for p in range(1, 257) for d in range(1, 256 // p + 1)]
    assert len(many) > pk.PARCAE_STATIC_MAX_CONFIGS
    wide, keep2 = _problem(many, N=256, T=2)
    assert lib.parcae_liveput_plan_static(ct.byref(wide), fake, fake, None, None, None, None, None, fake, None, None,
                                          None, None) == pk.PARCAE_EINVAL
    # required outputs
    ok, keep3 = _problem([(1, 1), (2, 1)])
    assert lib.parcae_liveput_plan_static(ct.byref(ok), fake, fake, None, None, None, None, None, None, None, None,
                                          None, None) == pk.PARCAE_EINVAL


def test_product_has_no_cpu_path():
    """Without a GPU the binding raises instead of computing anything."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    import parcae_inputs as pi
    with pytest.raises(RuntimeError):
        pk.upload(pi.workload("tiny"))
