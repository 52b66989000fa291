"""Python binding of the liveput optimizer's HIP library (argument marshalling only).

Every step of the path runs in the library's kernels; this module turns torch
tensors into pointers, checks shapes and raises on error codes.  PyTorch is used
for device memory and the stream handle, nothing else.  There is no CPU
fallback: if `libparcae_hip.so` is missing or no GPU is present the calls raise.

Function names mirror include/parcae.h.
"""
from __future__ import annotations

import ctypes as ct
import os
from dataclasses import dataclass, field
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libparcae_hip.so")
if os.environ.get("PARCAE_HOST_SANITIZE") == "1":   # host code under the sanitizers (see build.build_host_sanitized)
    LIB_PATH = os.path.join(_HERE, "libparcae_hip_asan.so")

PARCAE_OK = 0
PARCAE_EINVAL = -1
PARCAE_EWORKSPACE = -2
PARCAE_EHIP = -3
PARCAE_EINFEASIBLE = -4
PARCAE_MAX_INSTANCES = 256
PARCAE_MAX_ZONES = 4
PARCAE_MAX_SCENARIOS = 1 << 24
PARCAE_POOL_USED = 0
PARCAE_POOL_ALL = 1
PARCAE_COLD_START = -2
PARCAE_REPLAY_PROACTIVE = 0
PARCAE_REPLAY_REACTIVE = 1
PARCAE_STATIC_WORKSPACE_BYTES = 16 << 20
PARCAE_STATIC_MAX_CONFIGS = 1024

EXPORTED_SYMBOLS = (
    "parcae_workspace_bytes", "parcae_hist_len", "parcae_liveput_eval", "parcae_plan_from_hist",
    "parcae_liveput_plan", "parcae_transition_weights", "parcae_dp_plan", "parcae_debug_sample",
    "parcae_strerror", "parcae_version", "parcae_replay", "parcae_replay_workspace_bytes",
    "parcae_liveput_plan_static",
)


class ParcaeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


class parcae_config(ct.Structure):
    _fields_ = [("D", ct.c_int32), ("P", ct.c_int32)]


class parcae_profile(ct.Structure):
    _fields_ = [("event_before_sampling", ct.c_void_p), ("event_after_sampling", ct.c_void_p),
                ("event_before_plan", ct.c_void_p), ("event_after_plan", ct.c_void_p)]


class parcae_problem(ct.Structure):
    _fields_ = [
        ("struct_size", ct.c_uint32),
        ("n_queries", ct.c_int32), ("n_instances", ct.c_int32), ("n_intervals", ct.c_int32),
        ("n_configs", ct.c_int32), ("n_scenarios", ct.c_int32), ("p_min", ct.c_int32),
        ("interval_sec", ct.c_float), ("flags", ct.c_uint32),
        ("configs", ct.POINTER(parcae_config)),
        ("avail", ct.c_void_p), ("thr", ct.c_void_p), ("cost", ct.c_void_p), ("seed", ct.c_void_p),
        ("stream_id", ct.c_void_p), ("cur_config", ct.c_void_p),
        ("group_size", ct.c_int32), ("n_zones", ct.c_int32),
        ("zone", ct.c_void_p), ("zone_weight", ct.c_void_p), ("cost_round", ct.c_void_p),
        ("profile", ct.POINTER(parcae_profile)),
        ("inst_weight", ct.c_void_p), ("cost_move", ct.c_void_p), ("hist_occ", ct.c_void_p),
    ]


_lib: Optional[ct.CDLL] = None


def load_library() -> ct.CDLL:
    """Load the C-ABI library (after torch, so that both use one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2403_14097_amd.build`")
    import torch  # noqa: F401  (loads the HIP runtime the library links against)
    lib = ct.CDLL(LIB_PATH)
    vp, i32, u32, sz = ct.c_void_p, ct.c_int32, ct.c_uint32, ct.c_size_t
    pp = ct.POINTER(parcae_problem)
    lib.parcae_workspace_bytes.argtypes = [pp, ct.POINTER(sz)]
    lib.parcae_hist_len.argtypes = [ct.POINTER(parcae_config), i32]
    lib.parcae_hist_len.restype = ct.c_int64
    lib.parcae_liveput_eval.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.parcae_plan_from_hist.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.parcae_liveput_plan.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.parcae_transition_weights.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.parcae_liveput_plan_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.parcae_dp_plan.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.parcae_debug_sample.argtypes = [pp, i32, i32, i32, u32, u32, vp, vp, vp, vp, sz, vp]
    lib.parcae_replay_workspace_bytes.argtypes = [pp, i32, i32, ct.POINTER(sz)]
    lib.parcae_replay.argtypes = [pp, i32, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.parcae_strerror.argtypes = [ct.c_int]
    lib.parcae_strerror.restype = ct.c_char_p
    lib.parcae_version.restype = ct.c_int
    for name in EXPORTED_SYMBOLS:
        if name not in ("parcae_hist_len", "parcae_strerror"):
            getattr(lib, name).restype = ct.c_int
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().parcae_strerror(int(code)).decode()


def parcae_version() -> int:
    return int(load_library().parcae_version())


def _require_gpu():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("paper_2403_14097_amd needs a GPU: there is no CPU path")
    return torch


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_handle() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


@dataclass
class Problem:
    """A batch of planning queries with its per-query tables resident on the GPU."""

    n_instances: int
    n_intervals: int
    interval_sec: float
    p_min: int
    n_scenarios: int
    configs: list                 # [(D, P)] host
    avail: "object"               # int32  [nq, T+1] device
    thr: "object"                 # float32 [nq, L] device
    cost: "object"                # float32 [nq, C, 3] device
    seed: "object"                # int64 view of uint64 [nq] device
    stream_id: "object" = None    # int32 view of uint32 [nq] device, or None
    cur_config: "object" = None   # int32 [nq] device, or None
    flags: int = 0                # PARCAE_POOL_USED or PARCAE_POOL_ALL
    group_size: int = 1           # GPUs per instance (preempted together)
    n_zones: int = 0              # 0: uniform preemption; else zones of unequal hazard
    zone: "object" = None         # uint8 [nq, N] device, zone of every instance
    zone_weight: "object" = None  # int32 view of uint32 [nq, PARCAE_MAX_ZONES] device
    cost_round: "object" = None   # float32 [nq, C] device: seconds per further transfer round, or None
    inst_weight: "object" = None  # uint8 [nq, N] device: hazard weight of every instance, or None
    cost_move: "object" = None    # float32 [nq, C] device: seconds per instance that must receive state, or None
    hist_occ: "object" = None     # int32 view of uint32 [nq, T, L] device: stage-occupancy statistic (with cost_move)
    profile_events: Optional[tuple] = None   # raw hipEvent_t handles (before sampling, after sampling, before plan,
                                             # after plan; each an int or None) for the library to record
    _profile: object = field(default=None, repr=False)
    _cfg_arr: object = field(default=None, repr=False)
    _workspace: object = field(default=None, repr=False)

    @property
    def n_queries(self) -> int:
        return int(self.avail.shape[0])

    @property
    def n_configs(self) -> int:
        return len(self.configs)

    @property
    def hist_len(self) -> int:
        return sum(d + 1 for d, _ in self.configs)

    def c_struct(self) -> parcae_problem:
        if self._cfg_arr is None:
            arr = (parcae_config * len(self.configs))()
            for i, (d, p) in enumerate(self.configs):
                arr[i].D, arr[i].P = int(d), int(p)
            self._cfg_arr = arr
        prof = None
        if self.profile_events is not None:
            self._profile = parcae_profile(*self.profile_events)   # kept alive by the Problem
            prof = ct.pointer(self._profile)
        return parcae_problem(
            ct.sizeof(parcae_problem), self.n_queries, self.n_instances, self.n_intervals, self.n_configs,
            self.n_scenarios, self.p_min, self.interval_sec, int(self.flags),
            ct.cast(self._cfg_arr, ct.POINTER(parcae_config)),
            _ptr(self.avail), _ptr(self.thr), _ptr(self.cost), _ptr(self.seed), _ptr(self.stream_id),
            _ptr(self.cur_config), int(self.group_size),
            int(self.n_zones), _ptr(self.zone), _ptr(self.zone_weight), _ptr(self.cost_round), prof,
            _ptr(self.inst_weight), _ptr(self.cost_move), _ptr(self.hist_occ) if self.cost_move is not None else None)

    def workspace(self):
        """Device workspace of the size the library asks for (allocated once per Problem)."""
        torch = _require_gpu()
        need = parcae_workspace_bytes(self)
        if self._workspace is None or self._workspace.numel() < need:
            self._workspace = torch.empty(need + 256, dtype=torch.uint8, device=self.avail.device)
        ptr = self._workspace.data_ptr()
        pad = (-ptr) % 256
        return ptr + pad, self._workspace.numel() - pad


def problem_from_arrays(n_instances, n_intervals, interval_sec, p_min, n_scenarios, configs, avail, thr, cost, seed,
                        stream_id=None, cur_config=None, device="cuda:0") -> Problem:
    """Upload numpy arrays (same layout as the C structure) and wrap them in a Problem."""
    torch = _require_gpu()
    import numpy as np

    def up(a, dt):
        return torch.from_numpy(np.array(a, dtype=dt, order="C")).to(device)   # a writable, contiguous copy

    seed_dev = up(np.asarray(seed, dtype=np.uint64).view(np.int64), np.int64)
    sid = None if stream_id is None else up(np.asarray(stream_id, dtype=np.uint32).view(np.int32), np.int32)
    cur = None if cur_config is None else up(cur_config, np.int32)
    return Problem(int(n_instances), int(n_intervals), float(interval_sec), int(p_min), int(n_scenarios),
                   [(int(d), int(p)) for d, p in np.asarray(configs).reshape(-1, 2)],
                   up(avail, np.int32), up(thr, np.float32), up(cost, np.float32), seed_dev, sid, cur)


def upload(batch, device="cuda:0", n_scenarios: Optional[int] = None) -> Problem:
    """Problem from any object with the attribute names of the C structure (numpy arrays)."""
    prob = problem_from_arrays(batch.n_instances, batch.n_intervals, batch.interval_sec, batch.p_min,
                               batch.n_scenarios if n_scenarios is None else n_scenarios, batch.configs, batch.avail,
                               batch.thr, batch.cost, batch.seed, batch.stream_id, batch.cur_config, device)
    prob.group_size = int(getattr(batch, "group_size", 1))
    if int(getattr(batch, "n_zones", 0)) > 0:
        torch = _require_gpu()
        import numpy as np
        prob.n_zones = int(batch.n_zones)
        prob.zone = torch.from_numpy(np.array(batch.zone, dtype=np.uint8, order="C")).to(device)
        prob.zone_weight = torch.from_numpy(
            np.array(batch.zone_weight, dtype=np.uint32, order="C").view(np.int32)).to(device)
    if getattr(batch, "cost_round", None) is not None:
        torch = _require_gpu()
        import numpy as np
        prob.cost_round = torch.from_numpy(np.array(batch.cost_round, dtype=np.float32, order="C")).to(device)
    if getattr(batch, "inst_weight", None) is not None:
        torch = _require_gpu()
        import numpy as np
        prob.inst_weight = torch.from_numpy(np.array(batch.inst_weight, dtype=np.uint8, order="C")).to(device)
    if getattr(batch, "cost_move", None) is not None:
        torch = _require_gpu()
        import numpy as np
        prob.cost_move = torch.from_numpy(np.array(batch.cost_move, dtype=np.float32, order="C")).to(device)
    return prob


def _check(rc: int, where: str):
    if rc != PARCAE_OK:
        raise ParcaeError(rc, where)


def parcae_workspace_bytes(p: Problem) -> int:
    out = ct.c_size_t(0)
    cs = p.c_struct()
    _check(load_library().parcae_workspace_bytes(ct.byref(cs), ct.byref(out)), "parcae_workspace_bytes")
    return int(out.value)


def parcae_hist_len(configs) -> int:
    arr = (parcae_config * len(configs))()
    for i, (d, pp) in enumerate(configs):
        arr[i].D, arr[i].P = int(d), int(pp)
    return int(load_library().parcae_hist_len(arr, len(configs)))


@dataclass
class EvalOut:
    hist_int: "object"   # int32 view of uint32 [nq, T, L]
    hist_min: "object"
    liveput: "object"    # [nq, 3, T, C]
    teff: "object"       # [nq, T, C]
    gain: "object"
    status: "object"     # [nq]
    hist_occ: "object" = None   # int32 view of uint32 [nq, T, L]: stage-occupancy statistic, with cost_move only


@dataclass
class PlanOut:
    F: "object"          # [nq, T+1, C]
    bp: "object"         # [nq, T, C]
    plan: "object"       # [nq, T]
    start: "object"      # [nq]
    objective: "object"  # [nq]
    status: "object"     # [nq]


def alloc_eval_out(p: Problem, tables: bool = True) -> EvalOut:
    torch = _require_gpu()
    dev = p.avail.device
    nq, T, C, L = p.n_queries, p.n_intervals, p.n_configs, p.hist_len
    f = lambda *s: torch.empty(s, dtype=torch.float32, device=dev)  # noqa: E731
    i = lambda *s: torch.empty(s, dtype=torch.int32, device=dev)    # noqa: E731
    return EvalOut(i(nq, T, L), i(nq, T, L), f(nq, 3, T, C) if tables else None, f(nq, T, C) if tables else None,
                   f(nq, T, C) if tables else None, i(nq), i(nq, T, L) if p.cost_move is not None else None)


def alloc_plan_out(p: Problem, full: bool = True) -> PlanOut:
    torch = _require_gpu()
    dev = p.avail.device
    nq, T, C = p.n_queries, p.n_intervals, p.n_configs
    f = lambda *s: torch.empty(s, dtype=torch.float32, device=dev)  # noqa: E731
    i = lambda *s: torch.empty(s, dtype=torch.int32, device=dev)    # noqa: E731
    return PlanOut(f(nq, T + 1, C) if full else None, i(nq, T, C) if full else None, i(nq, T), i(nq), f(nq), i(nq))


def parcae_liveput_eval(p: Problem, out: Optional[EvalOut] = None) -> EvalOut:
    out = out or alloc_eval_out(p)
    p.hist_occ = out.hist_occ          # the third statistic travels in the problem structure
    ws, nbytes = p.workspace()
    cs = p.c_struct()
    _check(load_library().parcae_liveput_eval(ct.byref(cs), _ptr(out.hist_int), _ptr(out.hist_min), _ptr(out.liveput),
                                              _ptr(out.teff), _ptr(out.gain), _ptr(out.status), ws, nbytes,
                                              _stream_handle()), "parcae_liveput_eval")
    return out


def parcae_plan_from_hist(p: Problem, hist_int, hist_min, out: Optional[PlanOut] = None) -> PlanOut:
    out = out or alloc_plan_out(p)
    ws, nbytes = p.workspace()
    cs = p.c_struct()
    _check(load_library().parcae_plan_from_hist(ct.byref(cs), _ptr(hist_int), _ptr(hist_min), _ptr(out.F), _ptr(out.bp),
                                                _ptr(out.plan), _ptr(out.start), _ptr(out.objective), _ptr(out.status),
                                                ws, nbytes, _stream_handle()), "parcae_plan_from_hist")
    return out


def parcae_liveput_plan(p: Problem, ev: Optional[EvalOut] = None, out: Optional[PlanOut] = None):
    ev = ev or alloc_eval_out(p)
    out = out or alloc_plan_out(p)
    p.hist_occ = ev.hist_occ
    ws, nbytes = p.workspace()
    cs = p.c_struct()
    _check(load_library().parcae_liveput_plan(ct.byref(cs), _ptr(ev.hist_int), _ptr(ev.hist_min), _ptr(ev.liveput),
                                              _ptr(ev.teff), _ptr(ev.gain), _ptr(out.F), _ptr(out.bp), _ptr(out.plan),
                                              _ptr(out.start), _ptr(out.objective), _ptr(out.status), ws, nbytes,
                                              _stream_handle()), "parcae_liveput_plan")
    return ev, out


def parcae_liveput_plan_static(p: Problem, ev: EvalOut, out: PlanOut):
    """parcae_liveput_plan on the library's built-in workspace; the output buffers must be passed in (this call
    allocates nothing)."""
    p.hist_occ = ev.hist_occ
    cs = p.c_struct()
    _check(load_library().parcae_liveput_plan_static(ct.byref(cs), _ptr(ev.hist_int), _ptr(ev.hist_min), _ptr(ev.liveput),
                                                     _ptr(ev.teff), _ptr(ev.gain), _ptr(out.F), _ptr(out.bp),
                                                     _ptr(out.plan), _ptr(out.start), _ptr(out.objective),
                                                     _ptr(out.status), _stream_handle()), "parcae_liveput_plan_static")
    return ev, out


def parcae_transition_weights(p: Problem, hist_int, hist_min, W=None):
    torch = _require_gpu()
    if W is None:
        W = torch.empty((p.n_queries, p.n_intervals, p.n_configs, p.n_configs), dtype=torch.float32,
                        device=p.avail.device)
    ws, nbytes = p.workspace()
    cs = p.c_struct()
    _check(load_library().parcae_transition_weights(ct.byref(cs), _ptr(hist_int), _ptr(hist_min), _ptr(W), ws, nbytes,
                                                    _stream_handle()), "parcae_transition_weights")
    return W


def parcae_dp_plan(W, out: Optional[PlanOut] = None) -> PlanOut:
    torch = _require_gpu()
    nq, T, C, C2 = W.shape
    assert C == C2 and W.dtype == torch.float32 and W.is_contiguous()
    if out is None:
        f = lambda *s: torch.empty(s, dtype=torch.float32, device=W.device)  # noqa: E731
        i = lambda *s: torch.empty(s, dtype=torch.int32, device=W.device)    # noqa: E731
        out = PlanOut(f(nq, T + 1, C), i(nq, T, C), i(nq, T), i(nq), f(nq), i(nq))
    _check(load_library().parcae_dp_plan(_ptr(W), nq, T, C, _ptr(out.F), _ptr(out.bp), _ptr(out.plan), _ptr(out.start),
                                         _ptr(out.objective), _ptr(out.status), _stream_handle()), "parcae_dp_plan")
    return out


def parcae_debug_sample(p: Problem, q: int, t: int, c: int, s0: int, ns: int):
    torch = _require_gpu()
    dev = p.avail.device
    masks = torch.empty((ns, 8), dtype=torch.int32, device=dev)
    n_int = torch.empty(ns, dtype=torch.int32, device=dev)
    d_min = torch.empty(ns, dtype=torch.int32, device=dev)
    ws, nbytes = p.workspace()
    cs = p.c_struct()
    _check(load_library().parcae_debug_sample(ct.byref(cs), q, t, c, s0, ns, _ptr(masks), _ptr(n_int), _ptr(d_min), ws,
                                              nbytes, _stream_handle()), "parcae_debug_sample")
    return masks, n_int, d_min


def parcae_replay(p: Problem, true_avail, windows, mode: int = PARCAE_REPLAY_PROACTIVE, with_status: bool = False):
    """Replay every query over H = true_avail.shape[1] - 1 steps; returns (chosen [nq, H], reward [nq, H], total [nq])
    and, with_status, the per-query status [nq] as a fourth element."""
    torch = _require_gpu()
    dev = p.thr.device
    nq, H = int(true_avail.shape[0]), int(true_avail.shape[1]) - 1
    assert true_avail.dtype == torch.int32 and true_avail.is_contiguous()
    if windows is not None:
        assert windows.dtype == torch.int32 and windows.is_contiguous()
        assert tuple(windows.shape) == (H, nq, p.n_intervals + 1)
    chosen = torch.empty((nq, H), dtype=torch.int32, device=dev)
    reward = torch.empty((nq, H), dtype=torch.float32, device=dev)
    total = torch.empty(nq, dtype=torch.float32, device=dev)
    cs = p.c_struct()
    need = ct.c_size_t(0)
    status = torch.empty(nq, dtype=torch.int32, device=dev) if with_status else None
    _check(load_library().parcae_replay_workspace_bytes(ct.byref(cs), H, int(mode), ct.byref(need)),
           "parcae_replay_workspace_bytes")
    ws = torch.empty(need.value + 256, dtype=torch.uint8, device=dev)
    ptr = ws.data_ptr()
    pad = (-ptr) % 256
    _check(load_library().parcae_replay(ct.byref(cs), H, _ptr(true_avail), _ptr(windows), int(mode), _ptr(chosen),
                                        _ptr(reward), _ptr(total), _ptr(status), ptr + pad, ws.numel() - pad,
                                        _stream_handle()), "parcae_replay")
    torch.cuda.current_stream().synchronize()   # the workspace tensor must outlive the enqueued work
    return (chosen, reward, total, status) if with_status else (chosen, reward, total)
