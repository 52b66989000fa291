"""ctypes front end of the CPU oracle (test infrastructure, not product code).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
It takes plain numpy arrays, calls `liboracle.so` (built from
`parcae_oracle.c` with gcc) and returns numpy arrays.  It imports nothing from
the GPU package.
"""
from __future__ import annotations

import ctypes as ct
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "parcae_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_LIB_SANITIZED = os.path.join(_HERE, "liboracle_asan.so")
SANITIZE_ENV = "PARCAE_ORACLE_SANITIZE"   # "1": load the build with AddressSanitizer and UndefinedBehaviorSanitizer
_lib: Optional[ct.CDLL] = None


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, OpenMP for the unit loop).

    sanitize=True builds liboracle_asan.so instead: the same source under -fsanitize=address,undefined (any
    finding aborts).  A process that loads it must have gcc's libasan preloaded (see sanitizer_runtime())."""
    out = _LIB_SANITIZED if sanitize else _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        flags = (["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
                 if sanitize else ["-O2"])
        cmd = ["gcc", "-std=c11", *flags, "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return out


def sanitizer_runtime() -> str:
    """Path of gcc's AddressSanitizer runtime, to be put first in LD_PRELOAD of a process that loads the sanitized build."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(ct.POINTER(ty))


def lib() -> ct.CDLL:
    global _lib
    if _lib is None:
        sanitized = os.environ.get(SANITIZE_ENV) == "1"
        _lib = ct.CDLL(build(sanitize=sanitized))
        _lib.orc_word.restype = ct.c_uint32
        _lib.orc_word.argtypes = [ct.c_uint64, ct.c_uint32, ct.c_uint32, ct.c_uint32, ct.c_uint32]
        _lib.orc_word_at.restype = ct.c_uint32
        _lib.orc_word_at.argtypes = [ct.c_uint64, ct.c_uint32, ct.c_uint32, ct.c_uint32, ct.c_uint32, ct.c_uint32]
        _lib.orc_dp_f32.restype = ct.c_int
        _lib.orc_dp_f64.restype = ct.c_double
        _lib.orc_num_threads.restype = ct.c_int
    return _lib


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c, ct.c_uint32), _p(k, ct.c_uint32), _p(out, ct.c_uint32))
    return out


def word(seed: int, stream_id: int, unit: int, s: int, i: int) -> int:
    return int(lib().orc_word(ct.c_uint64(seed), stream_id, unit, s, i))


def sample_preempted(M: int, k: int, seed: int, stream_id: int, unit: int, s: int) -> np.ndarray:
    out = np.zeros(M, dtype=np.uint8)
    lib().orc_sample_preempted(ct.c_int(M), ct.c_int(k), ct.c_uint64(seed), ct.c_uint32(stream_id),
                               ct.c_uint32(unit), ct.c_uint32(s), _p(out, ct.c_uint8))
    return out


def _zones(zone, weight):
    """(n_zones, zone pointer, weight pointer, keep-alive arrays) for the C calls; uniform when zone is None.
    weight == "instances": `zone` holds a hazard weight per instance (n_zones = -1 in the C calls)."""
    if zone is None:
        return ct.c_int(0), None, None, ()
    z = np.ascontiguousarray(zone, dtype=np.uint8)
    if isinstance(weight, str) and weight == "instances":
        return ct.c_int(-1), _p(z, ct.c_uint8), None, (z,)
    w = np.ascontiguousarray(weight, dtype=np.uint32)
    return ct.c_int(int(w.size)), _p(z, ct.c_uint8), _p(w, ct.c_uint32), (z, w)


def sample_preempted_weighted(M: int, k: int, weight, seed: int, stream_id: int, unit: int, s: int) -> np.ndarray:
    """Successive weighted sampling without replacement with a hazard weight (1..255) per instance."""
    out = np.zeros(M, dtype=np.uint8)
    w = np.ascontiguousarray(weight, dtype=np.uint8)
    assert w.size >= M and (M == 0 or w[:M].min() >= 1)
    lib().orc_sample_preempted_weighted(ct.c_int(M), ct.c_int(k), _p(w, ct.c_uint8), ct.c_uint64(seed),
                                        ct.c_uint32(stream_id), ct.c_uint32(unit), ct.c_uint32(s), _p(out, ct.c_uint8))
    return out


def word_at(seed: int, stream_id: int, unit: int, s: int, prefix: int, i: int) -> int:
    return int(lib().orc_word_at(ct.c_uint64(seed), stream_id, unit, s, prefix, i))


def sample_preempted_zoned(M: int, k: int, zone, weight, seed: int, stream_id: int, unit: int, s: int) -> np.ndarray:
    out = np.zeros(M, dtype=np.uint8)
    nz, zp, wp, keep = _zones(zone, weight)
    assert len(keep[0]) >= M
    lib().orc_sample_preempted_zoned(ct.c_int(M), ct.c_int(k), nz, zp, wp, ct.c_uint64(seed), ct.c_uint32(stream_id),
                                     ct.c_uint32(unit), ct.c_uint32(s), _p(out, ct.c_uint8))
    return out


def reduce(D: int, P: int, preempted: np.ndarray):
    pre = np.ascontiguousarray(preempted, dtype=np.uint8)
    assert pre.size == D * P
    n_int, d_min = ct.c_int(0), ct.c_int(0)
    occ = np.zeros(P, dtype=np.int32)
    lib().orc_reduce(ct.c_int(D), ct.c_int(P), _p(pre, ct.c_uint8), ct.byref(n_int), ct.byref(d_min),
                     _p(occ, ct.c_int32))
    return n_int.value, d_min.value, occ


def debug_sample(D: int, P: int, a_next: int, seed: int, stream_id: int, unit: int, s0: int, ns: int,
                 a_prev: int = -1, group: int = 1, zone=None, weight=None):
    """a_prev >= 0: preemptions drawn among all a_prev available instances (the first D * P run the grid)."""
    masks = np.zeros((ns, 8), dtype=np.uint32)
    n_int = np.zeros(ns, dtype=np.int32)
    d_min = np.zeros(ns, dtype=np.int32)
    nz, zp, wp, _keep = _zones(zone, weight)
    lib().orc_debug_sample(ct.c_int(D), ct.c_int(P), ct.c_int(group), ct.c_int(a_prev), ct.c_int(a_next), nz, zp, wp,
                           ct.c_uint64(seed),
                           ct.c_uint32(stream_id), ct.c_uint32(unit), ct.c_uint32(s0), ct.c_uint32(ns),
                           _p(masks, ct.c_uint32), _p(n_int, ct.c_int32), _p(d_min, ct.c_int32))
    return masks, n_int, d_min


def eval_unit(D: int, P: int, a_next: int, seed: int, stream_id: int, unit: int, s_begin: int, s_end: int,
              a_prev: int = -1, group: int = 1, zone=None, weight=None, with_occ: bool = False):
    """Histograms [D + 1] of one unit (unit = t * C + c) over scenarios [s_begin, s_end); with_occ adds the
    stage-occupancy statistic as a third array."""
    hi = np.zeros(D + 1, dtype=np.uint32)
    hm = np.zeros(D + 1, dtype=np.uint32)
    ho = np.zeros(D + 1, dtype=np.uint32) if with_occ else None
    nz, zp, wp, _keep = _zones(zone, weight)
    lib().orc_eval_unit(ct.c_int(D), ct.c_int(P), ct.c_int(group), ct.c_int(a_prev), ct.c_int(a_next), nz, zp, wp,
                        ct.c_uint64(seed),
                        ct.c_uint32(stream_id),
                        ct.c_uint32(unit), ct.c_uint32(s_begin), ct.c_uint32(s_end), _p(hi, ct.c_uint32),
                        _p(hm, ct.c_uint32), None if ho is None else _p(ho, ct.c_uint32))
    return (hi, hm, ho) if with_occ else (hi, hm)


def eval_hist(configs, thr_off, avail, seed: int, stream_id: int, s_begin: int, s_end: int, n_threads: int = 1,
              pool_all: bool = False, group: int = 1, zone=None, weight=None, want=None, with_occ: bool = False):
    """Histograms [T][L] of one query over scenarios [s_begin, s_end).  want: optional uint8 [T, C]; only the units
    with a non-zero entry are evaluated, the rows of the others stay zero.  with_occ adds the stage-occupancy
    statistic as a third array."""
    nz, zp, wp, _keep = _zones(zone, weight)
    configs = np.ascontiguousarray(configs, dtype=np.int32)
    thr_off = np.ascontiguousarray(thr_off, dtype=np.int32)
    avail = np.ascontiguousarray(avail, dtype=np.int32)
    C, T, L = configs.shape[0], avail.shape[0] - 1, int(thr_off[-1])
    hi = np.zeros((T, L), dtype=np.uint32)
    hm = np.zeros((T, L), dtype=np.uint32)
    ho = np.zeros((T, L), dtype=np.uint32) if with_occ else None
    wanted = None if want is None else np.ascontiguousarray(want, dtype=np.uint8).reshape(T * C)
    lib().orc_eval_hist_some(ct.c_int(T), ct.c_int(C), _p(configs, ct.c_int32), _p(thr_off, ct.c_int32),
                             _p(avail, ct.c_int32), ct.c_uint64(seed), ct.c_uint32(stream_id),
                             ct.c_uint32(s_begin), ct.c_uint32(s_end), _p(hi, ct.c_uint32), _p(hm, ct.c_uint32),
                             ct.c_int(n_threads), ct.c_int(1 if pool_all else 0), ct.c_int(group), nz, zp, wp,
                             None if wanted is None else _p(wanted, ct.c_uint8),
                             None if ho is None else _p(ho, ct.c_uint32))
    return (hi, hm, ho) if with_occ else (hi, hm)


@dataclass
class Tables:
    liveput_d: np.ndarray  # [3][T][C] double
    teff_d: np.ndarray
    gain_d: np.ndarray
    liveput_f: np.ndarray  # same, fixed-order float
    teff_f: np.ndarray
    gain_f: np.ndarray


def _rounds(cost_round):
    if cost_round is None:
        return None, None
    r = np.ascontiguousarray(cost_round, dtype=np.float32)
    return _p(r, ct.c_float), r


def _moves(cost_move, hist_occ):
    if cost_move is None:
        return None, None, ()
    m = np.ascontiguousarray(cost_move, dtype=np.float32)
    o = np.ascontiguousarray(hist_occ, dtype=np.uint32)
    return _p(m, ct.c_float), _p(o, ct.c_uint32), (m, o)


def finalise(configs, thr_off, avail, thr, cost, tau: float, S: int, hist_int, hist_min,
             pool_all: bool = False, group: int = 1, cost_round=None, cost_move=None, hist_occ=None) -> Tables:
    configs = np.ascontiguousarray(configs, dtype=np.int32)
    thr_off = np.ascontiguousarray(thr_off, dtype=np.int32)
    avail = np.ascontiguousarray(avail, dtype=np.int32)
    thr = np.ascontiguousarray(thr, dtype=np.float32)
    cost = np.ascontiguousarray(cost, dtype=np.float32)
    hi = np.ascontiguousarray(hist_int, dtype=np.uint32)
    hm = np.ascontiguousarray(hist_min, dtype=np.uint32)
    C, T = configs.shape[0], avail.shape[0] - 1
    out = Tables(np.zeros((3, T, C)), np.zeros((T, C)), np.zeros((T, C)),
                 np.zeros((3, T, C), np.float32), np.zeros((T, C), np.float32), np.zeros((T, C), np.float32))
    rp, _keep = _rounds(cost_round)
    mp, op, _keep2 = _moves(cost_move, hist_occ)
    lib().orc_finalise(ct.c_int(T), ct.c_int(C), _p(configs, ct.c_int32), _p(thr_off, ct.c_int32),
                       _p(avail, ct.c_int32), _p(thr, ct.c_float), _p(cost, ct.c_float), rp, ct.c_float(tau),
                       ct.c_uint32(S), ct.c_int(1 if pool_all else 0), ct.c_int(group), _p(hi, ct.c_uint32),
                       _p(hm, ct.c_uint32), _p(out.liveput_d, ct.c_double), _p(out.teff_d, ct.c_double), _p(out.gain_d, ct.c_double),
                       _p(out.liveput_f, ct.c_float), _p(out.teff_f, ct.c_float), _p(out.gain_f, ct.c_float), mp, op)
    return out


def transition(configs, thr_off, avail, thr, cost, tau: float, S: int, p_min: int, cur_config: int,
               hist_int, hist_min, group: int = 1, cost_round=None, cost_move=None, hist_occ=None):
    """W[T][C][C] in double and in fixed-order float."""
    configs = np.ascontiguousarray(configs, dtype=np.int32)
    thr_off = np.ascontiguousarray(thr_off, dtype=np.int32)
    avail = np.ascontiguousarray(avail, dtype=np.int32)
    thr = np.ascontiguousarray(thr, dtype=np.float32)
    cost = np.ascontiguousarray(cost, dtype=np.float32)
    hi = np.ascontiguousarray(hist_int, dtype=np.uint32)
    hm = np.ascontiguousarray(hist_min, dtype=np.uint32)
    C, T = configs.shape[0], avail.shape[0] - 1
    W_d = np.zeros((T, C, C), dtype=np.float64)
    W_f = np.zeros((T, C, C), dtype=np.float32)
    rp, _keep = _rounds(cost_round)
    mp, op, _keep2 = _moves(cost_move, hist_occ)
    lib().orc_transition(ct.c_int(T), ct.c_int(C), _p(configs, ct.c_int32), _p(thr_off, ct.c_int32),
                         _p(avail, ct.c_int32), _p(thr, ct.c_float), _p(cost, ct.c_float), rp, ct.c_float(tau),
                         ct.c_uint32(S), ct.c_int(p_min), ct.c_int(cur_config), ct.c_int(group),
                         _p(hi, ct.c_uint32), _p(hm, ct.c_uint32), _p(W_d, ct.c_double), _p(W_f, ct.c_float), mp, op)
    return W_d, W_f


@dataclass
class Plan:
    F: np.ndarray          # [T+1][C] float32
    bp: np.ndarray         # [T][C] int32
    plan: np.ndarray       # [T] int32
    start: int
    objective: float       # float32 value
    feasible: bool


def dp_f32(W: np.ndarray) -> Plan:
    W = np.ascontiguousarray(W, dtype=np.float32)
    T, C = W.shape[0], W.shape[1]
    F = np.zeros((T + 1, C), dtype=np.float32)
    bp = np.zeros((T, C), dtype=np.int32)
    plan = np.zeros(T, dtype=np.int32)
    start = ct.c_int32(0)
    obj = ct.c_float(0)
    ok = lib().orc_dp_f32(ct.c_int(T), ct.c_int(C), _p(W, ct.c_float), _p(F, ct.c_float), _p(bp, ct.c_int32),
                          _p(plan, ct.c_int32), ct.byref(start), ct.byref(obj))
    return Plan(F, bp, plan, int(start.value), float(obj.value), bool(ok))


def dp_f64(W: np.ndarray) -> float:
    W = np.ascontiguousarray(W, dtype=np.float64)
    return float(lib().orc_dp_f64(ct.c_int(W.shape[0]), ct.c_int(W.shape[1]), _p(W, ct.c_double)))


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ---------------------------------------------------------------- whole-batch helpers

@dataclass
class QueryResult:
    hist_int: np.ndarray
    hist_min: np.ndarray
    tables: Tables
    W_d: np.ndarray
    W_f: np.ndarray
    plan: Plan
    objective_d: float
    hist_occ: Optional[np.ndarray] = None


def batch_zones(batch, q: int):
    """(zone[N], weight[n_zones]) of query q, (weight per instance [N], "instances") when the batch carries
    per-instance hazard weights, or (None, None) when it draws uniformly."""
    per_instance = getattr(batch, "inst_weight", None)
    if per_instance is not None:
        return per_instance[q], "instances"
    zone = getattr(batch, "zone", None)
    if zone is None:
        return None, None
    return zone[q], batch.zone_weight[q][: int(batch.n_zones)]


def batch_moves(batch, q: int):
    """cost_move[C] of query q, or None."""
    m = getattr(batch, "cost_move", None)
    return None if m is None else m[q]


def batch_rounds(batch, q: int):
    """cost_round[C] of query q, or None when inter-stage migrations have one fixed cost."""
    r = getattr(batch, "cost_round", None)
    return None if r is None else r[q]


def run_query(batch, q: int, n_scenarios: Optional[int] = None, n_threads: int = 1, want_plan: bool = True,
              pool_all: bool = False) -> QueryResult:
    """Whole path for query q of a batch object that carries the input arrays."""
    group = int(getattr(batch, "group_size", 1))
    S = batch.n_scenarios if n_scenarios is None else int(n_scenarios)
    zone, weight = batch_zones(batch, q)
    moves = batch_moves(batch, q)
    hists = eval_hist(batch.configs, batch.thr_off, batch.avail[q], int(batch.seed[q]), int(batch.stream_id[q]),
                      0, S, n_threads, pool_all, group, zone, weight, with_occ=moves is not None)
    hi, hm = hists[0], hists[1]
    ho = hists[2] if moves is not None else None
    rounds = batch_rounds(batch, q)
    tab = finalise(batch.configs, batch.thr_off, batch.avail[q], batch.thr[q], batch.cost[q],
                   batch.interval_sec, S, hi, hm, pool_all, group, rounds, moves, ho)
    if not want_plan:
        return QueryResult(hi, hm, tab, None, None, None, float("nan"), ho)
    W_d, W_f = transition(batch.configs, batch.thr_off, batch.avail[q], batch.thr[q], batch.cost[q],
                          batch.interval_sec, S, batch.p_min, int(batch.cur_config[q]), hi, hm, group, rounds, moves, ho)
    return QueryResult(hi, hm, tab, W_d, W_f, dp_f32(W_f), dp_f64(W_d), ho)
