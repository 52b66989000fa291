"""Seeded synthetic planning inputs for the liveput optimizer.

This module only *draws inputs* (availability walks, throughput tables,
migration-cost tables, candidate lists, seeds).  It contains none of the
method's arithmetic: no sampling of preemption scenarios, no liveput, no
dynamic program.  Both the CPU oracle's tests and the GPU library's tests and
benchmark import it so that the two sides see byte-identical arrays.

The recipes stand in for the paper's measured inputs, which are not public:
predicted availability of a 32-instance spot cluster (section 9.1, Table 1),
profiled throughputs (appendix C.1) and profiled migration costs (appendix A,
Table 4).  Shapes follow the paper (N = 32 with a 12-interval look-ahead of
one-minute intervals in the "small" workload); magnitudes of the three cost
classes sit inside Table 4's ranges.

Randomness is SplitMix64 (Steele, Lea, Flood 2014), written out here so the
streams do not depend on the numpy version.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence

import numpy as np

BASE_SEED = 0x240314097
MAX_ZONES = 4
_GOLDEN = 0x9E3779B97F4A7C15
_MASK64 = (1 << 64) - 1


def _mix64(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


class SplitMix64:
    """Sequential SplitMix64 stream."""

    def __init__(self, seed: int):
        self.state = seed & _MASK64

    def next_u64(self) -> int:
        self.state = (self.state + _GOLDEN) & _MASK64
        return _mix64(self.state)

    def uniform(self, lo: float, hi: float) -> float:
        u = (self.next_u64() >> 11) * (1.0 / (1 << 53))
        return lo + (hi - lo) * u

    def randint(self, lo: int, hi: int) -> int:
        """Integer in [lo, hi] (inclusive)."""
        return lo + self.next_u64() % (hi - lo + 1)


@dataclass(frozen=True)
class WorkloadSpec:
    """One row of the workload table (sizes, walk and scenario count)."""

    name: str
    n_queries: int
    n_instances: int
    n_intervals: int
    interval_sec: float
    depths: Sequence[int]
    p_min: int
    walk_step: int
    burst_drop: int
    burst_prob: float          # fixed probability, or upper end of U[0, x] if burst_prob_random
    burst_prob_random: bool
    avail_floor: int
    n_scenarios: int


WORKLOADS: Dict[str, WorkloadSpec] = {
    "tiny": WorkloadSpec("tiny", 1, 8, 4, 60.0, (1, 2, 4, 8), 1, 2, 0, 0.0, False, 1, 256),
    "small": WorkloadSpec("small", 1, 32, 12, 60.0, (1, 2, 4, 8, 16), 2, 4, 8, 0.1, False, 2, 4096),
    "medium": WorkloadSpec("medium", 1, 64, 30, 60.0, (1, 2, 4, 8, 16, 32), 4, 6, 16, 0.05, False, 4, 16384),
    "large": WorkloadSpec("large", 1, 256, 60, 30.0, (1, 2, 4, 8, 16, 32, 64), 8, 16, 64, 0.03, False, 8, 65536),
    "sweep": WorkloadSpec("sweep", 1024, 64, 30, 60.0, (1, 2, 4, 8, 16, 32), 4, 6, 16, 0.15, True, 4, 4096),
}
_WORKLOAD_INDEX = {"tiny": 0, "small": 1, "medium": 2, "large": 3, "sweep": 4}


@dataclass
class ProblemBatch:
    """A batch of planning queries that share the candidate list and sizes.

    Arrays (all C-contiguous numpy):
      configs     int32  [C, 2]      (D, P) per candidate, sorted by P then D
      thr_off     int32  [C + 1]     offsets of each candidate's throughput row
      avail       int32  [nq, T + 1] avail[q, 0] = availability now, avail[q, 1 + t] = interval t
      thr         float32 [nq, sum(D+1)] thr[q, thr_off[c] + d] = throughput of d pipelines of depth P_c
      cost        float32 [nq, C, 3] seconds: intra-stage, inter-stage, re-partition
      seed        uint64 [nq]
      stream_id   uint32 [nq]
      cur_config  int32  [nq]        index of the configuration running now, or -1
    group_size > 1: instances of that many GPUs; n_instances and avail then count instances, D * P counts GPUs.
    n_zones > 0: preemption is not uniform; zone uint8 [nq, N] is the zone of every instance,
    zone_weight uint32 [nq, 4] the hazard weight of every zone (entries at and above n_zones unused).
    cost_round float32 [nq, C] (optional): seconds per further state-transfer round of an inter-stage migration.
    inst_weight uint8 [nq, N] (optional): hazard weight (1..255) of every instance, for preemption that is not
    uniform instance by instance.
    cost_move float32 [nq, C] (optional): seconds per instance that must receive state in an inter-stage migration.
    """

    name: str
    n_instances: int
    n_intervals: int
    interval_sec: float
    p_min: int
    n_scenarios: int
    configs: np.ndarray
    thr_off: np.ndarray
    avail: np.ndarray
    thr: np.ndarray
    cost: np.ndarray
    seed: np.ndarray
    stream_id: np.ndarray
    cur_config: np.ndarray
    meta: dict = field(default_factory=dict)
    group_size: int = 1        # GPUs per instance (preempted together); availability counts instances
    n_zones: int = 0           # 0: every instance equally likely to be preempted
    zone: np.ndarray | None = None
    zone_weight: np.ndarray | None = None
    cost_round: np.ndarray | None = None   # float32 [nq, C] seconds per further state-transfer round, or None
    inst_weight: np.ndarray | None = None  # uint8 [nq, N] hazard weight of every instance, or None
    cost_move: np.ndarray | None = None    # float32 [nq, C] seconds per instance that must receive state, or None

    @property
    def n_queries(self) -> int:
        return int(self.avail.shape[0])

    @property
    def n_configs(self) -> int:
        return int(self.configs.shape[0])

    @property
    def hist_len(self) -> int:
        return int(self.thr_off[-1])

    def take(self, queries: Sequence[int]) -> "ProblemBatch":
        """Sub-batch holding the listed queries."""
        idx = np.asarray(list(queries), dtype=np.int64)
        return ProblemBatch(
            self.name, self.n_instances, self.n_intervals, self.interval_sec, self.p_min,
            self.n_scenarios, self.configs, self.thr_off,
            np.ascontiguousarray(self.avail[idx]), np.ascontiguousarray(self.thr[idx]),
            np.ascontiguousarray(self.cost[idx]), np.ascontiguousarray(self.seed[idx]),
            np.ascontiguousarray(self.stream_id[idx]), np.ascontiguousarray(self.cur_config[idx]),
            dict(self.meta), self.group_size, self.n_zones,
            None if self.zone is None else np.ascontiguousarray(self.zone[idx]),
            None if self.zone_weight is None else np.ascontiguousarray(self.zone_weight[idx]),
            None if self.cost_round is None else np.ascontiguousarray(self.cost_round[idx]),
            None if self.inst_weight is None else np.ascontiguousarray(self.inst_weight[idx]),
            None if self.cost_move is None else np.ascontiguousarray(self.cost_move[idx]))

    def with_rounds(self, lo: float = 2.0, hi: float = 8.0, seed: int = 11) -> "ProblemBatch":
        """Same inputs with a per-candidate cost of every further state-transfer round of an inter-stage
        migration, drawn from U[lo, hi] seconds (the state-transfer share of the cost, which section 8.4 and
        appendix A put at up to a minute)."""
        out = self.take(range(self.n_queries))
        rounds = np.zeros((self.n_queries, self.n_configs), dtype=np.float32)
        for q in range(self.n_queries):
            rng = SplitMix64(_mix64(BASE_SEED ^ (seed * 0x9E3779B1 + q)))
            for c in range(self.n_configs):
                rounds[q, c] = np.float32(rng.uniform(lo, hi))
        out.cost_round = rounds
        return out

    def with_weights(self, seed: int = 13, max_weight: int = 8, heavy_share: float = 0.15) -> "ProblemBatch":
        """Same inputs with a hazard weight per instance: most instances draw their weight from U{1..max_weight},
        a share of them (instances on a market about to be reclaimed, say) gets up to sixteen times that, capped
        at 255.  Stand-in for per-instance preemption estimates (section 5.1)."""
        out = self.take(range(self.n_queries))
        nq, N = self.n_queries, self.n_instances
        weight = np.ones((nq, N), dtype=np.uint8)
        for q in range(nq):
            rng = SplitMix64(_mix64(BASE_SEED ^ (seed * 0x2545F491 + q)))
            for j in range(N):
                w = rng.randint(1, max_weight)
                if rng.uniform(0.0, 1.0) < heavy_share:
                    w = min(255, w * rng.randint(2, 16))
                weight[q, j] = w
        out.inst_weight = weight
        out.n_zones, out.zone, out.zone_weight = 0, None, None
        return out

    def with_moves(self, seed: int = 17) -> "ProblemBatch":
        """Same inputs with a per-candidate cost of every instance that must receive state in an inter-stage
        migration (alpha-beta model of section 8.4 with alpha = the inter-stage cost): drawn so that the dearest
        inter-stage migration of the candidate, all stages down to one holder, costs between the inter-stage cost
        and min(interval, re-partition cost)."""
        out = self.take(range(self.n_queries))
        move = np.zeros((self.n_queries, self.n_configs), dtype=np.float32)
        tau = np.float32(self.interval_sec)
        for q in range(self.n_queries):
            rng = SplitMix64(_mix64(BASE_SEED ^ (seed * 0x9E3779B1 + q)))
            for c in range(self.n_configs):
                d, p = int(self.configs[c, 0]), int(self.configs[c, 1])
                worst = (d - 1) * p
                room = float(min(tau, self.cost[q, c, 2])) - float(self.cost[q, c, 1])
                u = rng.uniform(0.0, 0.95)
                move[q, c] = np.float32(u * max(room, 0.0) / worst) if worst > 0 else np.float32(u)
        out.cost_move = move
        out.cost_round = None
        return out

    def with_zones(self, n_zones: int, seed: int = 7, max_weight: int = 8) -> "ProblemBatch":
        """Same inputs with the instances spread over zones of unequal preemption hazard.

        Stand-in for a cluster that spans availability zones or instance types (section 4.1): per query the
        zone shares are drawn from U[0.5, 1.5] and normalised, every instance falls into a zone by those
        shares, and every zone gets an integer weight in [1, max_weight].
        """
        out = self.take(range(self.n_queries))
        nq, N = self.n_queries, self.n_instances
        zone = np.zeros((nq, N), dtype=np.uint8)
        weight = np.ones((nq, MAX_ZONES), dtype=np.uint32)
        for q in range(nq):
            rng = SplitMix64(_mix64(BASE_SEED ^ (seed * 0x1000193 + q)))
            share = np.asarray([rng.uniform(0.5, 1.5) for _ in range(n_zones)])
            edges = np.cumsum(share / share.sum())
            for j in range(N):
                zone[q, j] = min(int(np.searchsorted(edges, rng.uniform(0.0, 1.0), side="right")), n_zones - 1)
            for z in range(n_zones):
                weight[q, z] = rng.randint(1, max_weight)
        out.n_zones, out.zone, out.zone_weight = int(n_zones), zone, weight
        return out

    def with_scenarios(self, n_scenarios: int) -> "ProblemBatch":
        """Same inputs with another scenario count (scenario s never depends on the count)."""
        out = self.take(range(self.n_queries))
        out.n_scenarios = int(n_scenarios)
        return out


def candidate_list(n_instances: int, depths: Sequence[int], p_min: int, feasible_only: bool = True) -> np.ndarray:
    """All (D, P) with P in `depths`, D * P <= N, ordered by P then D.

    feasible_only drops depths below the memory floor p_min; otherwise they are
    kept (the planner treats them as infeasible).
    """
    out: List[tuple] = []
    for p in sorted(set(int(x) for x in depths)):
        if feasible_only and p < p_min:
            continue
        for d in range(1, n_instances // p + 1):
            out.append((d, p))
    return np.asarray(out, dtype=np.int32).reshape(-1, 2)


def throughput_offsets(configs: np.ndarray) -> np.ndarray:
    off = np.zeros(configs.shape[0] + 1, dtype=np.int32)
    np.cumsum(configs[:, 0].astype(np.int64) + 1, out=off[1:])
    return off


def availability_walk(rng: SplitMix64, n: int, t: int, step: int, drop: int, p_drop: float, floor: int) -> np.ndarray:
    """a[0] = N; a[i] = clip(a[i-1] + U{-step..step} - drop * Bernoulli(p_drop), floor, N)."""
    a = np.empty(t + 1, dtype=np.int32)
    a[0] = n
    cur = n
    for i in range(1, t + 1):
        delta = rng.randint(-step, step)
        burst = drop if (rng.uniform(0.0, 1.0) < p_drop) else 0
        cur = min(n, max(floor, cur + delta - burst))
        a[i] = cur
    return a


def throughput_table(configs: np.ndarray, thr_off: np.ndarray, c0: float, c1: float, c2: float) -> np.ndarray:
    """thr(d, P) = d / (c0 / P + c1 + c2 * (P - 1) / P), evaluated in fp32 in this order."""
    f = np.float32
    c0, c1, c2 = f(c0), f(c1), f(c2)
    out = np.zeros(int(thr_off[-1]), dtype=np.float32)
    for c in range(configs.shape[0]):
        d_max, p = int(configs[c, 0]), int(configs[c, 1])
        denom = f(f(f(c0 / f(p)) + c1) + f(f(c2 * f(p - 1)) / f(p)))
        for d in range(d_max + 1):
            out[thr_off[c] + d] = f(f(d) / denom)
    return out


def make_batch(spec: WorkloadSpec, *, dense: bool = False, n_queries: int | None = None,
               n_scenarios: int | None = None, seed: int | None = None) -> ProblemBatch:
    """Draw one batch for a workload row.

    dense=True keeps candidate depths below p_min (planner-infeasible rows that
    make the configuration-by-configuration transition matrix large).
    """
    nq = spec.n_queries if n_queries is None else int(n_queries)
    base = (BASE_SEED + _WORKLOAD_INDEX.get(spec.name, 99)) if seed is None else int(seed)
    configs = candidate_list(spec.n_instances, spec.depths, spec.p_min, feasible_only=not dense)
    thr_off = throughput_offsets(configs)
    n_cfg = configs.shape[0]
    t = spec.n_intervals

    avail = np.empty((nq, t + 1), dtype=np.int32)
    thr = np.empty((nq, int(thr_off[-1])), dtype=np.float32)
    cost = np.empty((nq, n_cfg, 3), dtype=np.float32)
    seeds = np.empty(nq, dtype=np.uint64)
    cur = np.empty(nq, dtype=np.int32)
    p_drops = np.empty(nq, dtype=np.float64)
    for q in range(nq):
        rng = SplitMix64(_mix64(base * 0x100000001B3 + q))
        p_drop = rng.uniform(0.0, spec.burst_prob) if spec.burst_prob_random else spec.burst_prob
        p_drops[q] = p_drop
        avail[q] = availability_walk(rng, spec.n_instances, t, spec.walk_step, spec.burst_drop,
                                     p_drop, spec.avail_floor)
        c0 = rng.uniform(0.5, 1.0)
        c1 = rng.uniform(0.02, 0.05)
        c2 = rng.uniform(0.01, 0.03)
        thr[q] = throughput_table(configs, thr_off, c0, c1, c2)
        for c in range(n_cfg):
            cost[q, c, 0] = rng.uniform(1.0, 3.0)
            cost[q, c, 1] = rng.uniform(5.0, 15.0)
            cost[q, c, 2] = rng.uniform(20.0, 60.0)
        seeds[q] = rng.next_u64()
        # configuration running now: highest-throughput candidate that fits avail[0] and the memory floor
        full = thr[q, thr_off[1:] - 1].astype(np.float64)
        ok = (configs[:, 0] * configs[:, 1] <= avail[q, 0]) & (configs[:, 1] >= spec.p_min)
        cur[q] = int(np.argmax(np.where(ok, full, -1.0))) if ok.any() else -1

    return ProblemBatch(
        name=spec.name + ("-dense" if dense else ""),
        n_instances=spec.n_instances, n_intervals=t, interval_sec=float(spec.interval_sec),
        p_min=spec.p_min, n_scenarios=spec.n_scenarios if n_scenarios is None else int(n_scenarios),
        configs=configs, thr_off=thr_off, avail=avail, thr=thr, cost=cost, seed=seeds,
        stream_id=np.zeros(nq, dtype=np.uint32), cur_config=cur,
        meta={"burst_prob": p_drops, "base_seed": base, "dense": dense})


def workload(name: str, **kw) -> ProblemBatch:
    """Batch for one of the named workloads: tiny, small, medium, large, sweep."""
    return make_batch(WORKLOADS[name], **kw)


def custom_batch(n_instances: int, configs: Sequence[Sequence[int]], avail: Sequence[Sequence[int]],
                 thr_per_pipeline: Sequence[float] | None = None, cost: Sequence[Sequence[float]] | None = None,
                 *, interval_sec: float = 60.0, p_min: int = 1, n_scenarios: int = 256,
                 seed: int = 1, cur_config: int = -1, thr: np.ndarray | None = None,
                 group_size: int = 1) -> ProblemBatch:
    """Hand-built batch for small worked examples.

    thr_per_pipeline[c] gives a linear table thr[c][d] = d * thr_per_pipeline[c]
    unless an explicit flat `thr` is passed.
    """
    cfg = np.asarray(configs, dtype=np.int32).reshape(-1, 2)
    off = throughput_offsets(cfg)
    av = np.atleast_2d(np.asarray(avail, dtype=np.int32))
    nq = av.shape[0]
    if thr is None:
        row = np.zeros(int(off[-1]), dtype=np.float32)
        for c in range(cfg.shape[0]):
            for d in range(int(cfg[c, 0]) + 1):
                row[off[c] + d] = np.float32(d) * np.float32(thr_per_pipeline[c])
        thr_arr = np.tile(row, (nq, 1))
    else:
        thr_arr = np.ascontiguousarray(np.broadcast_to(np.asarray(thr, dtype=np.float32), (nq, int(off[-1]))))
    if cost is None:
        cost_arr = np.tile(np.asarray([2.0, 10.0, 40.0], dtype=np.float32), (nq, cfg.shape[0], 1))
    else:
        cost_arr = np.ascontiguousarray(
            np.broadcast_to(np.asarray(cost, dtype=np.float32).reshape(-1, 3), (nq, cfg.shape[0], 3)))
    seeds = np.asarray([_mix64(seed + i) for i in range(nq)], dtype=np.uint64)
    return ProblemBatch(
        name="custom", n_instances=int(n_instances), n_intervals=av.shape[1] - 1,
        interval_sec=float(interval_sec), p_min=int(p_min), n_scenarios=int(n_scenarios),
        configs=cfg, thr_off=off, avail=np.ascontiguousarray(av), thr=np.ascontiguousarray(thr_arr),
        cost=np.ascontiguousarray(cost_arr), seed=seeds, stream_id=np.zeros(nq, dtype=np.uint32),
        cur_config=np.full(nq, cur_config, dtype=np.int32), group_size=int(group_size))
