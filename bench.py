#!/usr/bin/env python3
"""Benchmark of the liveput optimizer's hot path on one MI355X.

One step = one pass of the whole path (clear and sample histograms, liveput tables, look-ahead dynamic program
with its input checks, walk back) over one batch of synthetic planning queries whose inputs are already resident
in HBM.  Prints ONE JSON line: the headline workload (the 1024-query what-if sweep unless --workload says
otherwise) and, under "other_workloads", the GPU legs of the other measured shapes.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload sweep|large|medium|small|tiny]
"""
from __future__ import annotations

import argparse
import ctypes as ct
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Plain 32-bit vector ALU peak: 256 compute units x 4 SIMDs x 32 lanes per cycle x 2.4 GHz = 78.6 T lane-op/s,
# i.e. the chip's fp32 vector rate of 157.3 TFLOP/s with a fused multiply-add counted as ONE lane operation.
ALU_PEAK_LANE_OPS = 256 * 4 * 32 * 2.4e9
HBM_PEAK_BYTES = 8e12

# Counters of the sampling kernel per launch from the rocprofv3 --pmc runs summarised under profiles/:
# HBM bytes (FETCH_SIZE and WRITE_SIZE scaled by a plain copy kernel of known size) and executed vector
# instructions (SQ_INSTS_VALU, wave instructions; x 64 = lane operations).  They belong to the sampling kernel's
# sources and launch shape (the files below); once one of them changes the figures are withheld (null) until the
# counters are taken again.
COUNTER_SOURCES = ("device_common.hpp", "eval_kernels.hpp", "eval_launch.hpp")
COUNTER_SOURCE_SHA256 = "2acce2d943f4f1777ecd874a84d9f6c7be181a7fd3ac921350616c60e9b674c1"
COUNTERS = {
    # workload tag: (HBM bytes read, HBM bytes written, SQ_INSTS_VALU)
    "sweep": (20523553, 46566496, 6116129796),
    "large": (5831181, 15271962, 751717061),
    "mediumx256": (10511269, 36863526, 5734618211),
    "largex256": (18611679, 933758758, 312438217035),
    "sweep+pool-all": (28277247, 58024378, 8686218050),
    "sweep+zones3": (22025575, 46375386, 27995753187),
    "sweep+moves": (20538611, 63833370, 7291402457),
    "sweep+weights": (22242043, 46544288, 63678165359),
}


def counter_digest() -> str:
    import hashlib
    digest = hashlib.sha256()
    for name in COUNTER_SOURCES:
        with open(os.path.join(ROOT, "paper_2403_14097_amd", "csrc", name), "rb") as fh:
            digest.update(fh.read())
    return digest.hexdigest()


LIVE_COUNTERS = {}   # workload tag: counters taken in this run (see live_counters)


def kernel_counters(workload_tag: str):
    """(HBM bytes per launch, executed VALU wave-instructions per launch, where they come from) of the sampling
    kernel, or (None, None, None)."""
    if workload_tag in LIVE_COUNTERS:
        read, written, valu = LIVE_COUNTERS[workload_tag]
        return read + written, valu, "rocprofv3 --pmc child runs of this bench run"
    if workload_tag not in COUNTERS or counter_digest() != COUNTER_SOURCE_SHA256:
        return None, None, None
    read, written, valu = COUNTERS[workload_tag]
    return read + written, valu, "rocprofv3 --pmc runs summarised in profiles/ (kernel sources unchanged since)"


def algorithmic_lane_ops(configs, avail, n_scenarios, pool_all=False, zoned=False):
    """Sum over units of S * A(M, k, P): the 32-bit lane operations the method itself needs.

    A(M, k, P) = 33 m + 2 P W + P + W (log2 P + 2) + 10 with M the pool, m = min(k, M - k) random words (25 operations for a
    quarter of a Philox4x32-10 block plus 8 for one step of the subset draw), W = ceil(M / 32) mask words (an
    and + popcount per stage and word, a min per stage, an OR-fold per word for the untouched pipelines) and 10
    for the two histogram updates.  Units whose scenarios all land in one bin (k = 0, k = M, a single stage, or a
    single pipeline) have a closed form and count as zero.
    With zones (non-uniform preemption) a scenario also draws the zone of each of its k departures: one more
    random word (25) and a compare chain over the zones (12) per departure; the subset draws inside the zones
    need at most m words together, which is what is counted.
    Returns (total lane-ops, scenarios of non-trivial units).
    """
    import numpy as np
    D = configs[:, 0].astype(np.int64)
    P = configs[:, 1].astype(np.int64)
    used = D * P
    a_prev = avail[:, :-1, None].astype(np.int64)
    a_next = avail[:, 1:, None].astype(np.int64)
    M = np.broadcast_to(used[None, None, :], a_next.shape[:2] + used.shape)                 # [nq, T, C]
    if pool_all:
        M = np.maximum(M, a_prev)
    k = np.maximum(0, M - a_next)
    m = np.minimum(k, M - k)
    W = (M + 31) // 32
    lg = np.ceil(np.log2(np.maximum(P, 1))).astype(np.int64)[None, None, :]
    Pb = P[None, None, :]
    fixed = 2 * Pb * W + Pb + W * (lg + 2) + 10
    grid_is_pool = M == used[None, None, :]
    sampled = (m > 0) & ~(grid_is_pool & ((P == 1) | (D == 1))[None, None, :])
    A = np.where(sampled, 33 * m + fixed + (37 * k if zoned else 0), 0)
    return float(A.sum()) * n_scenarios, int(sampled.sum()) * n_scenarios


class HipEvents:
    """HIP events through the runtime torch already loaded (timing on the stream the kernels run on)."""

    def __init__(self):
        import torch  # noqa: F401
        self.hip = ct.CDLL("libamdhip64.so.7") if _soname_loaded("libamdhip64.so.7") else ct.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ct.POINTER(ct.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ct.POINTER(ct.c_float), ct.c_void_p, ct.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ct.c_void_p]

    def create(self) -> int:
        ev = ct.c_void_p()
        rc = self.hip.hipEventCreate(ct.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        out = ct.c_float(0)
        rc = self.hip.hipEventElapsedTime(ct.byref(out), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(out.value)

    def destroy(self, ev: int):
        self.hip.hipEventDestroy(ev)


def _soname_loaded(name: str) -> bool:
    try:
        with open("/proc/self/maps") as fh:
            return any(name in line for line in fh)
    except OSError:
        return False


def live_counters(timeout_s: float = 60.0):
    """Counters of the sampling kernel on the headline workload, taken in THIS run: three child processes under
    `rocprofv3 --pmc` (FETCH_SIZE, WRITE_SIZE, SQ_INSTS_VALU; one counter set per run), each a short run of this
    script that also launches a plain elementwise kernel of known size, which scales the two byte counters.
    Must be called before this process touches the GPU (the children are started with fork + exec).
    Returns (bytes read, bytes written, SQ_INSTS_VALU) per launch, or None if anything goes wrong."""
    import csv
    import shutil
    import signal
    import subprocess
    import tempfile
    rocprof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(rocprof):
        return None
    script = os.path.abspath(__file__)
    env = dict(os.environ, TMPDIR="/tmp")
    found = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE", "SQ_INSTS_VALU"):
        out_dir = tempfile.mkdtemp(prefix="parcae_pmc_", dir="/tmp")
        try:
            cmd = [rocprof, "--pmc", counter, "--output-format", "csv", "-d", out_dir, "-o", "x", "--",
                   sys.executable, script, "--counter-child"]
            # a process group of its own, so that a run that does not end can be ended with everything it started
            child = subprocess.Popen(cmd, cwd="/tmp", env=env, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL,
                                     start_new_session=True)
            try:
                child.wait(timeout=timeout_s)
            except subprocess.TimeoutExpired:
                try:
                    os.killpg(child.pid, signal.SIGKILL)
                except OSError:
                    pass
                child.wait()
                return None
            if child.returncode != 0:
                return None
            kernel, copy = [], []
            for root, _dirs, files in os.walk(out_dir):
                for name in files:
                    if not name.endswith("counter_collection.csv"):
                        continue
                    with open(os.path.join(root, name), newline="") as fh:
                        for row in csv.DictReader(fh):
                            if row.get("Counter_Name") != counter:
                                continue
                            if "eval_hist_kernel" in row["Kernel_Name"]:
                                kernel.append(float(row["Counter_Value"]))
                            elif "FunctorOnSelf_add" in row["Kernel_Name"]:
                                copy.append(float(row["Counter_Value"]))
            if not kernel or (counter != "SQ_INSTS_VALU" and not copy):
                return None
            value = sum(kernel) / len(kernel)
            if counter != "SQ_INSTS_VALU":
                # the elementwise kernel reads 1 GiB and writes 1 GiB; the counters are in KiB up to a constant factor
                value = value * (1 << 30) / (sum(copy) / len(copy))
            found[counter] = value
        except (OSError, subprocess.SubprocessError, ValueError, KeyError):
            return None
        finally:
            shutil.rmtree(out_dir, ignore_errors=True)
    return found["FETCH_SIZE"], found["WRITE_SIZE"], found["SQ_INSTS_VALU"]


def measured_copy_bandwidth() -> float:
    """Bytes per second (read + written) of a plain device-to-device copy of 1 GiB: what a streaming kernel reaches
    on this machine, for comparison with the 8 TB/s figure the plan's HBM fraction is quoted against."""
    import torch
    src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda:0")   # written once, so every page is backed
    dst = torch.zeros_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    sec = a.elapsed_time(b) / 5 / 1e3
    del src, dst
    torch.cuda.empty_cache()
    return 2.0 * (1 << 30) / sec


def cpu_baseline(batch, budget_queries: int, pool_all: bool = False, max_threads: int | None = None):
    """The oracle, as it stands, on a bounded sample of the same workload (first queries, all scenarios)."""
    import oracle
    threads = min(oracle.num_threads(), os.cpu_count() or 1)
    if max_threads:
        threads = max(1, min(threads, max_threads))
    nq = min(budget_queries, batch.n_queries)
    units = batch.n_intervals * batch.n_configs
    s_cpu = min(batch.n_scenarios, max(256, int(6e7 * threads // (units * nq))))   # scenario prefix if one query is too big
    t0 = time.perf_counter()
    for q in range(nq):
        oracle.run_query(batch, q, n_scenarios=s_cpu, n_threads=threads, pool_all=pool_all)
    dt = time.perf_counter() - t0
    scen = nq * units * s_cpu
    return {"value": scen / dt, "unit": "evals/s", "cores": threads, "kind": "oracle",
            "sample": f"first {nq} of {batch.n_queries} queries, first {s_cpu} of {batch.n_scenarios} scenarios per "
                      f"unit (the oracle samples every unit, also those the GPU path writes in closed form), "
                      f"sampling + tables + plan, {dt:.2f} s"}


def measure(pk, pi, events, name, steps, warmup, *, dense=False, queries=None, pool_all=False, zones=0, rounds=False,
            weights=False, moves=False, graph=False):
    """GPU legs of one workload: whole steps (wall clock), the sampling kernel and the plan (HIP events recorded by
    the library around them), the plan alone from stored histograms.  Returns (result dict, batch)."""
    import torch
    batch = pi.workload(name, dense=dense, n_queries=queries)
    if zones:
        batch = batch.with_zones(zones)
    if rounds:
        batch = batch.with_rounds()
    if weights:
        batch = batch.with_weights()
    if moves:
        batch = batch.with_moves()
    prob = pk.upload(batch, device="cuda:0")
    if pool_all:
        prob.flags = pk.PARCAE_POOL_ALL
    ev_out = pk.alloc_eval_out(prob)
    pl_out = pk.alloc_plan_out(prob)
    nq, T, C, S = batch.n_queries, batch.n_intervals, batch.n_configs, batch.n_scenarios
    scenarios = nq * T * C * S
    cells = nq * T * C * C
    alg_ops, nontrivial = algorithmic_lane_ops(batch.configs, batch.avail, S, pool_all, zones > 0)

    # whole steps by the wall clock, enqueued back to back, nothing recorded in between
    for _ in range(warmup):
        pk.parcae_liveput_plan(prob, ev_out, pl_out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        pk.parcae_liveput_plan(prob, ev_out, pl_out)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps

    # the same steps once more with the library's events around the sampling kernel and around the plan (an event
    # between two kernels costs a few microseconds of its own, so these steps are not the ones timed above)
    ev_steps = min(steps, 10)
    quads = [tuple(events.create() for _ in range(4)) for _ in range(ev_steps)]
    for i in range(ev_steps):
        prob.profile_events = quads[i]
        pk.parcae_liveput_plan(prob, ev_out, pl_out)
    torch.cuda.synchronize()
    prob.profile_events = None
    kern_s = sum(events.elapsed_ms(q[0], q[1]) for q in quads) / ev_steps / 1e3
    plan_in_step_s = sum(events.elapsed_ms(q[2], q[3]) for q in quads) / ev_steps / 1e3

    # the plan alone, from the histograms already in memory: device time between the library's own events around
    # it, and wall clock per call with the calls enqueued back to back
    reps = max(5, steps)
    for _ in range(2):
        pk.parcae_plan_from_hist(prob, ev_out.hist_int, ev_out.hist_min, pl_out)
    torch.cuda.synchronize()
    pairs = [(events.create(), events.create()) for _ in range(reps)]
    t1 = time.perf_counter()
    for i in range(reps):
        prob.profile_events = (None, None, pairs[i][0], pairs[i][1])
        pk.parcae_plan_from_hist(prob, ev_out.hist_int, ev_out.hist_min, pl_out)
    torch.cuda.synchronize()
    dp_wall_s = (time.perf_counter() - t1) / reps
    prob.profile_events = None
    dp_s = sorted(events.elapsed_ms(a, b) for a, b in pairs)[len(pairs) // 2] / 1e3   # median: a single launch is short
    for q in quads:
        for e in q:
            events.destroy(e)
    for a, b in pairs:
        events.destroy(a)
        events.destroy(b)

    graph_ms = None
    if graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            pk.parcae_liveput_plan(prob, ev_out, pl_out)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            pk.parcae_liveput_plan(prob, ev_out, pl_out)
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t2) / steps * 1e3

    status = pl_out.status.cpu().numpy()
    tag = (batch.name + ("+pool-all" if pool_all else "") + (f"+zones{zones}" if zones else "") +
           ("+rounds" if rounds else "") + ("+weights" if weights else "") + ("+moves" if moves else ""))
    plain = not (dense or pool_all or zones or rounds or weights or moves)
    counter_tag = (batch.name + (f"x{nq}" if queries else "")) if plain else ("" if (dense or queries) else tag)
    traffic, valu_insts, counter_source = kernel_counters(counter_tag)
    achieved = alg_ops / kern_s
    # the plan reads both histograms once and writes F and the back-pointers: its algorithmic HBM bytes
    dp_bytes = nq * T * batch.hist_len * 8 + nq * (T + 1) * C * 4 + nq * T * C * 4
    res = {
        "workload": tag, "n_queries": nq, "n_instances": batch.n_instances, "n_intervals": T, "n_configs": C,
        "n_scenarios": S, "scenarios_per_step": scenarios, "sampled_scenarios_per_step": nontrivial,
        "dp_cells_per_step": cells, "infeasible_queries": int((status != 0).sum()),
        "ms_per_step": dt * 1e3, "sampling_kernel_ms": kern_s * 1e3, "plan_ms_in_step": plan_in_step_s * 1e3,
        "dp_ms": dp_s * 1e3, "dp_wall_ms_per_call": dp_wall_s * 1e3,
        "sampled_evals_per_sec": nontrivial / dt, "all_units_evals_per_sec": scenarios / dt,
        "dp_cells_per_sec": cells / dp_s,
        "roofline": {"bound": "alu", "achieved": achieved / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12,
                     "unit": "T lane-op/s", "frac": achieved / ALU_PEAK_LANE_OPS,
                     "issue_frac": None if valu_insts is None else valu_insts * 64 / kern_s / ALU_PEAK_LANE_OPS,
                     "model_ops": alg_ops, "executed_valu_wave_instructions": valu_insts,
                     # method operations per executed lane operation (above 1: the kernel issues fused forms)
                     "useful_op_efficiency": None if valu_insts is None else alg_ops / (valu_insts * 64.0),
                     "traffic": traffic, "traffic_unit": "bytes per launch (HBM read + written)",
                     "counter_source": counter_source,
                     "kernel": "eval_hist_kernel"},
        # The plan is T dependent steps per query, so it cannot reach a throughput peak; what bounds a batch is the
        # HBM traffic it cannot avoid (histograms read once, F and back-pointers written once).
        "dp_roofline": {"bound": "hbm", "achieved": dp_bytes / dp_s / 1e9, "peak": HBM_PEAK_BYTES / 1e9, "unit": "GB/s",
                        "frac": dp_bytes / dp_s / HBM_PEAK_BYTES, "algorithmic_bytes": dp_bytes,
                        "steps_in_chain": T, "us_per_step": dp_s * 1e6 / T,
                        # latency floor of the chain: T dependent steps at 440 cycles (a step of the wave planner with
                        # every load and scan removed, measured) plus 5 us of launch and set-up, at 2.4 GHz
                        "latency_floor_ms": (T * 440 / 2.4e9 + 5e-6) * 1e3,
                        "measured_over_floor": dp_s / (T * 440 / 2.4e9 + 5e-6),
                        "alu_frac_at_15_ops_per_cell": cells / dp_s * 15 / ALU_PEAK_LANE_OPS},
    }
    if graph_ms is not None:
        res["graph_replay_ms_per_step"] = graph_ms
    del prob, ev_out, pl_out
    torch.cuda.empty_cache()
    return res, batch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="sweep", choices=["tiny", "small", "medium", "large", "sweep"])
    ap.add_argument("--dense", action="store_true", help="keep candidate depths below the memory floor")
    ap.add_argument("--queries", type=int, default=None, help="override the number of queries in the batch")
    ap.add_argument("--pool-all", action="store_true",
                    help="draw preemptions among all available instances (idle ones included) instead of the used ones")
    ap.add_argument("--zones", type=int, default=0,
                    help="spread the instances over this many zones of unequal preemption hazard (0 = uniform)")
    ap.add_argument("--rounds", action="store_true",
                    help="inter-stage migration cost by state-transfer rounds (a per-candidate cost per further round)")
    ap.add_argument("--weights", action="store_true", help="a hazard weight per instance (preemption not uniform)")
    ap.add_argument("--moves", action="store_true",
                    help="inter-stage migration cost per instance that must receive state (third histogram)")
    ap.add_argument("--graph", action="store_true",
                    help="also time replays of a HIP graph that captured one whole call (reported as "
                         "graph_replay_ms_per_step next to the eager figures; the call enqueues kernels only)")
    ap.add_argument("--no-others", action="store_true", help="skip the other measured workloads (other_workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-queries", type=int, default=None, help="queries the CPU baseline runs")
    ap.add_argument("--cpu-threads", type=int, default=None, help="threads the CPU baseline may use (default: all)")
    ap.add_argument("--no-live-counters", action="store_true",
                    help="do not take the sampling kernel's counters in this run (three short rocprofv3 --pmc child "
                         "runs before the measurement); the stored ones are used while the kernel sources match")
    ap.add_argument("--counter-child", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB elementwise copy kernel three times (known traffic, for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU; --gpus N with N > 1 is not supported "
              "(queries would shard across GPUs with no exchange, which this program does not launch)", file=sys.stderr)
        sys.exit(2)

    if args.counter_child:   # a short run of the headline workload under the profiler, with the calibration kernel
        args.steps, args.warmup, args.calibrate_copy = 2, 1, True
        args.no_others = args.no_cpu_baseline = args.no_live_counters = True
    plain_sweep = args.workload == "sweep" and not (args.dense or args.pool_all or args.zones or args.rounds or
                                                    args.weights or args.moves or args.queries)
    if plain_sweep and not args.no_live_counters:
        live = live_counters()   # before anything here touches the GPU
        if live is not None:
            LIVE_COUNTERS["sweep"] = tuple(int(round(v)) for v in live)

    import torch

    import paper_2403_14097_amd as pk
    import parcae_inputs as pi

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    pk.load_library()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")   # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)   # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    events = HipEvents()
    head, batch = measure(pk, pi, events, args.workload, args.steps, args.warmup, dense=args.dense, queries=args.queries,
                          pool_all=args.pool_all, zones=args.zones, rounds=args.rounds, weights=args.weights,
                          moves=args.moves, graph=args.graph)
    out = {
        "metric": "liveput_evals_per_sec",
        # scenarios that go through the sampler and the reducer, per second of the whole step; the units whose
        # scenarios all fall into one bin are written in closed form and are NOT counted here (all_units_evals_per_sec
        # counts them)
        "value": head["sampled_evals_per_sec"],
        "unit": "evals/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32+f32",
        "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "n_queries", "n_instances", "n_intervals", "n_configs", "n_scenarios",
                                        "scenarios_per_step", "sampled_scenarios_per_step", "dp_cells_per_step",
                                        "infeasible_queries")},
        "all_units_evals_per_sec": head["all_units_evals_per_sec"],
        "dp_cells_per_sec": head["dp_cells_per_sec"],
        "dp_ms": head["dp_ms"],
        "dp_wall_ms_per_call": head["dp_wall_ms_per_call"],
        "plan_ms_in_step": head["plan_ms_in_step"],
        "sampling_kernel_ms": head["sampling_kernel_ms"],
        "dp_roofline": head["dp_roofline"],
        "roofline": head["roofline"],
    }
    copy_bps = measured_copy_bandwidth()
    out["dp_roofline"]["measured_copy_GBps"] = copy_bps / 1e9
    out["dp_roofline"]["frac_of_measured_copy"] = out["dp_roofline"]["achieved"] * 1e9 / copy_bps
    out["roofline"]["note"] = (
        "frac = model_ops / kernel time / peak: model_ops is the textbook operation count of the method, the sum over "
        "units of S * A(M, k, P) (see algorithmic_lane_ops); issue_frac = executed vector instructions x 64 lanes / "
        "kernel time / peak, from SQ_INSTS_VALU; traffic from FETCH_SIZE and WRITE_SIZE scaled by an elementwise "
        "kernel of known size; counter_source says whether the counters were taken in this run (three rocprofv3 --pmc "
        "child runs before the measurement) or are the stored ones of profiles/, which are withheld (null) once the "
        "kernel sources change; the kernel issues fused forms (64-bit multiply-add, three-input logic, bit-sliced "
        "counters), so it executes fewer operations than the model counts; peak = 256 CUs x 4 SIMDs x 32 lanes/cycle "
        "x 2.4 GHz, the rate of simple 32-bit vector ops; multiplies, shifts, compares and popcounts issue at half "
        "that rate")
    if "graph_replay_ms_per_step" in head:
        out["graph_replay_ms_per_step"] = head["graph_replay_ms_per_step"]

    if plain_sweep and not args.no_others:
        others = []
        for name, nq, k in (("large", None, 10), ("medium", 256, 5), ("large", 256, 2), ("medium", None, 20)):
            res, _ = measure(pk, pi, events, name, k, 2, queries=nq)
            res["workload"] = name + (f" x {nq} seeds" if nq else "")
            others.append(res)
        out["other_workloads"] = others

    if not args.no_cpu_baseline:
        nq, T, C, S = batch.n_queries, batch.n_intervals, batch.n_configs, batch.n_scenarios
        per_query = T * C * S
        threads_hint = args.cpu_threads or (os.cpu_count() or 1)
        budget = args.cpu_queries or max(1, min(nq, int(6e7 * min(threads_hint, 16) // max(per_query, 1)) or 1))
        out["cpu_baseline"] = cpu_baseline(batch, budget, args.pool_all, args.cpu_threads)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
