// C ABI of the liveput optimizer's hot path: argument checks, workspace layout and kernel launches.
// The semantics of every entry point are stated in include/parcae.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <vector>

#include "../../include/parcae.h"
#include "device_common.hpp"
#include "eval_kernels.hpp"
#include "eval_launch.hpp"
#include "plan_kernels.hpp"
#include "plan_wave.hpp"
#include "replay_kernels.hpp"

namespace {

using parcae::Batch;
using parcae::CfgRec;

constexpr size_t kAlign = 256;
constexpr int kMaxConfigsDp = 4096;
constexpr int kFusedMinQueries = 32;     // fewer queries than this: weights go to memory, steps are spread over the chip
constexpr int kSingleBlockMaxConfigs = 128;  // stepwise DP: up to this many candidates one block per query does all steps
constexpr size_t kMaxBpLds = 16 * 1024;  // back-pointers stay in LDS (16-bit) when they fit in this
constexpr size_t kMaxPlanLds = 60 * 1024;  // dynamic LDS per block, leaves room for the static part within 64 KB
constexpr size_t kLdsPerCu = 160 * 1024;   // LDS of one compute unit
constexpr size_t kPlanStaticLds = 512;     // static LDS of the planning kernel, rounded up
constexpr size_t kMaxPlanBlocksPerCu = 8;  // 32 waves per compute unit / 4 waves per block

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t cfg_off, valid_off, bp_off, queue_off, list_off, w_off, f_off, total;
    bool stepwise;  // few queries: weights are written out and the DP runs on them
    int64_t L;
    int max_row;  // bins of the widest candidate, max over c of D_c + 1
};

// Histogram bins the planning kernels keep in LDS at a time: all of them if they fit, else as many as
// the LDS budget allows; -1 if not even the widest row fits next to the per-candidate tables.
int pick_plan_cap(int C, const Layout& lay, size_t bp16_bytes, bool per_query)
{
    const size_t fixed = parcae::plan_lds_bytes(C, 0, bp16_bytes, per_query);
    if (fixed >= kMaxPlanLds) return -1;
    int64_t cap = (int64_t)((kMaxPlanLds - fixed) / 8);
    if (cap > lay.L) cap = lay.L;
    return cap >= lay.max_row ? (int)cap : -1;
}

// The caller's structure may be older (shorter) or newer (longer) than this library's: copies what both sides know,
// zero-fills the rest.  False if the pointer is null or the size is below the members every release has.
constexpr size_t kMinProblemSize = offsetof(parcae_problem, cost_round) + sizeof(const float*);
bool load_problem(const parcae_problem* in, parcae_problem* out)
{
    if (!in || in->struct_size < kMinProblemSize) return false;
    std::memset(out, 0, sizeof(*out));
    std::memcpy(out, in, in->struct_size < sizeof(*out) ? in->struct_size : sizeof(*out));
    out->struct_size = (uint32_t)sizeof(*out);
    return true;
}

int record(void* event, hipStream_t st)
{
    if (!event) return PARCAE_OK;
    return hipEventRecord(static_cast<hipEvent_t>(event), st) == hipSuccess ? PARCAE_OK : PARCAE_EHIP;
}

// Host-visible shape checks; fills the packed candidate table (table may be null; table_cap = its capacity).
int check_problem(const parcae_problem* p, CfgRec* table, size_t table_cap, Layout* lay)
{
    if (!p || !p->configs || !p->avail || !p->thr || !p->cost || !p->seed) return PARCAE_EINVAL;
    if (p->n_queries < 1 || p->n_intervals < 1 || p->n_configs < 1) return PARCAE_EINVAL;
    if (p->n_instances < 1 || p->n_instances > PARCAE_MAX_INSTANCES) return PARCAE_EINVAL;
    if (p->n_scenarios < 1 || p->n_scenarios > PARCAE_MAX_SCENARIOS) return PARCAE_EINVAL;
    if ((p->flags & ~(uint32_t)PARCAE_POOL_ALL) != 0u) return PARCAE_EINVAL;
    if (!(p->interval_sec > 0.0f) || !std::isfinite(p->interval_sec)) return PARCAE_EINVAL;
    if ((int64_t)p->n_configs * p->n_intervals >= (int64_t)1 << 31) return PARCAE_EINVAL;
    if (p->group_size < 0 || p->group_size > 64) return PARCAE_EINVAL;
    if (p->n_zones < 0 || p->n_zones > PARCAE_MAX_ZONES) return PARCAE_EINVAL;
    if (p->n_zones > 0 && (!p->zone || !p->zone_weight)) return PARCAE_EINVAL;
    if (p->n_zones > 0 && p->inst_weight) return PARCAE_EINVAL;     // zones or a weight per instance, not both
    if (p->cost_move && (p->cost_round || !p->hist_occ)) return PARCAE_EINVAL;
    const int group = p->group_size > 1 ? p->group_size : 1;
    int64_t L = 0;
    int max_row = 0;
    if (table && (size_t)p->n_configs > table_cap) return PARCAE_EINVAL;
    for (int c = 0; c < p->n_configs; ++c) {
        const parcae_config g = p->configs[c];
        if (g.D < 1 || g.P < 1 || g.D > PARCAE_MAX_INSTANCES || g.D % group != 0) return PARCAE_EINVAL;
        if ((int64_t)(g.D / group) * g.P > p->n_instances) return PARCAE_EINVAL;
        if (c > 0) {
            const parcae_config h = p->configs[c - 1];
            if (!(h.P < g.P || (h.P == g.P && h.D < g.D))) return PARCAE_EINVAL;  // strictly increasing (P, D)
        }
        if (table) {
            int lg = -1;
            if ((g.P & (g.P - 1)) == 0) {
                lg = 0;
                while ((1 << lg) < g.P) ++lg;
            }
            table[c] = CfgRec{g.D, g.P, (int32_t)L, lg};
        }
        L += g.D + 1;
        max_row = g.D + 1 > max_row ? g.D + 1 : max_row;
    }
    if ((int64_t)p->n_queries * p->n_intervals * L >= (int64_t)1 << 40) return PARCAE_EINVAL;
    if (p->cost_move) {  // a bin of the stage-occupancy statistic counts up to S * P stages
        int max_depth = 0;
        for (int c = 0; c < p->n_configs; ++c) max_depth = p->configs[c].P > max_depth ? p->configs[c].P : max_depth;
        if ((int64_t)p->n_scenarios * max_depth >= (int64_t)1 << 32) return PARCAE_EINVAL;
    }
    if (lay) {
        lay->L = L;
        lay->max_row = max_row;
        lay->cfg_off = 0;
        lay->valid_off = align_up(sizeof(CfgRec) * (size_t)p->n_configs);
        lay->bp_off = lay->valid_off + align_up(sizeof(int32_t) * (size_t)p->n_queries);
        const size_t n_units = (size_t)p->n_queries * (size_t)p->n_intervals * (size_t)p->n_configs;
        lay->queue_off = lay->bp_off + align_up(sizeof(int32_t) * n_units);
        lay->list_off = lay->queue_off + kAlign * (1 + parcae::kQueueShards);  // item count, then one line per shard counter
        lay->w_off = lay->list_off + align_up(sizeof(uint32_t) * n_units);
        // the per-query planner needs more LDS per candidate; where it does not fit the weights go through memory
        // (and with a cost per moved instance the weights always go through memory)
        lay->stepwise = p->n_queries < kFusedMinQueries || pick_plan_cap(p->n_configs, *lay, 0, true) < 0 ||
                        p->cost_move != nullptr;
        const size_t w_bytes = lay->stepwise ? sizeof(float) * n_units * (size_t)p->n_configs : 0;
        const size_t f_bytes =
            lay->stepwise ? sizeof(float) * (size_t)p->n_queries * ((size_t)p->n_intervals + 1) * (size_t)p->n_configs : 0;
        lay->f_off = lay->w_off + align_up(w_bytes);
        lay->total = lay->f_off + align_up(f_bytes);
    }
    return PARCAE_OK;
}

int check_problem(const parcae_problem* p, std::vector<CfgRec>* table, Layout* lay)
{
    if (!table) return check_problem(p, nullptr, 0, lay);
    if (p && p->n_configs >= 1) table->resize((size_t)p->n_configs);
    return check_problem(p, table->data(), table->size(), lay);
}

int check_workspace(const Layout& lay, const void* ws, size_t bytes)
{
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0 || bytes < lay.total) return PARCAE_EWORKSPACE;
    return PARCAE_OK;
}

Batch make_batch(const parcae_problem* p, const Layout& lay, void* ws)
{
    Batch b;
    b.nq = p->n_queries; b.N = p->n_instances; b.T = p->n_intervals; b.C = p->n_configs; b.S = p->n_scenarios;
    b.p_min = p->p_min; b.L = (int32_t)lay.L; b.tau = p->interval_sec;
    b.pool_all = (p->flags & PARCAE_POOL_ALL) ? 1 : 0;
    b.group = p->group_size > 1 ? p->group_size : 1;
    b.avail_stride = p->n_intervals + 1;
    b.stream_offset = 0u;
    b.cfg = reinterpret_cast<const CfgRec*>(static_cast<unsigned char*>(ws) + lay.cfg_off);
    b.avail = p->avail; b.thr = p->thr; b.cost = p->cost; b.seed = p->seed; b.stream_id = p->stream_id;
    b.cur_config = p->cur_config;
    b.n_zones = p->n_zones; b.zone = p->zone; b.zone_weight = p->zone_weight;
    b.cost_round = p->cost_round;
    b.inst_weight = p->inst_weight;
    b.cost_move = p->cost_move;
    b.hist_occ = p->cost_move ? p->hist_occ : nullptr;
    return b;
}

// The candidate table reaches the device as kernel arguments, a slice at a time: no host-to-device
// copy is enqueued, so the host vector may go away as soon as the launches are made.
constexpr int kTableSlice = 120;
struct TableSlice {
    CfgRec rec[kTableSlice];
};

__global__ void __launch_bounds__(128) table_slice_kernel(TableSlice slice, int count, CfgRec* __restrict__ dst)
{
    const int i = threadIdx.x;
    if (i < count) dst[i] = slice.rec[i];
}

// Writes the candidate table into the workspace.
int write_table(const CfgRec* table, size_t table_len, const Layout& lay, void* ws, hipStream_t st)
{
    CfgRec* dst = reinterpret_cast<CfgRec*>(static_cast<unsigned char*>(ws) + lay.cfg_off);
    for (size_t first = 0; first < table_len; first += kTableSlice) {
        TableSlice slice;
        const int count = (int)((table_len - first < (size_t)kTableSlice) ? table_len - first : kTableSlice);
        std::memcpy(slice.rec, table + first, sizeof(CfgRec) * (size_t)count);
        if (count < kTableSlice) std::memset(slice.rec + count, 0, sizeof(CfgRec) * (size_t)(kTableSlice - count));
        table_slice_kernel<<<dim3(1), dim3(128), 0, st>>>(slice, count, dst + first);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    }
    return PARCAE_OK;
}

// Checks the device inputs of every query (valid[q] in the workspace; needs the table in the workspace).
int check_inputs(const Layout& lay, const Batch& b, void* ws, hipStream_t st)
{
    int32_t* valid = reinterpret_cast<int32_t*>(static_cast<unsigned char*>(ws) + lay.valid_off);
    parcae::validate_kernel<<<dim3((unsigned)b.nq), dim3(256), 0, st>>>(b, valid);
    return hipGetLastError() == hipSuccess ? PARCAE_OK : PARCAE_EHIP;
}

// Table into the workspace and, if asked, the input check (the wave planner checks its own query and needs none).
int stage_inputs(const CfgRec* table, size_t table_len, const Layout& lay, const Batch& b, void* ws, hipStream_t st,
                 bool validate = true)
{
    const int rc = write_table(table, table_len, lay, ws, st);
    if (rc != PARCAE_OK || !validate) return rc;
    return check_inputs(lay, b, ws, st);
}

int stage_inputs(const std::vector<CfgRec>& table, const Layout& lay, const Batch& b, void* ws, hipStream_t st,
                 bool validate = true)
{
    return stage_inputs(table.data(), table.size(), lay, b, ws, st, validate);
}

int32_t* valid_ptr(const Layout& lay, void* ws)
{
    return reinterpret_cast<int32_t*>(static_cast<unsigned char*>(ws) + lay.valid_off);
}

// Bytes of a 16-bit copy of the back-pointers of one query if it is small enough to live in LDS, else 0.
size_t bp16_bytes_for(int T, int C)
{
    const size_t need = sizeof(uint16_t) * (size_t)T * (size_t)C;
    return need <= kMaxBpLds ? need : 0;
}

parcae::WorkQueue make_queue(const Layout& lay, void* ws)
{
    unsigned char* base = static_cast<unsigned char*>(ws);
    parcae::WorkQueue wq;
    wq.count = reinterpret_cast<uint32_t*>(base + lay.queue_off);
    wq.next = wq.count + kAlign / sizeof(uint32_t);
    wq.list = reinterpret_cast<uint32_t*>(base + lay.list_off);
    return wq;
}

// What a call of launch_eval does besides the sampling itself.
struct EvalOpts {
    const CfgRec* table = nullptr;  // host copy of the candidate table if the workspace does not hold it yet
    bool validate = false;          // with `table`: check the device inputs of every query once the table is in place
    bool tables_later = false;      // the liveput tables are written by a kernel the caller launches afterwards
};

int launch_eval(const parcae_problem* p, const Batch& b, const Layout& lay, void* ws, uint32_t* hist_int,
                uint32_t* hist_min, float* liveput, float* teff, float* gain, int32_t* status, hipStream_t st,
                const EvalOpts& opts = EvalOpts())
{
    const int64_t n_units = (int64_t)b.nq * b.T * b.C;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return PARCAE_EHIP;
    const bool moves = b.cost_move != nullptr;
    const bool wide = b.inst_weight || b.n_zones > 0;  // the variants with the larger register budget
    const int resident_waves = cus * (wide ? parcae::kEvalWavesPerCuWide : parcae::kEvalWavesPerCu);
    const int64_t max_items = parcae::max_eval_items(n_units, b.S, resident_waves);
    if (max_items >= (int64_t)1 << 31) return PARCAE_EINVAL;  // leaves room for the queue counters to overshoot
    const parcae::WorkQueue wq = make_queue(lay, ws);

    // a small problem whose table still has to reach the workspace: table, histogram rows and work list in one launch
    const bool one_launch = opts.table && b.C <= parcae::kStageMaxConfigs && n_units <= parcae::kStageMaxUnits &&
                            (int64_t)b.nq * b.T * b.L <= parcae::kStageMaxBins;
    if (one_launch) {
        parcae::StageTable tab;
        std::memcpy(tab.rec, opts.table, sizeof(CfgRec) * (size_t)b.C);
        if (b.C < parcae::kStageMaxConfigs)
            std::memset(tab.rec + b.C, 0, sizeof(CfgRec) * (size_t)(parcae::kStageMaxConfigs - b.C));
        parcae::stage_small_kernel<<<dim3(1), dim3(parcae::kStageThreads), 0, st>>>(
            b, tab, reinterpret_cast<CfgRec*>(static_cast<unsigned char*>(ws) + lay.cfg_off), wq, hist_int, hist_min);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    } else if (opts.table) {
        const int rc = write_table(opts.table, (size_t)b.C, lay, ws, st);
        if (rc != PARCAE_OK) return rc;
    }
    if (opts.table && opts.validate) {
        const int rc = check_inputs(lay, b, ws, st);
        if (rc != PARCAE_OK) return rc;
    }
    if (!one_launch) {
        const int64_t elems = (int64_t)b.nq * b.T * b.L;
        int64_t prep_blocks = (elems + 255) / 256;
        if (prep_blocks > 65536) prep_blocks = 65536;
        parcae::prep_hist_kernel<<<dim3((unsigned)prep_blocks), dim3(256), 0, st>>>(b, wq, hist_int, hist_min);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
        parcae::build_work_kernel<<<dim3((unsigned)((n_units + parcae::kBuildThreads - 1) / parcae::kBuildThreads)),
                                    dim3(parcae::kBuildThreads), 0, st>>>(b, wq);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    }

    const int64_t eval_blocks = parcae::eval_grid_blocks(cus, max_items);
    if (p->profile && record(p->profile->event_before_sampling, st) != PARCAE_OK) return PARCAE_EHIP;
    const dim3 grid((unsigned)eval_blocks), block(parcae::kEvalThreads);
    if (b.inst_weight) {
        if (moves) parcae::eval_hist_kernel<parcae::kDrawWeighted, true><<<grid, block, 0, st>>>(b, wq, resident_waves, hist_int, hist_min);
        else parcae::eval_hist_kernel<parcae::kDrawWeighted, false><<<grid, block, 0, st>>>(b, wq, resident_waves, hist_int, hist_min);
    } else if (b.n_zones > 0) {
        if (moves) parcae::eval_hist_kernel<parcae::kDrawZoned, true><<<grid, block, 0, st>>>(b, wq, resident_waves, hist_int, hist_min);
        else parcae::eval_hist_kernel<parcae::kDrawZoned, false><<<grid, block, 0, st>>>(b, wq, resident_waves, hist_int, hist_min);
    } else {
        if (moves) parcae::eval_hist_kernel<parcae::kDrawUniform, true><<<grid, block, 0, st>>>(b, wq, resident_waves, hist_int, hist_min);
        else parcae::eval_hist_kernel<parcae::kDrawUniform, false><<<grid, block, 0, st>>>(b, wq, resident_waves, hist_int, hist_min);
    }
    if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    if (p->profile && record(p->profile->event_after_sampling, st) != PARCAE_OK) return PARCAE_EHIP;

    if ((liveput || teff || gain) && !opts.tables_later) {
        parcae::finalise_kernel<<<dim3((unsigned)((n_units + 255) / 256)), dim3(256), 0, st>>>(b, hist_int, hist_min,
                                                                                                 liveput, teff, gain);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    }
    if (status) {
        parcae::status_from_valid_kernel<<<dim3((unsigned)((b.nq + 255) / 256)), dim3(256), 0, st>>>(
            b.nq, valid_ptr(lay, ws), status, PARCAE_EINVAL);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    }
    return PARCAE_OK;
}

// The DP on weights held in memory.  F_scratch is used when the caller wants no F and the stepwise kernels need one.
int launch_dp(const float* W, int nq, int T, int C, const int32_t* valid, float* F, float* F_scratch, int32_t* bp,
              int32_t* plan, int32_t* start, float* objective, int32_t* status, hipStream_t st)
{
    const bool spread = C > kSingleBlockMaxConfigs && nq < kFusedMinQueries && (F || F_scratch) && bp;
    if (!spread) {
        const size_t b16 = bp16_bytes_for(T, C);
        const size_t lds = parcae::dp_lds_bytes(C, b16);
        parcae::dp_kernel<<<dim3((unsigned)nq), dim3(parcae::kPlanThreads), lds, st>>>(
            W, T, C, b16 ? 1 : 0, valid, F, bp, plan, start, objective, status, PARCAE_EINVAL, PARCAE_EINFEASIBLE);
        return hipGetLastError() == hipSuccess ? PARCAE_OK : PARCAE_EHIP;
    }
    float* F_use = F ? F : F_scratch;
    for (int t = 0; t < T; ++t) {
        parcae::dp_step_kernel<<<dim3((unsigned)((C + parcae::kStepCols - 1) / parcae::kStepCols), (unsigned)nq),
                                 dim3(parcae::kPlanThreads), sizeof(float) * (size_t)C, st>>>(W, T, C, t, F_use, bp);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    }
    parcae::dp_finish_kernel<<<dim3((unsigned)((nq + 63) / 64)), dim3(64), 0, st>>>(
        nq, T, C, valid, F_use, bp, plan, start, objective, status, PARCAE_EINVAL, PARCAE_EINFEASIBLE);
    return hipGetLastError() == hipSuccess ? PARCAE_OK : PARCAE_EHIP;
}

// Launch shape of the wave planner (candidate lists of at most 64 entries): threads per query, steps per chunk,
// whether the 16-bit back-pointers of all steps stay in local memory.  False if the problem does not fit.
struct WaveLaunch {
    int threads, steps_per_chunk, bp_in_lds;
    size_t lds;
};

bool pick_wave_launch(int nq, int T, int C, int64_t L, const parcae::WaveGeom& g, int cus, bool packed, WaveLaunch* out)
{
    // A handful of queries with long candidate lists: one workgroup per query leaves the chip empty while it works
    // through the weights and back-pointers of every step, and writing the weights out with a workgroup per
    // (query, step) is quicker (measured: one query of 60 candidates and 60 steps 0.23 ms here, 0.14 ms there).
    if (nq < kFusedMinQueries && C > 32) return false;
    // four waves per query share the work that is parallel (weights, back-pointers) and hide each other's waits on
    // local memory; very large batches take two, a handful of queries eight
    int threads = nq >= 8 * cus ? 128 : (nq > cus ? 256 : 512);
    while ((int64_t)parcae::kWaveRowRegs * threads < L && threads < 512) threads *= 2;  // a step's rows must fit the prefetch registers
    if ((int64_t)parcae::kWaveRowRegs * threads < L) return false;
    int resident = (nq + cus - 1) / cus;  // workgroups that should share a compute unit
    resident = resident < 1 ? 1 : (resident > 8 ? 8 : resident);
    const size_t budget = std::min(kMaxPlanLds, kLdsPerCu / (size_t)resident - kPlanStaticLds);
    const size_t per_step = parcae::wave_step_lds(C, (int)L, g, packed);
    for (int attempt = 0; attempt < 4; ++attempt) {
        const bool bp16 = (attempt & 1) == 0 && bp16_bytes_for(T, C) != 0;
        const size_t room = attempt < 2 ? budget : kMaxPlanLds;
        const size_t fixed = parcae::wave_fixed_lds(C, T, g, bp16);
        if (fixed + per_step > room) continue;
        int64_t tc = (int64_t)((room - fixed) / per_step);
        const int64_t by_regs = (int64_t)parcae::kWaveRowRegs * threads / L;
        tc = std::min(std::min(tc, (int64_t)32), std::min(by_regs, (int64_t)T));  // one bit per step of a chunk in a 32-bit mask
        if (tc < 1) continue;
        // the back-pointers of a chunk are one item per (step, candidate) and thread: a chunk that needs one more
        // round of the workgroup for a few items is cut back to whole rounds if that costs no further chunk
        const int64_t rounds = tc * C / threads;
        if (rounds >= 1 && tc * C > rounds * threads) {
            const int64_t fit = rounds * threads / C;
            if (fit >= 1 && (T + fit - 1) / fit == (T + tc - 1) / tc) tc = fit;
        }
        out->threads = threads;
        out->steps_per_chunk = (int)tc;
        out->bp_in_lds = bp16 ? 1 : 0;
        out->lds = fixed + (size_t)tc * per_step;
        return true;
    }
    return false;
}

int compute_units(int* cus)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || *cus < 1)
        return PARCAE_EHIP;
    return PARCAE_OK;
}

// Whether the wave planner keeps the two tails of a bin in one word: every count has to stay below 2^16, and the
// weights by transfer rounds read the tails one histogram at a time.
bool wave_tails_packed(int n_scenarios, const float* cost_round) { return n_scenarios < 65536 && !cost_round; }

// Whether the plan of this problem goes to the wave planner (which checks the device inputs itself).
bool takes_wave_planner(const parcae_problem* p, const CfgRec* table, const Layout& lay)
{
    int cus = 0;
    if (p->n_configs > parcae::kWaveMaxConfigs || p->cost_move || compute_units(&cus) != PARCAE_OK) return false;
    WaveLaunch wl;
    return pick_wave_launch(p->n_queries, p->n_intervals, p->n_configs, lay.L,
                            parcae::wave_geometry(table, p->n_configs), cus, wave_tails_packed(p->n_scenarios, p->cost_round),
                            &wl);
}

int launch_plan_kernels(const Batch& b, const CfgRec* table, const Layout& lay, void* ws, const uint32_t* hist_int,
                        const uint32_t* hist_min, float* F, int32_t* bp, int32_t* plan, int32_t* start,
                        float* objective, int32_t* status, hipStream_t st, const parcae::TablesOut& tables);

// The dynamic program, bracketed by the caller's profiling events if there are any.  `tables` (liveput tables to
// write in the same launch) may be given only where takes_wave_planner() holds.
int launch_plan(const Batch& b, const CfgRec* table, const Layout& lay, void* ws, const uint32_t* hist_int,
                const uint32_t* hist_min, float* F, int32_t* bp, int32_t* plan, int32_t* start, float* objective,
                int32_t* status, hipStream_t st, const parcae_profile* prof = nullptr,
                const parcae::TablesOut& tables = parcae::TablesOut{nullptr, nullptr, nullptr})
{
    if (prof && record(prof->event_before_plan, st) != PARCAE_OK) return PARCAE_EHIP;
    const int rc =
        launch_plan_kernels(b, table, lay, ws, hist_int, hist_min, F, bp, plan, start, objective, status, st, tables);
    if (rc != PARCAE_OK) return rc;
    return prof ? record(prof->event_after_plan, st) : PARCAE_OK;
}

int launch_plan_kernels(const Batch& b, const CfgRec* table, const Layout& lay, void* ws, const uint32_t* hist_int,
                        const uint32_t* hist_min, float* F, int32_t* bp, int32_t* plan, int32_t* start,
                        float* objective, int32_t* status, hipStream_t st, const parcae::TablesOut& tables)
{
    const bool with_tables = tables.liveput || tables.teff || tables.gain;
    unsigned char* base = static_cast<unsigned char*>(ws);
    int32_t* bp_use = bp ? bp : reinterpret_cast<int32_t*>(base + lay.bp_off);
    if (b.C <= parcae::kWaveMaxConfigs && !b.cost_move) {
        int cus = 0;
        if (compute_units(&cus) != PARCAE_OK) return PARCAE_EHIP;
        const parcae::WaveGeom g = parcae::wave_geometry(table, b.C);
        WaveLaunch wl;
        const bool packed = wave_tails_packed(b.S, b.cost_round);
        if (pick_wave_launch(b.nq, b.T, b.C, lay.L, g, cus, packed, &wl)) {
            parcae::WaveTable wt;
            parcae::wave_fill_table(table, b.C, wt);
            // back-pointers that do not stay in local memory are walked through memory: the caller's, else the workspace's
            int32_t* bp_arg = wl.bp_in_lds ? bp : bp_use;
            // workgroups past the last query write the liveput tables, a thread per unit
            const int64_t n_units = (int64_t)b.nq * b.T * b.C;
            const int64_t table_blocks = with_tables ? (n_units + wl.threads - 1) / wl.threads : 0;
            const dim3 grid((unsigned)(b.nq + table_blocks)), block((unsigned)wl.threads);
            if (b.cost_round)
                parcae::plan_wave_kernel<true, false><<<grid, block, wl.lds, st>>>(
                    b, wt, g, wl.steps_per_chunk, wl.bp_in_lds, hist_int, hist_min, F, bp_arg, plan, start, objective,
                    status, PARCAE_EINVAL, PARCAE_EINFEASIBLE, tables);
            else if (packed)
                parcae::plan_wave_kernel<false, true><<<grid, block, wl.lds, st>>>(
                    b, wt, g, wl.steps_per_chunk, wl.bp_in_lds, hist_int, hist_min, F, bp_arg, plan, start, objective,
                    status, PARCAE_EINVAL, PARCAE_EINFEASIBLE, tables);
            else
                parcae::plan_wave_kernel<false, false><<<grid, block, wl.lds, st>>>(
                    b, wt, g, wl.steps_per_chunk, wl.bp_in_lds, hist_int, hist_min, F, bp_arg, plan, start, objective,
                    status, PARCAE_EINVAL, PARCAE_EINFEASIBLE, tables);
            return hipGetLastError() == hipSuccess ? PARCAE_OK : PARCAE_EHIP;
        }
    }
    if (with_tables) return PARCAE_EINVAL;  // only the wave planner writes them
    if (lay.stepwise) {
        // few queries: every (query, step) writes its weights in parallel, then the DP runs on them
        const int cap = pick_plan_cap(b.C, lay, 0, false);
        if (cap < 0 || b.C > kMaxConfigsDp) return PARCAE_EINVAL;
        float* W = reinterpret_cast<float*>(base + lay.w_off);
        parcae::transition_kernel<<<dim3((unsigned)(b.nq * b.T)), dim3(parcae::kPlanThreads),
                                    parcae::plan_lds_bytes(b.C, cap, 0, false), st>>>(b, cap, hist_int, hist_min, W);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
        return launch_dp(W, b.nq, b.T, b.C, valid_ptr(lay, ws), F, reinterpret_cast<float*>(base + lay.f_off), bp_use,
                         plan, start, objective, status, st);
    }
    const size_t b16 = bp16_bytes_for(b.T, b.C);
    int cap = pick_plan_cap(b.C, lay, b16, true);
    size_t b16_use = b16;
    if (cap < 0) {  // no room for the LDS copy of the back-pointers: walk back through memory instead
        b16_use = 0;
        cap = pick_plan_cap(b.C, lay, 0, true);
    }
    if (cap < 0) return PARCAE_EINVAL;
    // small problems keep the histogram rows of every step in LDS (no memory access inside the chain of steps)
    const int64_t all_bins = (int64_t)b.T * lay.L;
    // ... as long as all queries still run at once: with more blocks than the chip holds at that LDS size, smaller
    // blocks that stream their rows finish sooner (measured crossover: 512 against 1024 queries of the sweep shape)
    const size_t resident_bytes = parcae::plan_lds_bytes(b.C, 0, b16_use, true) + 8 * (size_t)all_bins;
    bool resident = resident_bytes <= kMaxPlanLds;
    if (resident) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            return PARCAE_EHIP;
        size_t per_cu = kLdsPerCu / (resident_bytes + kPlanStaticLds);
        if (per_cu > kMaxPlanBlocksPerCu) per_cu = kMaxPlanBlocksPerCu;
        resident = (size_t)b.nq <= per_cu * (size_t)cus;
    }
    if (resident) cap = (int)all_bins;
    parcae::plan_fused_kernel<<<dim3((unsigned)b.nq), dim3(parcae::kPlanThreads),
                                parcae::plan_lds_bytes(b.C, cap, b16_use, true), st>>>(
        b, cap, b16_use ? 1 : 0, resident ? 1 : 0, hist_int, hist_min, valid_ptr(lay, ws), F, bp_use, plan, start,
        objective, status, PARCAE_EINVAL, PARCAE_EINFEASIBLE);
    return hipGetLastError() == hipSuccess ? PARCAE_OK : PARCAE_EHIP;
}

// Whether the planning kernels can take this problem (LDS budget, candidate limit of the stepwise path).
bool plan_fits(const parcae_problem* p, const Layout& lay)
{
    if (lay.stepwise && p->n_configs > kMaxConfigsDp) return false;
    return pick_plan_cap(p->n_configs, lay, 0, !lay.stepwise) >= 0;
}

// ---- workspace of the entry point that allocates nothing: one array per GPU, held until the process ends.
// `scratch` is only a host-side handle here; its device address on the current GPU comes from
// hipGetSymbolAddress, once per device, and is what every kernel and every pointer computation uses.
static __device__ __align__(256) unsigned char scratch[PARCAE_STATIC_WORKSPACE_BYTES];

constexpr int kMaxStaticDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxStaticDevices];

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxStaticDevices) return PARCAE_EHIP;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PARCAE_EHIP;
        if ((reinterpret_cast<uintptr_t>(ptr) % kAlign) != 0) return PARCAE_EHIP;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // every thread would store the same address
    }
    *out = ptr;
    return PARCAE_OK;
}

}  // namespace

extern "C" {

int parcae_version(void) { return 200; }

const char* parcae_strerror(int code)
{
    switch (code) {
        case PARCAE_OK: return "ok";
        case PARCAE_EINVAL: return "invalid argument or input data";
        case PARCAE_EWORKSPACE: return "workspace missing, misaligned or too small";
        case PARCAE_EHIP: return "HIP call or kernel launch failed";
        case PARCAE_EINFEASIBLE: return "no feasible configuration sequence";
        default: return "unknown parcae error code";
    }
}

int64_t parcae_hist_len(const parcae_config* configs, int32_t n_configs)
{
    if (!configs || n_configs < 1) return PARCAE_EINVAL;
    int64_t L = 0;
    for (int c = 0; c < n_configs; ++c) {
        if (configs[c].D < 1 || configs[c].D > PARCAE_MAX_INSTANCES) return PARCAE_EINVAL;
        L += configs[c].D + 1;
    }
    return L;
}

int parcae_workspace_bytes(const parcae_problem* problem, size_t* bytes)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    if (!bytes) return PARCAE_EINVAL;
    Layout lay;
    const int rc = check_problem(p, nullptr, &lay);
    if (rc != PARCAE_OK) return rc;
    *bytes = lay.total;
    return PARCAE_OK;
}

int parcae_liveput_eval(const parcae_problem* problem, uint32_t* hist_int, uint32_t* hist_min, float* liveput, float* teff,
                        float* gain, int32_t* status, void* workspace, size_t workspace_bytes, void* stream)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    std::vector<CfgRec> table;
    Layout lay;
    int rc = check_problem(p, &table, &lay);
    if (rc != PARCAE_OK) return rc;
    if (!hist_int || !hist_min) return PARCAE_EINVAL;
    if ((rc = check_workspace(lay, workspace, workspace_bytes)) != PARCAE_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Batch b = make_batch(p, lay, workspace);
    EvalOpts opts;
    opts.table = table.data();
    opts.validate = true;
    return launch_eval(p, b, lay, workspace, hist_int, hist_min, liveput, teff, gain, status, st, opts);
}

int parcae_plan_from_hist(const parcae_problem* problem, const uint32_t* hist_int, const uint32_t* hist_min, float* F,
                          int32_t* bp, int32_t* plan, int32_t* start, float* objective, int32_t* status,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    std::vector<CfgRec> table;
    Layout lay;
    int rc = check_problem(p, &table, &lay);
    if (rc != PARCAE_OK) return rc;
    if (!hist_int || !hist_min || !plan) return PARCAE_EINVAL;
    if ((rc = check_workspace(lay, workspace, workspace_bytes)) != PARCAE_OK) return rc;
    if (!plan_fits(p, lay)) return PARCAE_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Batch b = make_batch(p, lay, workspace);
    // the wave planner takes the candidate table as a kernel argument and checks the inputs itself: one launch
    if (!takes_wave_planner(p, table.data(), lay) && (rc = stage_inputs(table, lay, b, workspace, st)) != PARCAE_OK)
        return rc;
    return launch_plan(b, table.data(), lay, workspace, hist_int, hist_min, F, bp, plan, start, objective, status, st,
                       p->profile);
}

int parcae_liveput_plan(const parcae_problem* problem, uint32_t* hist_int, uint32_t* hist_min, float* liveput, float* teff,
                        float* gain, float* F, int32_t* bp, int32_t* plan, int32_t* start, float* objective,
                        int32_t* status, void* workspace, size_t workspace_bytes, void* stream)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    std::vector<CfgRec> table;
    Layout lay;
    int rc = check_problem(p, &table, &lay);
    if (rc != PARCAE_OK) return rc;
    if (!hist_int || !hist_min || !plan) return PARCAE_EINVAL;
    if ((rc = check_workspace(lay, workspace, workspace_bytes)) != PARCAE_OK) return rc;
    if (!plan_fits(p, lay)) return PARCAE_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Batch b = make_batch(p, lay, workspace);
    // with the wave planner the input check and the liveput tables are part of the planner's launch
    const bool wave = takes_wave_planner(p, table.data(), lay);
    EvalOpts opts;
    opts.table = table.data();
    opts.validate = !wave;
    opts.tables_later = wave;
    if ((rc = launch_eval(p, b, lay, workspace, hist_int, hist_min, liveput, teff, gain, nullptr, st, opts)) != PARCAE_OK)
        return rc;
    const parcae::TablesOut tables = wave ? parcae::TablesOut{liveput, teff, gain} : parcae::TablesOut{nullptr, nullptr, nullptr};
    return launch_plan(b, table.data(), lay, workspace, hist_int, hist_min, F, bp, plan, start, objective, status, st,
                       p->profile, tables);
}

int parcae_liveput_plan_static(const parcae_problem* problem, uint32_t* hist_int, uint32_t* hist_min, float* liveput,
                               float* teff, float* gain, float* F, int32_t* bp, int32_t* plan, int32_t* start,
                               float* objective, int32_t* status, void* stream)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    CfgRec table[PARCAE_STATIC_MAX_CONFIGS];  // on the stack: this entry point allocates nothing, on either side
    Layout lay;
    int rc = check_problem(p, table, PARCAE_STATIC_MAX_CONFIGS, &lay);
    if (rc != PARCAE_OK) return rc;
    if (!hist_int || !hist_min || !plan) return PARCAE_EINVAL;
    if (lay.total > sizeof(scratch)) return PARCAE_EWORKSPACE;  // larger problems take parcae_liveput_plan
    if (!plan_fits(p, lay)) return PARCAE_EINVAL;
    void* workspace = nullptr;
    if ((rc = static_scratch(&workspace)) != PARCAE_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Batch b = make_batch(p, lay, workspace);
    const bool wave = takes_wave_planner(p, table, lay);
    EvalOpts opts;
    opts.table = table;
    opts.validate = !wave;
    opts.tables_later = wave;
    if ((rc = launch_eval(p, b, lay, workspace, hist_int, hist_min, liveput, teff, gain, nullptr, st, opts)) != PARCAE_OK)
        return rc;
    const parcae::TablesOut tables = wave ? parcae::TablesOut{liveput, teff, gain} : parcae::TablesOut{nullptr, nullptr, nullptr};
    return launch_plan(b, table, lay, workspace, hist_int, hist_min, F, bp, plan, start, objective, status, st, p->profile,
                       tables);
}

int parcae_transition_weights(const parcae_problem* problem, const uint32_t* hist_int, const uint32_t* hist_min, float* W,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    std::vector<CfgRec> table;
    Layout lay;
    int rc = check_problem(p, &table, &lay);
    if (rc != PARCAE_OK) return rc;
    if (!hist_int || !hist_min || !W) return PARCAE_EINVAL;
    if ((rc = check_workspace(lay, workspace, workspace_bytes)) != PARCAE_OK) return rc;
    const int cap = pick_plan_cap(p->n_configs, lay, 0, false);
    if (cap < 0) return PARCAE_EINVAL;
    const size_t lds = parcae::plan_lds_bytes(p->n_configs, cap, 0, false);
    if ((int64_t)p->n_queries * p->n_intervals >= (int64_t)1 << 31) return PARCAE_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Batch b = make_batch(p, lay, workspace);
    if ((rc = stage_inputs(table, lay, b, workspace, st)) != PARCAE_OK) return rc;
    parcae::transition_kernel<<<dim3((unsigned)(b.nq * b.T)), dim3(256), lds, st>>>(b, cap, hist_int, hist_min, W);
    return hipGetLastError() == hipSuccess ? PARCAE_OK : PARCAE_EHIP;
}

int parcae_dp_plan(const float* W, int32_t n_queries, int32_t n_intervals, int32_t n_configs, float* F, int32_t* bp,
                   int32_t* plan, int32_t* start, float* objective, int32_t* status, void* stream)
{
    if (!W || !plan) return PARCAE_EINVAL;
    if (!bp && bp16_bytes_for(n_intervals, n_configs) == 0) return PARCAE_EINVAL;  // no room in LDS: the walk back needs bp in memory
    if (n_queries < 1 || n_intervals < 1 || n_configs < 1 || n_configs > kMaxConfigsDp) return PARCAE_EINVAL;
    if ((int64_t)n_queries * n_intervals >= (int64_t)1 << 31 || n_queries > 65535 * 32) return PARCAE_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return launch_dp(W, n_queries, n_intervals, n_configs, nullptr, F, nullptr, bp, plan, start, objective, status, st);
}

namespace {

struct ReplayLayout {
    size_t hist_int_off, hist_min_off, plan_off, hist1_int_off, hist1_min_off, state_off, total;
};

// The replay's own buffers sit behind the workspace of the calls it makes.  The reactive baseline never plans: it
// needs the evaluation part of that workspace only (everything before the planner's weights) and no plan buffers.
ReplayLayout replay_layout(const parcae_problem* p, const Layout& lay, bool plans)
{
    const size_t nq = (size_t)p->n_queries, T = (size_t)p->n_intervals, L = (size_t)lay.L;
    ReplayLayout r;
    r.hist_int_off = plans ? lay.total : lay.w_off;
    r.hist_min_off = r.hist_int_off + (plans ? align_up(sizeof(uint32_t) * nq * T * L) : 0);
    r.plan_off = r.hist_min_off + (plans ? align_up(sizeof(uint32_t) * nq * T * L) : 0);
    r.hist1_int_off = r.plan_off + (plans ? align_up(sizeof(int32_t) * nq * T) : 0);
    r.hist1_min_off = r.hist1_int_off + align_up(sizeof(uint32_t) * nq * L);
    r.state_off = r.hist1_min_off + align_up(sizeof(uint32_t) * nq * L);
    r.total = r.state_off + align_up(sizeof(int32_t) * nq);
    return r;
}

// The problem as the replay sees it: availability comes from the windows, no profiling events.
parcae_problem replay_problem(const parcae_problem* p, const int32_t* windows)
{
    parcae_problem q = *p;
    q.avail = windows;
    q.profile = nullptr;
    return q;
}

}  // namespace

int parcae_replay_workspace_bytes(const parcae_problem* problem, int32_t n_steps, int32_t mode, size_t* bytes)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    if (!bytes || n_steps < 1) return PARCAE_EINVAL;
    if (mode != PARCAE_REPLAY_PROACTIVE && mode != PARCAE_REPLAY_REACTIVE) return PARCAE_EINVAL;
    int32_t dummy = 0;
    const parcae_problem q = replay_problem(p, p->avail ? p->avail : &dummy);
    Layout lay;
    const int rc = check_problem(&q, nullptr, &lay);
    if (rc != PARCAE_OK) return rc;
    *bytes = replay_layout(&q, lay, mode == PARCAE_REPLAY_PROACTIVE).total;
    return PARCAE_OK;
}

int parcae_replay(const parcae_problem* problem, int32_t n_steps, const int32_t* true_avail, const int32_t* windows,
                  int32_t mode, int32_t* chosen, float* reward, float* total, int32_t* status, void* workspace,
                  size_t workspace_bytes, void* stream)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    if (!true_avail || !chosen || !reward || !total || n_steps < 1) return PARCAE_EINVAL;
    if (mode != PARCAE_REPLAY_PROACTIVE && mode != PARCAE_REPLAY_REACTIVE) return PARCAE_EINVAL;
    const bool plans = mode == PARCAE_REPLAY_PROACTIVE;
    if (plans && !windows) return PARCAE_EINVAL;
    if (p->cost_move) return PARCAE_EINVAL;  // the replay's reward has no cost per moved instance
    if ((int64_t)p->n_queries * ((int64_t)n_steps + 1) >= (int64_t)1 << 31) return PARCAE_EINVAL;
    if ((int64_t)p->n_queries * n_steps * ((int64_t)p->n_intervals + 1) >= (int64_t)1 << 40) return PARCAE_EINVAL;
    const parcae_problem q = replay_problem(p, windows ? windows : true_avail);
    std::vector<CfgRec> table;
    Layout lay;
    int rc = check_problem(&q, &table, &lay);
    if (rc != PARCAE_OK) return rc;
    if (plans && !plan_fits(&q, lay)) return PARCAE_EINVAL;
    const ReplayLayout rl = replay_layout(&q, lay, plans);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < rl.total)
        return PARCAE_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* base = static_cast<unsigned char*>(workspace);
    uint32_t* hist_int = reinterpret_cast<uint32_t*>(base + rl.hist_int_off);
    uint32_t* hist_min = reinterpret_cast<uint32_t*>(base + rl.hist_min_off);
    int32_t* plan = reinterpret_cast<int32_t*>(base + rl.plan_off);
    uint32_t* hist1_int = reinterpret_cast<uint32_t*>(base + rl.hist1_int_off);
    uint32_t* hist1_min = reinterpret_cast<uint32_t*>(base + rl.hist1_min_off);
    int32_t* state = reinterpret_cast<int32_t*>(base + rl.state_off);

    // tables and starting configuration are checked once; the availability entries of the whole true walk and of
    // every window by a kernel of their own (the table check sees one row of the walk only)
    Batch b = make_batch(&q, lay, workspace);
    b.avail = true_avail;
    b.avail_stride = n_steps + 1;
    b.T = 1;
    if ((rc = stage_inputs(table, lay, b, workspace, st)) != PARCAE_OK) return rc;
    b = make_batch(&q, lay, workspace);
    parcae::replay_validate_kernel<<<dim3((unsigned)b.nq), dim3(256), 0, st>>>(b.nq, n_steps, b.T, b.N, true_avail,
                                                                              plans ? windows : nullptr,
                                                                              valid_ptr(lay, workspace));
    if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    const unsigned qblocks = (unsigned)((b.nq + 255) / 256);
    parcae::replay_init_kernel<<<dim3(qblocks), dim3(256), 0, st>>>(b.nq, b.C, p->cur_config, state, total);
    if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;

    for (int i = 0; i < n_steps; ++i) {
        const int32_t* window = nullptr;
        if (plans) {
            Batch bi = b;
            window = windows + (int64_t)i * b.nq * (b.T + 1);
            bi.avail = window;
            bi.cur_config = state;
            bi.stream_offset = 2u * (uint32_t)i;
            if ((rc = launch_eval(&q, bi, lay, workspace, hist_int, hist_min, nullptr, nullptr, nullptr, nullptr, st)) !=
                PARCAE_OK)
                return rc;
            if ((rc = launch_plan(bi, table.data(), lay, workspace, hist_int, hist_min, nullptr, nullptr, plan, nullptr, nullptr,
                                  nullptr, st)) != PARCAE_OK)
                return rc;
        }
        // the interval that actually happened: one step from true[i] to true[i + 1]
        Batch b1 = b;
        b1.T = 1;
        b1.avail = true_avail + i;
        b1.avail_stride = n_steps + 1;
        b1.cur_config = state;
        b1.stream_offset = 2u * (uint32_t)i + 1u;
        if ((rc = launch_eval(&q, b1, lay, workspace, hist1_int, hist1_min, nullptr, nullptr, nullptr, nullptr, st)) !=
            PARCAE_OK)
            return rc;
        parcae::replay_step_kernel<<<dim3(qblocks), dim3(256), 0, st>>>(b1, mode, i, n_steps, b.T, true_avail, window,
                                                                         plan, hist1_int, hist1_min, state, chosen,
                                                                         reward, total);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    }
    if (status) {
        parcae::status_from_valid_kernel<<<dim3(qblocks), dim3(256), 0, st>>>(b.nq, valid_ptr(lay, workspace), status,
                                                                               PARCAE_EINVAL);
        if (hipGetLastError() != hipSuccess) return PARCAE_EHIP;
    }
    return PARCAE_OK;
}

int parcae_debug_sample(const parcae_problem* problem, int32_t q, int32_t t, int32_t c, uint32_t s0, uint32_t ns,
                        uint32_t* masks, int32_t* n_int, int32_t* d_min, void* workspace, size_t workspace_bytes,
                        void* stream)
{
    parcae_problem local;
    if (!load_problem(problem, &local)) return PARCAE_EINVAL;
    const parcae_problem* p = &local;
    std::vector<CfgRec> table;
    Layout lay;
    int rc = check_problem(p, &table, &lay);
    if (rc != PARCAE_OK) return rc;
    if (!masks || !n_int || !d_min) return PARCAE_EINVAL;
    if (q < 0 || q >= p->n_queries || t < 0 || t >= p->n_intervals || c < 0 || c >= p->n_configs) return PARCAE_EINVAL;
    if (ns == 0u) return PARCAE_OK;
    if ((uint64_t)s0 + ns > (uint64_t)1 << 32 || ns > (1u << 30)) return PARCAE_EINVAL;
    if ((rc = check_workspace(lay, workspace, workspace_bytes)) != PARCAE_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Batch b = make_batch(p, lay, workspace);
    if ((rc = stage_inputs(table, lay, b, workspace, st)) != PARCAE_OK) return rc;
    parcae::debug_sample_kernel<<<dim3((ns + 255u) / 256u), dim3(parcae::kEvalThreads), 0, st>>>(b, q, t, c, s0, ns, masks, n_int,
                                                                                  d_min);
    return hipGetLastError() == hipSuccess ? PARCAE_OK : PARCAE_EHIP;
}

}  // extern "C"
