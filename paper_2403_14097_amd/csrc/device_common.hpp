// Shared device-side definitions of the liveput kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

namespace parcae {

constexpr int kWave = 64;
constexpr int kMaxInstances = 256;
constexpr int kMaxZones = 4;

// One candidate configuration as the kernels see it (16 bytes, one vector load).
struct CfgRec {
    int32_t D;      // data-parallel pipelines
    int32_t P;      // pipeline stages
    int32_t off;    // offset of the candidate's row in the throughput table and in the histograms
    int32_t log2P;  // log2(P) if P is a power of two, else -1
};

// Everything a kernel needs to know about the batch; passed by value.
struct Batch {
    int32_t nq, N, T, C, S, p_min, L;
    int32_t pool_all;           // 0: preemptions fall on the used instances, 1: on all available ones
    int32_t group;              // GPUs per instance (>= 1); availability counts instances, D * P counts GPUs
    int32_t avail_stride;       // ints between the availability rows of consecutive queries (T + 1 if packed)
    uint32_t stream_offset;     // added to every query's Philox stream id
    float tau;
    const CfgRec* cfg;          // [C]
    const int32_t* avail;       // [nq][T+1]
    const float* thr;           // [nq][L]
    const float* cost;          // [nq][C][3]
    const uint64_t* seed;       // [nq]
    const uint32_t* stream_id;  // [nq] or null
    const int32_t* cur_config;  // [nq] or null
    int32_t n_zones;              // 0: uniform preemption; else instances fall into zones of unequal hazard
    const uint8_t* zone;          // [nq][N] zone of every instance, or null
    const uint32_t* zone_weight;  // [nq][kMaxZones] hazard weight of every zone, or null
    const float* cost_round;      // [nq][C] seconds per further state-transfer round of an inter-stage migration, or null
    const uint8_t* inst_weight;   // [nq][N] hazard weight of every instance (1..255), or null
    const float* cost_move;       // [nq][C] seconds per instance that must receive state in an inter-stage migration, or null
    uint32_t* hist_occ;           // [nq][T][L] stage-occupancy statistic (with cost_move), or null
};

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

// Pool (M instances, the first D * P / group of them run the grid) and preempted count k of unit (q, t, c).
// Used-instance pool: M = instances used, k = max(0, M - a_t) (section 4.2).  Whole-cluster pool
// (section 6.3: the N- preemptions fall on any of the N_i available instances, idle ones included):
// M = max(a_{t-1}, instances used), k = max(0, M - a_t); a configuration that does not fit a_{t-1} keeps
// the pool of its own instances.
// With multi-GPU instances (section 9.2) an instance holds one stage of `group` neighbouring pipelines, so
// the instances form a (D / group) x P grid and every count on the GPU grid is `group` times the count on
// the instance grid; the kernels sample and reduce on the instance grid.
__device__ __forceinline__ void unit_pool(const Batch& b, int q, int t, int D, int P, int& M, int& k)
{
    const int32_t* av = b.avail + (int64_t)q * b.avail_stride + t;
    M = (D / b.group) * P;
    if (b.pool_all) {
        const int a_prev = clampi(av[0], 0, b.N);
        M = a_prev > M ? a_prev : M;
    }
    k = M - clampi(av[1], 0, b.N);
    k = k < 0 ? 0 : k;
}

// Units whose scenarios all fall into one histogram bin (the same bin in both histograms), so that no
// sampling is needed: nothing preempted (bin D), everything preempted (bin 0) and, when the pool is the
// grid itself, a single stage (every preemption removes exactly one pipeline: bin D - k) or a single
// pipeline that is hit (bin 0).
__device__ __forceinline__ bool unit_closed_form(int D, int P, int M, int k, int& bin)
{
    if (k == 0) { bin = D; return true; }
    if (k == M) { bin = 0; return true; }
    if (M == D * P) {
        if (P == 1) { bin = D - k; return true; }
        if (D == 1) { bin = 0; return true; }
    }
    return false;
}

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>).  Register arrays are
// only ever indexed with these constants, so they are split into scalar registers before any other
// optimisation sees them (a run-time loop, even one unrolled later, lets the optimiser turn a chain of
// selects into one indexed load from scratch memory).
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

}  // namespace parcae
