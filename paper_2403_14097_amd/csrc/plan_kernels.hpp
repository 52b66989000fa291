// Liveput tables, transition weights and the max-plus dynamic program (Eq. 1, Eq. 4, Eq. 6, section 6.2).
//
// All float arithmetic here is written with explicit round-to-nearest intrinsics so that
// no product and sum are ever fused: the integer plan must not depend on contraction.
#pragma once

#include "device_common.hpp"

namespace parcae {

constexpr float kNegInf = -__builtin_inff();

__device__ __forceinline__ float max0(float x) { return x > 0.0f ? x : 0.0f; }

// sum / S, correctly rounded.  When S is a power of two the quotient is an exact scaling, so one multiplication by
// 2^-log2(S) gives the same bits (denormal results included) at a tenth of the instructions of a division; the
// condition is the same for every lane of a launch.
__device__ __forceinline__ float div_by_count(float sum, uint32_t S)
{
    if ((S & (S - 1u)) == 0u) return __fmul_rn(sum, __uint_as_float((uint32_t)(127 - (31 - __clz((int)S))) << 23));
    return __fdiv_rn(sum, (float)S);
}

// Expected effective seconds from the class counts of a unit read at width w (see the header's teff()).
// n0 = scenarios needing no migration, n01 = those needing at most intra-stage migration,
// h0 = scenarios that lost a whole stage.
__device__ __forceinline__ float teff_from_counts(uint32_t n0, uint32_t n01, uint32_t h0, int w, uint32_t S,
                                                  float tau, float e0, float e1, float e2)
{
    const uint32_t n1 = n01 - n0;
    const uint32_t n3 = (w >= 1) ? h0 : 0u;
    const uint32_t n2 = S - n01 - n3;
    const float q0 = __fmul_rn((float)n0, tau);
    const float q1 = __fmul_rn((float)n1, e0);
    const float q2 = __fmul_rn((float)n2, e1);
    const float q3 = __fmul_rn((float)n3, e2);
    float sum = __fadd_rn(q0, q1);
    sum = __fadd_rn(sum, q2);
    sum = __fadd_rn(sum, q3);
    return div_by_count(sum, S);
}

// Inter-stage share of the expected effective seconds when the cost of an inter-stage migration depends on
// the scenario (section 8.4: the state-transfer cost varies with the preemptions, alpha-beta model): a stage with
// j survivors brings w instances to hold its state by doubling, the worst stage (j = d_min) sets the number of
// rounds r (smallest r with j * 2^r >= w), the migration costs c_inter + round_sec * (r - 1), at most c_repart.
// tail(x) = scenarios with d_min >= x (x >= 1).  Sum over r ascending of (float)count_r * max(0, tau - cost_r);
// bands past the one that reaches j = 1 are empty and would add +0.
template <typename Tail>
__device__ __forceinline__ float inter_seconds_by_rounds(Tail tail, int w, float tau, float c_inter, float c_repart,
                                                         float round_sec)
{
    float acc = 0.0f;
    if (w < 2) return acc;
    uint32_t above = tail(w);  // scenarios that need no inter-stage migration at this width
    for (int r = 1; r <= 8; ++r) {
        const int lo = (w + (1 << r) - 1) >> r;  // smallest j with j * 2^r >= w
        const uint32_t from_lo = tail(lo);
        float cost = __fadd_rn(c_inter, __fmul_rn(round_sec, (float)(r - 1)));
        cost = cost > c_repart ? c_repart : cost;
        acc = __fadd_rn(acc, __fmul_rn((float)(from_lo - above), max0(__fsub_rn(tau, cost))));
        above = from_lo;
        if (lo <= 1) break;
    }
    return acc;
}

// Inter-stage share of the expected effective seconds when an inter-stage migration costs c_inter + move_sec per
// instance that must receive state (section 8.4, alpha-beta model): n2 scenarios at max(0, tau - c_inter) each, less
// move_sec for every instance moved over all of them.  occ = the unit's stage-occupancy statistic (bins 0..D): a stage
// with j < w survivors needs w - j instances, and only scenarios that need an inter-stage migration have such stages.
__device__ __forceinline__ float inter_seconds_by_moves(const uint32_t* occ, int D, int w, uint32_t n2, float e1,
                                                        float move_sec)
{
    unsigned long long total_moves = 0ull;
    for (int j = 1; j <= D && j < w; ++j) total_moves += (unsigned long long)occ[j] * (unsigned long long)(w - j);
    return __fsub_rn(__fmul_rn((float)n2, e1), __fmul_rn(move_sec, __ull2float_rn(total_moves)));
}

// teff with the inter-stage share given as a sum of seconds (see the header's teff() with transfer rounds).
__device__ __forceinline__ float teff_with_inter(uint32_t n0, uint32_t n01, uint32_t h0, int w, uint32_t S, float tau,
                                                 float e0, float e2, float inter)
{
    const uint32_t n1 = n01 - n0;
    const uint32_t n3 = (w >= 1) ? h0 : 0u;
    float sum = __fadd_rn(__fmul_rn((float)n0, tau), __fmul_rn((float)n1, e0));
    sum = __fadd_rn(sum, inter);
    sum = __fadd_rn(sum, __fmul_rn((float)n3, e2));
    return div_by_count(sum, S);
}

// ------------------------------------------------------------------ input checks

// Whether this thread finds a broken rule among the device inputs of query q; the threads of a block split the
// tables between them (thread `tid` of `nthreads`), so the verdict is the OR over the block.  cfg = candidate table.
__device__ __forceinline__ int query_inputs_bad(const Batch& b, const CfgRec* cfg, int q, int tid, int nthreads)
{
    int my_bad = 0;
    for (int i = tid; i <= b.T; i += nthreads) {
        const int a = b.avail[(int64_t)q * b.avail_stride + i];
        if (a < 0 || a > b.N) my_bad = 1;
    }
    // throughputs: every entry finite and not negative (one flat pass over the table), the first entry of a row 0
    const float* th = b.thr + (int64_t)q * b.L;
    for (int i = tid; i < b.L; i += nthreads) {
        const float v = th[i];
        if (!(v >= 0.0f) || !(v < __builtin_inff())) my_bad = 1;
    }
    for (int c = tid; c < b.C; c += nthreads) {
        if (!(th[cfg[c].off] == 0.0f)) my_bad = 1;
        const float* co = b.cost + ((int64_t)q * b.C + c) * 3;
        const float c0 = co[0], c1 = co[1], c2 = co[2];
        if (!(c0 >= 0.0f) || !(c0 <= c1) || !(c1 <= c2) || !(c2 < __builtin_inff())) my_bad = 1;
    }
    if (tid == 0 && b.cur_config) {
        const int cur = b.cur_config[q];
        if (cur < -2 || cur >= b.C) my_bad = 1;
    }
    if (b.cost_round) {
        for (int c = tid; c < b.C; c += nthreads) {
            const float v = b.cost_round[(int64_t)q * b.C + c];
            if (!(v >= 0.0f) || !(v < __builtin_inff())) my_bad = 1;
        }
    }
    if (b.inst_weight) {
        for (int j = tid; j < b.N; j += nthreads)
            if (b.inst_weight[(int64_t)q * b.N + j] < 1u) my_bad = 1;
    }
    if (b.cost_move) {
        // the dearest inter-stage migration into c (every stage down to one holder) must not cost more than a
        // re-partition or than the interval lasts: the expectation is then linear in the move counts
        for (int c = tid; c < b.C; c += nthreads) {
            const float v = b.cost_move[(int64_t)q * b.C + c];
            const float* co = b.cost + ((int64_t)q * b.C + c) * 3;
            const float worst = (float)((cfg[c].D - 1) * cfg[c].P);
            const float cap = co[2] < b.tau ? co[2] : b.tau;
            if (!(v >= 0.0f) || !(v < __builtin_inff()) || !(co[1] + v * worst <= cap)) my_bad = 1;
        }
    }
    if (b.n_zones > 0) {
        for (int j = tid; j < b.N; j += nthreads)
            if ((int)b.zone[(int64_t)q * b.N + j] >= b.n_zones) my_bad = 1;
        if (tid < b.n_zones) {
            const uint32_t w = b.zone_weight[(int64_t)q * kMaxZones + tid];
            if (w < 1u || w > 255u) my_bad = 1;
        }
    }
    return my_bad;
}

// valid[q] = 1 if the query's device inputs obey the documented ranges, else 0.  One block per query.
__global__ void __launch_bounds__(256) validate_kernel(Batch b, int32_t* __restrict__ valid)
{
    __shared__ int bad;
    const int q = blockIdx.x;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    if (query_inputs_bad(b, b.cfg, q, (int)threadIdx.x, (int)blockDim.x)) atomicOr(&bad, 1);
    __syncthreads();
    if (threadIdx.x == 0) valid[q] = bad ? 0 : 1;
}

__global__ void __launch_bounds__(256) status_from_valid_kernel(int nq, const int32_t* __restrict__ valid,
                                                                int32_t* __restrict__ status, int einval)
{
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q < nq) status[q] = valid[q] ? 0 : einval;
}

// ------------------------------------------------------------------ liveput tables (Eq. 1, Eq. 4)

// The tables of unit u = (q, t, c); `cfg` is the candidate table (in memory or in the kernel's arguments).
__device__ __forceinline__ void finalise_unit(const Batch& b, const CfgRec* __restrict__ cfg, int64_t u,
                                              const uint32_t* __restrict__ hist_int,
                                              const uint32_t* __restrict__ hist_min, float* __restrict__ liveput,
                                              float* __restrict__ teff, float* __restrict__ gain)
{
    const int64_t n_units = (int64_t)b.nq * b.T * b.C;
    if (u >= n_units) return;
    const int c = (int)(u % b.C);
    const int64_t qt = u / b.C;
    const int t = (int)(qt % b.T);
    const int q = (int)(qt / b.T);
    const CfgRec cr = cfg[c];
    int M, k;
    unit_pool(b, q, t, cr.D, cr.P, M, k);
    const uint32_t* hi = hist_int + qt * b.L + cr.off;
    const uint32_t* hm = hist_min + qt * b.L + cr.off;
    const float* th = b.thr + (int64_t)q * b.L + cr.off;
    const float* co = b.cost + ((int64_t)q * b.C + c) * 3;
    const int d_cap = b.group * ((M - k) / cr.P);  // surviving instances fill whole blocks of pipelines
    const int d_star = cr.D < d_cap ? cr.D : d_cap;
    const uint32_t S = (uint32_t)b.S;

    float acc_i = 0.0f, acc_m = 0.0f;
    uint32_t n0 = 0u, n01 = 0u;
    for (int j = 0; j <= cr.D; ++j) {
        const uint32_t a = hi[j], m = hm[j];
        const float w = th[j];
        acc_i = __fadd_rn(acc_i, __fmul_rn((float)a, w));
        acc_m = __fadd_rn(acc_m, __fmul_rn((float)m, w));
        if (j >= d_star) {
            n0 += a;
            n01 += m;
        }
    }
    const float fS = (float)S;
    const float full = th[d_star];
    const float round_sec = b.cost_round ? b.cost_round[(int64_t)q * b.C + c] : 0.0f;
    const float move_sec = b.cost_move ? b.cost_move[(int64_t)q * b.C + c] : 0.0f;
    float te;
    if (move_sec != 0.0f) {
        const uint32_t n3 = d_star >= 1 ? hm[0] : 0u;
        const float inter = inter_seconds_by_moves(b.hist_occ + qt * b.L + cr.off, cr.D, d_star, S - n01 - n3,
                                                   max0(__fsub_rn(b.tau, co[1])), move_sec);
        te = teff_with_inter(n0, n01, hm[0], d_star, S, b.tau, max0(__fsub_rn(b.tau, co[0])),
                             max0(__fsub_rn(b.tau, co[2])), inter);
    } else if (round_sec == 0.0f) {
        te = teff_from_counts(n0, n01, hm[0], d_star, S, b.tau, max0(__fsub_rn(b.tau, co[0])),
                              max0(__fsub_rn(b.tau, co[1])), max0(__fsub_rn(b.tau, co[2])));
    } else {
        auto tail = [&](int x) {
            uint32_t sum = 0u;
            for (int j = x; j <= cr.D; ++j) sum += hm[j];
            return sum;
        };
        const float inter = inter_seconds_by_rounds(tail, d_star, b.tau, co[1], co[2], round_sec);
        te = teff_with_inter(n0, n01, hm[0], d_star, S, b.tau, max0(__fsub_rn(b.tau, co[0])),
                             max0(__fsub_rn(b.tau, co[2])), inter);
    }
    const int64_t lvl = (int64_t)b.T * b.C;
    const int64_t o = (int64_t)t * b.C + c;
    if (liveput) {
        float* lp = liveput + (int64_t)q * 3 * lvl;
        lp[o] = __fdiv_rn(acc_i, fS);
        lp[lvl + o] = __fdiv_rn(acc_m, fS);
        lp[2 * lvl + o] = full;
    }
    if (teff) teff[u] = te;
    if (gain) gain[u] = __fmul_rn(full, te);
}

// One thread per unit (q, t, c).
__global__ void __launch_bounds__(256) finalise_kernel(Batch b, const uint32_t* __restrict__ hist_int,
                                                       const uint32_t* __restrict__ hist_min,
                                                       float* __restrict__ liveput, float* __restrict__ teff,
                                                       float* __restrict__ gain)
{
    finalise_unit(b, b.cfg, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, hist_int, hist_min, liveput, teff, gain);
}

// ------------------------------------------------------------------ transition weights from histogram tails

// Tables of one query kept in LDS by the planning kernels.  The histogram rows of a step are brought in
// a chunk of consecutive source candidates at a time (a chunk holds at most `cap` bins), so the LDS
// footprint does not grow with the total number of bins.
struct PlanShared {
    CfgRec* cfg;         // [C]
    float* full;         // [C] thr[c][D_c]
    float* e;            // [C][3] max(0, tau - cost)
    float* rnd;          // [C][3] inter-stage cost, re-partition cost, seconds per further transfer round
    int* from_ok;        // [C] may be left at this step
    int* to_ok;          // [C] may be entered at this step
    int* chunk_start;    // [n_chunks + 1] first candidate of each chunk
    // the per-query planner only:
    float* F;                 // [C] value function of the previous step
    float* Feff;              // [C] the same, -inf where the candidate may not be left at this step
    float* R;                 // [C] thr[c][D_c] * max(0, tau - re-partition cost): weight of reaching c from another depth
    uint32_t* gspan;          // [C] candidates of the same depth as c: first | (one past last) << 16
    unsigned long long* key;  // [C] best (value, source) offered to each target in the step being built
    uint32_t* tail_int;  // [cap] suffix sums of hist_int inside each row of the current chunk
    uint32_t* tail_min;  // [cap] same for hist_min, except that slot 0 of a row keeps the raw bin 0
    uint16_t* bp16;      // [T][C] back-pointers (0xffff = none) if they fit in LDS, else null
    int n_chunks;
    int tile_log2;       // log2 of the tile width of the same-depth cells: smallest power of two >= the largest depth group
    int cold;            // this step starts from nothing running (t == 0 and cur_config == -2)
};

constexpr int kPlanThreads = 256;
constexpr int kStreamRegs = 2;  // registers per thread and histogram that hold the rows of the next step (512 bins)
constexpr uint16_t kNoPred16 = 0xffffu;

// per_query: the layout of plan_fused_kernel (value function, offers, depth groups); else that of transition_kernel.
inline size_t plan_lds_bytes(int C, int cap, size_t bp16_bytes, bool per_query)
{
    return (per_query ? 88 : 56) * (size_t)C + 32 + 8 * (size_t)cap + ((bp16_bytes + 15) & ~(size_t)15);
}

__device__ __forceinline__ void carve(unsigned char* smem, int C, int cap, bool bp_in_lds, bool per_query,
                                      PlanShared& sh)
{
    size_t o = 0;
    sh.cfg = reinterpret_cast<CfgRec*>(smem + o); o += sizeof(CfgRec) * (size_t)C;
    sh.full = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)C;
    sh.e = reinterpret_cast<float*>(smem + o); o += 12 * (size_t)C;
    sh.rnd = reinterpret_cast<float*>(smem + o); o += 12 * (size_t)C;
    sh.from_ok = reinterpret_cast<int*>(smem + o); o += 4 * (size_t)C;
    sh.to_ok = reinterpret_cast<int*>(smem + o); o += 4 * (size_t)C;
    sh.chunk_start = reinterpret_cast<int*>(smem + o); o += 4 * (size_t)(C + 1);
    sh.F = sh.Feff = sh.R = nullptr;
    sh.gspan = nullptr;
    sh.key = nullptr;
    if (per_query) {
        o = (o + 7) & ~(size_t)7;
        sh.key = reinterpret_cast<unsigned long long*>(smem + o); o += 8 * (size_t)C;
        sh.F = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)C;
        sh.Feff = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)C;
        sh.R = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)C;
        sh.gspan = reinterpret_cast<uint32_t*>(smem + o); o += 4 * (size_t)C;
    }
    o = (o + 15) & ~(size_t)15;
    sh.tail_int = reinterpret_cast<uint32_t*>(smem + o); o += 4 * (size_t)cap;
    sh.tail_min = reinterpret_cast<uint32_t*>(smem + o); o += 4 * (size_t)cap;
    sh.bp16 = bp_in_lds ? reinterpret_cast<uint16_t*>(smem + o) : nullptr;
}

// Per-query tables and the chunking of the candidate list (the same for every step).
__device__ __forceinline__ void load_query_tables(const Batch& b, int q, int cap, PlanShared& sh)
{
    __shared__ int n_chunks_s;
    __shared__ int widest_group_s;
    if (threadIdx.x == 0) widest_group_s = 1;
    __syncthreads();
    for (int c = threadIdx.x; c < b.C; c += blockDim.x) {
        const CfgRec cr = b.cfg[c];
        sh.cfg[c] = cr;

        sh.full[c] = b.thr[(int64_t)q * b.L + cr.off + cr.D];
        const float* co = b.cost + ((int64_t)q * b.C + c) * 3;
        sh.e[3 * c + 0] = max0(__fsub_rn(b.tau, co[0]));
        sh.e[3 * c + 1] = max0(__fsub_rn(b.tau, co[1]));
        sh.e[3 * c + 2] = max0(__fsub_rn(b.tau, co[2]));
        sh.rnd[3 * c + 0] = co[1];
        sh.rnd[3 * c + 1] = co[2];
        sh.rnd[3 * c + 2] = b.cost_round ? b.cost_round[(int64_t)q * b.C + c] : 0.0f;
        if (sh.R) sh.R[c] = __fmul_rn(sh.full[c], sh.e[3 * c + 2]);
    }
    __syncthreads();
    if (sh.gspan) {  // candidates are sorted by depth: the candidates of the depth of c are a run around c
        for (int c = threadIdx.x; c < b.C; c += blockDim.x) {
            const int P = sh.cfg[c].P;
            int lo = c, hi = c + 1;
            while (lo > 0 && sh.cfg[lo - 1].P == P) --lo;
            while (hi < b.C && sh.cfg[hi].P == P) ++hi;
            sh.gspan[c] = (uint32_t)lo | ((uint32_t)hi << 16);
            atomicMax(&widest_group_s, hi - lo);
        }
    }
    if (threadIdx.x == 0) {
        int n = 0, c = 0;
        while (c < b.C) {
            sh.chunk_start[n++] = c;
            const int first = sh.cfg[c].off;
            int end = c + 1;  // a row never exceeds cap (checked on the host)
            while (end < b.C && sh.cfg[end].off + sh.cfg[end].D + 1 - first <= cap) ++end;
            c = end;
        }
        sh.chunk_start[n] = b.C;
        n_chunks_s = n;
    }
    __syncthreads();
    sh.n_chunks = n_chunks_s;
    int lg = 0;
    while ((1 << lg) < widest_group_s) ++lg;
    sh.tile_log2 = lg;
}

// Feasibility of leaving / entering each candidate at step t (constraint D * P <= N of Eq. 6, memory floor,
// and the current configuration at t = 0) from the availability before and after the boundary.  Ends with a
// barrier.
__device__ __forceinline__ void set_step_flags(const Batch& b, int t, int cur, int a_prev, int a_next, PlanShared& sh)
{
    sh.cold = (t == 0 && cur == -2) ? 1 : 0;
    for (int c = threadIdx.x; c < b.C; c += blockDim.x) {
        const CfgRec cr = sh.cfg[c];
        const int used = cr.D * cr.P;
        const bool deep = cr.P >= b.p_min;
        sh.from_ok[c] = (used <= b.group * a_prev) && deep && (t > 0 || cur < 0 || c == cur);
        sh.to_ok[c] = (used <= b.group * a_next) && deep;
    }
    __syncthreads();
}

__device__ __forceinline__ void load_step_flags(const Batch& b, int q, int t, PlanShared& sh)
{
    const int a_prev = clampi(b.avail[(int64_t)q * b.avail_stride + t], 0, b.N);
    const int a_next = clampi(b.avail[(int64_t)q * b.avail_stride + t + 1], 0, b.N);
    set_step_flags(b, t, b.cur_config ? b.cur_config[q] : -1, a_prev, a_next, sh);
}

// Suffix sums inside the histogram row of candidate cr that starts at bin o of the LDS arrays (slot 0 of
// tail_min keeps the raw bin 0).
__device__ __forceinline__ void suffix_row(const PlanShared& sh, const CfgRec cr, int o)
{
    uint32_t ri = 0u, rm = 0u;
    int j = cr.D;
    // eight bins at a time: the loads are independent of the running sums, so they travel together
    for (; j >= 8; j -= 8) {
        uint32_t vi[8], vm[8];
        static_for<8>([&](auto x) {
            vi[x.value] = sh.tail_int[o + j - x.value];
            vm[x.value] = sh.tail_min[o + j - x.value];
        });
        static_for<8>([&](auto x) {
            ri += vi[x.value];
            rm += vm[x.value];
            sh.tail_int[o + j - x.value] = ri;
            sh.tail_min[o + j - x.value] = rm;
        });
    }
    for (; j >= 1; --j) {
        ri += sh.tail_int[o + j];
        rm += sh.tail_min[o + j];
        sh.tail_int[o + j] = ri;
        sh.tail_min[o + j] = rm;
    }
}

// The histogram rows of ALL steps of query q into LDS as suffix sums (step t at bins [t * L, (t + 1) * L)), for
// problems small enough that they fit: the sequential steps then touch no memory.  Ends with a barrier.
__device__ __forceinline__ void load_all_steps(const Batch& b, int q, const uint32_t* __restrict__ hist_int,
                                               const uint32_t* __restrict__ hist_min, const PlanShared& sh)
{
    const int64_t base = (int64_t)q * b.T * b.L;
    const int total = b.T * b.L;
    for (int i = threadIdx.x; i < total; i += blockDim.x) {
        sh.tail_int[i] = hist_int[base + i];
        sh.tail_min[i] = hist_min[base + i];
    }
    __syncthreads();
    for (int row = threadIdx.x; row < b.T * b.C; row += blockDim.x) {
        const int t = row / b.C;
        const CfgRec cr = sh.cfg[row - t * b.C];
        suffix_row(sh, cr, t * b.L + cr.off);
    }
    __syncthreads();
}

// Histogram rows of candidates [c_lo, c_hi) of step (q, t) into LDS as suffix sums.  Starts and ends with a barrier.
__device__ __forceinline__ void load_chunk(const Batch& b, int q, int t, int c_lo, int c_hi,
                                           const uint32_t* __restrict__ hist_int,
                                           const uint32_t* __restrict__ hist_min, const PlanShared& sh)
{
    __syncthreads();  // the previous chunk is no longer read
    const int first = sh.cfg[c_lo].off;
    const int last = sh.cfg[c_hi - 1].off + sh.cfg[c_hi - 1].D + 1;
    const int64_t base = ((int64_t)q * b.T + t) * b.L + first;
    for (int i = threadIdx.x; i < last - first; i += blockDim.x) {
        sh.tail_int[i] = hist_int[base + i];
        sh.tail_min[i] = hist_min[base + i];
    }
    __syncthreads();
    for (int c = c_lo + threadIdx.x; c < c_hi; c += blockDim.x) {
        const CfgRec cr = sh.cfg[c];
        suffix_row(sh, cr, cr.off - first);
    }
    __syncthreads();
}

// Weight of a same-depth transition c -> c2 (both feasible, not a cold start): throughput of c2 times the expected
// effective seconds of unit (t, c) read at the width of c2.  `first` = first bin of the rows held in LDS.
// occ_step / move_sec: with a cost per moved instance, the stage-occupancy statistic of the step (all candidates,
// in memory) and the rate of the target; otherwise null / 0.
template <bool kRounds>
__device__ __forceinline__ float same_depth_weight(const Batch& b, const PlanShared& sh, int first, int c, int c2,
                                                   const uint32_t* occ_step = nullptr, float move_sec = 0.0f)
{
    // every table value is loaded before the first use, so that the loads travel together
    const CfgRec a = sh.cfg[c], z = sh.cfg[c2];
    const float full = sh.full[c2];
    const float e0 = sh.e[3 * c2], e1 = sh.e[3 * c2 + 1], e2 = sh.e[3 * c2 + 2];
    const int o = a.off - first;
    // a target wider than the source keeps nothing; the loads stay unconditional on a clamped index
    const int at = z.D <= a.D ? z.D : a.D;  // z.D >= 1, so the raw slot 0 is never read as a suffix sum
    const uint32_t t_int = sh.tail_int[o + at], t_min = sh.tail_min[o + at];
    const uint32_t n0 = z.D <= a.D ? t_int : 0u, n01 = z.D <= a.D ? t_min : 0u;
    const uint32_t h0 = sh.tail_min[o];
    if (move_sec != 0.0f) {
        const uint32_t n3 = h0;  // the width of a target is at least 1
        const float inter = inter_seconds_by_moves(occ_step + a.off, a.D, z.D, (uint32_t)b.S - n01 - n3, e1, move_sec);
        return __fmul_rn(full, teff_with_inter(n0, n01, h0, z.D, (uint32_t)b.S, b.tau, e0, e2, inter));
    }
    if constexpr (kRounds) {
        const float round_sec = sh.rnd[3 * c2 + 2];
        if (round_sec != 0.0f) {
            auto tail = [&](int x) { return x <= a.D ? sh.tail_min[o + x] : 0u; };
            const float inter =
                inter_seconds_by_rounds(tail, z.D, b.tau, sh.rnd[3 * c2], sh.rnd[3 * c2 + 1], round_sec);
            return __fmul_rn(full, teff_with_inter(n0, n01, h0, z.D, (uint32_t)b.S, b.tau, e0, e2, inter));
        }
    }
    return __fmul_rn(full, teff_from_counts(n0, n01, h0, z.D, (uint32_t)b.S, b.tau, e0, e1, e2));
}

// W_t[c][c'] for a source c inside the chunk that starts at bin `first`.  occ_step, move: see same_depth_weight.
__device__ __forceinline__ float transition_weight(const Batch& b, const PlanShared& sh, int first, int c, int c2,
                                                   const uint32_t* occ_step = nullptr, const float* move = nullptr)
{
    if (sh.cold)  // nothing is running: the first configuration comes up at its re-partition cost
        return (c == c2 && sh.to_ok[c2]) ? __fmul_rn(sh.full[c2], sh.e[3 * c2 + 2]) : kNegInf;
    if (!sh.from_ok[c] || !sh.to_ok[c2]) return kNegInf;
    if (sh.cfg[c].P != sh.cfg[c2].P) return __fmul_rn(sh.full[c2], sh.e[3 * c2 + 2]);
    if (move) return same_depth_weight<false>(b, sh, first, c, c2, occ_step, move[c2]);
    return b.cost_round ? same_depth_weight<true>(b, sh, first, c, c2) : same_depth_weight<false>(b, sh, first, c, c2);
}

// Writes W[q][t][c][c'] (one block per (q, t)).
__global__ void __launch_bounds__(256) transition_kernel(Batch b, int cap, const uint32_t* __restrict__ hist_int,
                                                         const uint32_t* __restrict__ hist_min, float* __restrict__ W)
{
    extern __shared__ __align__(16) unsigned char smem[];
    PlanShared sh;
    carve(smem, b.C, cap, false, false, sh);
    const int q = blockIdx.x / b.T;
    const int t = blockIdx.x - q * b.T;
    load_query_tables(b, q, cap, sh);
    load_step_flags(b, q, t, sh);
    float* Wt = W + ((int64_t)q * b.T + t) * b.C * b.C;
    const uint32_t* occ_step = b.cost_move ? b.hist_occ + ((int64_t)q * b.T + t) * b.L : nullptr;
    const float* move = b.cost_move ? b.cost_move + (int64_t)q * b.C : nullptr;
    for (int ch = 0; ch < sh.n_chunks; ++ch) {
        const int c_lo = sh.chunk_start[ch], c_hi = sh.chunk_start[ch + 1];
        load_chunk(b, q, t, c_lo, c_hi, hist_int, hist_min, sh);
        const int first = sh.cfg[c_lo].off;
        const int cells = (c_hi - c_lo) * b.C;
        for (int i = threadIdx.x; i < cells; i += blockDim.x) {
            const int c = c_lo + i / b.C;
            const int c2 = i % b.C;
            Wt[(int64_t)c * b.C + c2] = transition_weight(b, sh, first, c, c2, occ_step, move);
        }
    }
}

// ------------------------------------------------------------------ dynamic program (Eq. 6)

// The 256 threads of a planning block form a grid of CW target columns x RG groups of source rows
// (CW * RG = 256, CW a power of two).  Every thread scans its rows in ascending order for its column;
// the group results are then merged in ascending group order with a strict comparison, so the
// smallest arg-max wins exactly as in a plain ascending scan.
struct ColumnGrid {
    int cw, cw_log2, rg, x, g;
};

__device__ __forceinline__ ColumnGrid column_grid(int C)
{
    ColumnGrid cg;
    cg.cw_log2 = C > 32 ? 6 : (C > 16 ? 5 : 4);
    cg.cw = 1 << cg.cw_log2;
    cg.rg = kPlanThreads >> cg.cw_log2;
    cg.x = (int)threadIdx.x & (cg.cw - 1);
    cg.g = (int)threadIdx.x >> cg.cw_log2;
    return cg;
}

// Order-preserving map of a float to an unsigned integer (a larger float gives a larger key; no float maps to 0).
__device__ __forceinline__ uint32_t float_key(float v)
{
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Offers value v reached from source c to a target's slot: the larger value wins and, among equal values, the
// smaller source, which is the order in which a plain ascending scan with a strict comparison decides.  -inf (and
// NaN) is no offer.  One LDS atomic; the result does not depend on the order of the offers.
__device__ __forceinline__ void offer(unsigned long long* slot, float v, int c)
{
    if (v > kNegInf) atomicMax(slot, ((unsigned long long)float_key(v) << 32) | (unsigned long long)(0xffffffffu - (uint32_t)c));
}

// Final arg-max and walk back along the back-pointers; thread 0 of the block only.
// bp16 (LDS, 0xffff = none) is used when present, else the back-pointers in memory.
__device__ __forceinline__ void finish_plan(int q, int T, int C, const float* F_last, const int32_t* bp_q,
                                            const uint16_t* bp16, int32_t* plan, int32_t* start, float* objective,
                                            int32_t* status, bool inputs_valid, int einval, int einfeasible)
{
    float top = kNegInf;
    int last = -1;
    for (int c = 0; c < C; ++c)
        if (F_last[c] > top) {
            top = F_last[c];
            last = c;
        }
    int32_t* pl = plan + (int64_t)q * T;
    int st = 0;
    if (last < 0) {
        for (int t = 0; t < T; ++t) pl[t] = -1;
        if (start) start[q] = -1;
        st = einfeasible;
    } else {
        pl[T - 1] = last;
        for (int t = T - 1; t >= 0; --t) {
            int prev;
            if (bp16) {
                const uint16_t v = bp16[t * C + last];
                prev = v == kNoPred16 ? -1 : (int)v;
            } else {
                prev = bp_q[(int64_t)t * C + last];
            }
            if (prev < 0) prev = 0;  // cannot happen on a finite path; keeps the walk in bounds
            if (t >= 1) pl[t - 1] = prev;
            else if (start) start[q] = prev;
            last = prev;
        }
    }
    if (objective) objective[q] = top;
    if (status) status[q] = inputs_valid ? st : einval;
}

// One block per query: T dependent max-plus steps with the weights computed on the fly from the
// histogram tails (the weights never touch HBM), then the walk back.  Used when there are enough
// queries to fill the chip.
//
// A step offers, for every pair (source c, target c2), F[c] + W[c][c2] to the target's slot (see offer()).  Pairs
// of different depth all carry the same weight R[c2], so they cost one addition each: a thread scans a slice of the
// sources for its target column and makes one offer.  Pairs of the same depth need the histogram tails of the source;
// the candidates of one depth are contiguous, so these pairs form square tiles on the diagonal: they are laid out
// row by row in tiles `1 << tile_log2` wide and dealt to the threads evenly, each pair one offer.
__global__ void __launch_bounds__(kPlanThreads) plan_fused_kernel(
    Batch b, int cap, int bp_in_lds, int resident, const uint32_t* __restrict__ hist_int,
    const uint32_t* __restrict__ hist_min, const int32_t* __restrict__ valid, float* __restrict__ F,
    int32_t* __restrict__ bp, int32_t* __restrict__ plan, int32_t* __restrict__ start, float* __restrict__ objective,
    int32_t* __restrict__ status, int einval, int einfeasible)
{
    extern __shared__ __align__(16) unsigned char smem[];
    PlanShared sh;
    carve(smem, b.C, cap, bp_in_lds != 0, true, sh);
    const int q = blockIdx.x;
    const int C = b.C;
    const int tid = (int)threadIdx.x;
    const ColumnGrid cg = column_grid(C);
    load_query_tables(b, q, cap, sh);
    float* Fq = F ? F + (int64_t)q * (b.T + 1) * C : nullptr;
    int32_t* bpq = bp ? bp + (int64_t)q * b.T * C : nullptr;
    for (int c = tid; c < C; c += kPlanThreads) {
        sh.F[c] = 0.0f;
        if (Fq) Fq[c] = 0.0f;
    }
    // resident: cap holds the rows of every step (T * L bins), loaded once; the steps then run out of LDS
    if (resident) load_all_steps(b, q, hist_int, hist_min, sh);
    uint32_t* const all_int = sh.tail_int;
    uint32_t* const all_min = sh.tail_min;
    const int n_chunks = resident ? 1 : sh.n_chunks;
    const int wlog = sh.tile_log2;
    const int rows_per_pass = kPlanThreads >> wlog;
    const int tile_row = tid >> wlog, tile_col = tid & ((1 << wlog) - 1);
    const int rpg = (C + cg.rg - 1) / cg.rg;  // sources per thread of the different-depth scan
    const int r0 = cg.g * rpg, r1 = r0 + rpg < C ? r0 + rpg : C;
    // availability is read one step ahead of its use, so its latency never sits on the chain of steps
    const int32_t* av = b.avail + (int64_t)q * b.avail_stride;
    const int cur = b.cur_config ? b.cur_config[q] : -1;
    int a_prev = clampi(av[0], 0, b.N);
    int a_next = clampi(av[1], 0, b.N);
    // Opens step t for candidate c whose value is f: Feff (feasibility of leaving c: constraint D * P <= N of Eq. 6,
    // memory floor, the current configuration at t = 0), to_ok (feasibility of entering c), empty offer slot.
    auto open_step = [&](int t, int c, float f, int before, int after) __attribute__((always_inline)) {
        const CfgRec cr = sh.cfg[c];
        const int used = cr.D * cr.P;
        const bool deep = cr.P >= b.p_min;
        const bool from = (used <= b.group * before) && deep && (t > 0 || cur < 0 || c == cur);
        sh.Feff[c] = from ? f : kNegInf;
        sh.to_ok[c] = (used <= b.group * after) && deep;
        sh.key[c] = 0ull;
    };
    for (int c = tid; c < C; c += kPlanThreads) open_step(0, c, 0.0f, a_prev, a_next);
    // streamed: the rows of a step fit in LDS at once and in kStreamRegs registers per thread; the rows of step t + 1
    // are read into registers while step t runs, so the memory latency is off the chain of steps
    const bool streamed = !resident && sh.n_chunks == 1 && b.L <= kStreamRegs * kPlanThreads;
    uint32_t next_int[kStreamRegs], next_min[kStreamRegs];
    auto fetch_rows = [&](int t) __attribute__((always_inline)) {
        const int64_t base = ((int64_t)q * b.T + t) * b.L;
        static_for<kStreamRegs>([&](auto x) {
            const int i = x.value * kPlanThreads + tid;
            next_int[x.value] = hist_int[base + (i < b.L ? i : 0)];  // unconditional, on a clamped index
            next_min[x.value] = hist_min[base + (i < b.L ? i : 0)];
        });
    };
    if (streamed) fetch_rows(0);
    __syncthreads();
    for (int t = 0; t < b.T; ++t) {
        const int a_after = av[t + 2 <= b.T ? t + 2 : b.T];
        if (streamed) {
            // nobody reads the previous rows any more (barrier at the end of the previous step)
            static_for<kStreamRegs>([&](auto x) {
                const int i = x.value * kPlanThreads + tid;
                if (i < b.L) {
                    sh.tail_int[i] = next_int[x.value];
                    sh.tail_min[i] = next_min[x.value];
                }
            });
            __syncthreads();
            for (int c = tid; c < C; c += kPlanThreads) suffix_row(sh, sh.cfg[c], sh.cfg[c].off);
            fetch_rows(t + 1 < b.T ? t + 1 : t);
            // the different-depth offers below do not touch the rows; the barrier before the tiles orders the sums
        }
        if (t == 0 && cur == -2) {
            // nothing is running: every candidate can only be "reached from itself", at its re-partition cost
            for (int c2 = tid; c2 < C; c2 += kPlanThreads)
                if (sh.to_ok[c2]) offer(&sh.key[c2], __fadd_rn(0.0f, sh.R[c2]), c2);
        } else {
            // sources of another depth
            for (int base = 0; base < C; base += cg.cw) {
                const int c2 = base + cg.x;
                if (c2 < C) {
                    const uint32_t span = sh.gspan[c2];
                    const int lo = (int)(span & 0xffffu), hi = (int)(span >> 16);
                    const float reach = sh.R[c2];
                    const int entered = sh.to_ok[c2];
                    float best = kNegInf;
                    int arg = -1;
                    for (int c0 = r0; c0 < r1; c0 += 4) {  // four sources at a time, loads on clamped indices
                        float f[4];
                        static_for<4>([&](auto x) { f[x.value] = sh.Feff[c0 + x.value < r1 ? c0 + x.value : r0]; });
                        static_for<4>([&](auto x) {
                            const int c = c0 + x.value;
                            const float v = __fadd_rn(f[x.value], reach);
                            if (c < r1 && (c < lo || c >= hi) && v > best) {
                                best = v;
                                arg = c;
                            }
                        });
                    }
                    if (entered && arg >= 0) offer(&sh.key[c2], best, arg);
                }
            }
            // sources of the same depth
            if (resident) {
                sh.tail_int = all_int + t * b.L;
                sh.tail_min = all_min + t * b.L;
            }
            for (int ch = 0; ch < n_chunks; ++ch) {
                const int c_lo = resident ? 0 : sh.chunk_start[ch], c_hi = resident ? C : sh.chunk_start[ch + 1];
                if (streamed) __syncthreads();
                else if (!resident) load_chunk(b, q, t, c_lo, c_hi, hist_int, hist_min, sh);  // barriers before and after
                const int first = sh.cfg[c_lo].off;
                auto tiles = [&](auto rounds, auto batch) __attribute__((always_inline)) {
                    constexpr int kTileBatch = decltype(batch)::value;
                    // `batch` passes at a time: table loads of the batch go out together, every load on clamped
                    // indices, only the offers are predicated
                    for (int row0 = c_lo; row0 < c_hi; row0 += kTileBatch * rows_per_pass) {
                        int cs[kTileBatch], c2s[kTileBatch];
                        bool live[kTileBatch];
                        uint32_t span[kTileBatch];
                        static_for<kTileBatch>([&](auto x) {
                            const int c = row0 + x.value * rows_per_pass + tile_row;
                            live[x.value] = c < c_hi;
                            cs[x.value] = live[x.value] ? c : c_lo;
                            span[x.value] = sh.gspan[cs[x.value]];
                        });
                        static_for<kTileBatch>([&](auto x) {
                            const int lo = (int)(span[x.value] & 0xffffu), hi = (int)(span[x.value] >> 16);
                            live[x.value] = live[x.value] && lo + tile_col < hi;
                            c2s[x.value] = live[x.value] ? lo + tile_col : lo;
                        });
                        float f[kTileBatch], w[kTileBatch];
                        int entered[kTileBatch];
                        static_for<kTileBatch>([&](auto x) {
                            f[x.value] = sh.Feff[cs[x.value]];
                            entered[x.value] = sh.to_ok[c2s[x.value]];
                            w[x.value] = same_depth_weight<decltype(rounds)::value>(b, sh, first, cs[x.value], c2s[x.value]);
                        });
                        static_for<kTileBatch>([&](auto x) {
                            if (live[x.value] && entered[x.value])
                                offer(&sh.key[c2s[x.value]], __fadd_rn(f[x.value], w[x.value]), cs[x.value]);
                        });
                    }
                };
                const bool few = c_hi - c_lo <= 2 * rows_per_pass;  // small candidate lists: no more slots than cells
                if (b.cost_round) {
                    if (few) tiles(std::true_type{}, std::integral_constant<int, 2>{});
                    else tiles(std::true_type{}, std::integral_constant<int, 4>{});
                } else {
                    if (few) tiles(std::false_type{}, std::integral_constant<int, 2>{});
                    else tiles(std::false_type{}, std::integral_constant<int, 4>{});
                }
            }
        }
        __syncthreads();
        // close step t and open step t + 1: one pass, the thread of candidate c2 holds its new value
        const int before = a_next, after = clampi(a_after, 0, b.N);
        for (int c2 = tid; c2 < C; c2 += kPlanThreads) {
            const unsigned long long k = sh.key[c2];
            const float v = k ? key_float((uint32_t)(k >> 32)) : kNegInf;
            const int a = k ? (int)(0xffffffffu - (uint32_t)k) : -1;
            sh.F[c2] = v;
            if (bpq) bpq[(int64_t)t * C + c2] = a;
            if (sh.bp16) sh.bp16[t * C + c2] = a < 0 ? kNoPred16 : (uint16_t)a;
            if (Fq) Fq[(int64_t)(t + 1) * C + c2] = v;
            open_step(t + 1, c2, v, before, after);
        }
        a_prev = before;
        a_next = after;
        __syncthreads();
    }
    __syncthreads();
    if (tid == 0) {
        finish_plan(q, b.T, C, sh.F, bpq, sh.bp16, plan, start, objective, status, valid ? valid[q] != 0 : true, einval,
                    einfeasible);
    }
}

// Scans source rows [r0, r1) of column c2 of a weight tile (in memory or in LDS), eight loads in flight
// at a time (a one-load-at-a-time loop is bound by latency).  f = F of the previous step (LDS).
__device__ __forceinline__ void scan_rows_memory(const float* __restrict__ Wt, int C, int c2, int r0, int r1,
                                                 const float* f, float& best, int& arg)
{
    for (int c = r0; c < r1; c += 8) {
        float w[8];
        static_for<8>([&](auto i) {
            const int row = c + i.value;
            w[i.value] = row < r1 ? Wt[(int64_t)row * C + c2] : kNegInf;
        });
        static_for<8>([&](auto i) {
            const int row = c + i.value;
            if (row < r1) {
                const float v = __fadd_rn(f[row], w[i.value]);
                if (v > best) {
                    best = v;
                    arg = row;
                }
            }
        });
    }
}

constexpr int kStagedMaxConfigs = 64;                                               // tiles up to 64 x 64 are staged in LDS
constexpr int kStageRegs = kStagedMaxConfigs * kStagedMaxConfigs / kPlanThreads;    // floats per thread per tile

inline size_t dp_lds_bytes(int C, size_t bp16_bytes)
{
    const size_t tiles = C <= kStagedMaxConfigs ? 2 * sizeof(float) * kStageRegs * kPlanThreads : 0;
    return 12 * (size_t)C + ((bp16_bytes + 15) & ~(size_t)15) + 16 + tiles;
}

// One block per query on weights held in memory: W[q][t][c][c'], c' contiguous.
// Tiles of up to 64 x 64 candidates travel memory -> registers -> LDS two steps ahead of the step that
// consumes them, so the T dependent steps never wait for memory; larger tiles are read in place.
// A step: every thread scans a slice of the sources for its target column and offers its best to the target's
// slot (see offer()); barrier; the thread of each target reads its slot, which becomes F of the next step.
__global__ void __launch_bounds__(kPlanThreads) dp_kernel(const float* __restrict__ W, int T, int C, int bp_in_lds,
                                                          const int32_t* __restrict__ valid, float* __restrict__ F,
                                                          int32_t* __restrict__ bp, int32_t* __restrict__ plan,
                                                          int32_t* __restrict__ start, float* __restrict__ objective,
                                                          int32_t* __restrict__ status, int einval, int einfeasible)
{
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* key = reinterpret_cast<unsigned long long*>(smem);  // [C] offers of the step being built
    float* Fc = reinterpret_cast<float*>(smem + 8 * (size_t)C);              // [C] value function of the previous step
    size_t o = 12 * (size_t)C;
    uint16_t* bp16 = bp_in_lds ? reinterpret_cast<uint16_t*>(smem + o) : nullptr;
    if (bp_in_lds) o += (sizeof(uint16_t) * (size_t)T * (size_t)C + 15) & ~(size_t)15;
    o = (o + 15) & ~(size_t)15;
    float* tile0 = reinterpret_cast<float*>(smem + o);
    const bool staged = C <= kStagedMaxConfigs;
    const int n_w = C * C;
    float* tile1 = tile0 + kStageRegs * kPlanThreads;

    const int q = blockIdx.x;
    const ColumnGrid cg = column_grid(C);
    float* Fq = F ? F + (int64_t)q * (T + 1) * C : nullptr;
    int32_t* bpq = bp ? bp + (int64_t)q * T * C : nullptr;
    const float* Wq = W + (int64_t)q * T * C * C;
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        Fc[c] = 0.0f;
        key[c] = 0ull;
        if (Fq) Fq[c] = 0.0f;
    }
    const int rpg = (C + cg.rg - 1) / cg.rg;
    const int r0 = cg.g * rpg;
    const int r1 = r0 + rpg < C ? r0 + rpg : C;

    float ra[kStageRegs], rb[kStageRegs];
    // Loads and LDS writes are unconditional (indices clamped into the tile, LDS tiles padded to a full
    // register set): with no branches around them the compiler can wait for exactly the older tile and
    // leave the newer one in flight.
    auto fetch = [&](int t, float (&r)[kStageRegs]) __attribute__((always_inline)) {
        const float* src = Wq + (int64_t)(t < T ? t : T - 1) * n_w;
        static_for<kStageRegs>([&](auto i) {
            const int idx = (int)threadIdx.x + kPlanThreads * i.value;
            r[i.value] = src[idx < n_w ? idx : n_w - 1];
        });
    };
    auto stash = [&](const float (&r)[kStageRegs], float* tile) __attribute__((always_inline)) {
        static_for<kStageRegs>([&](auto i) { tile[(int)threadIdx.x + kPlanThreads * i.value] = r[i.value]; });
    };
    // offers of step t from the tile (LDS) or from W_t in memory; the caller puts a barrier after it
    auto offers = [&](int t, const float* tile) __attribute__((always_inline)) {
        const float* Wt = Wq + (int64_t)t * n_w;
        for (int base = 0; base < C; base += cg.cw) {
            const int c2 = base + cg.x;
            float best = kNegInf;
            int arg = -1;
            if (c2 < C) {
                if (tile) scan_rows_memory(tile, C, c2, r0, r1, Fc, best, arg);
                else scan_rows_memory(Wt, C, c2, r0, r1, Fc, best, arg);
                if (arg >= 0) offer(&key[c2], best, arg);
            }
        }
    };
    // slots -> F, back-pointers; empties the slots; the caller puts a barrier after it
    auto close = [&](int t) __attribute__((always_inline)) {
        for (int c2 = threadIdx.x; c2 < C; c2 += blockDim.x) {
            const unsigned long long k = key[c2];
            const float v = k ? key_float((uint32_t)(k >> 32)) : kNegInf;
            const int a = k ? (int)(0xffffffffu - (uint32_t)k) : -1;
            Fc[c2] = v;
            key[c2] = 0ull;
            if (bpq) bpq[(int64_t)t * C + c2] = a;
            if (bp16) bp16[t * C + c2] = a < 0 ? kNoPred16 : (uint16_t)a;
            if (Fq) Fq[(int64_t)(t + 1) * C + c2] = v;
        }
    };

    if (staged) {
        fetch(0, ra);
        fetch(1, rb);
        stash(ra, tile0);
        __syncthreads();
        for (int t = 0; t < T; t += 2) {
            // even step: tile0 holds W_t, rb holds W_{t+1}; ra is free for W_{t+2}
            fetch(t + 2, ra);
            offers(t, tile0);
            stash(rb, tile1);
            __syncthreads();
            close(t);
            __syncthreads();
            if (t + 1 >= T) break;
            // odd step: tile1 holds W_{t+1}, ra holds W_{t+2}; rb is free for W_{t+3}
            fetch(t + 3, rb);
            offers(t + 1, tile1);
            stash(ra, tile0);
            __syncthreads();
            close(t + 1);
            __syncthreads();
        }
    } else {
        __syncthreads();
        for (int t = 0; t < T; ++t) {
            offers(t, nullptr);
            __syncthreads();
            close(t);
            __syncthreads();
        }
    }
    if (threadIdx.x == 0)
        finish_plan(q, T, C, Fc, bpq, bp16, plan, start, objective, status, valid ? valid[q] != 0 : true, einval,
                    einfeasible);
}

// One max-plus step for 16 target columns of one query (grid: column blocks x queries), weights and F in
// memory.  Launched once per step when a few queries have many candidates, so that a step is spread
// over many compute units.  F is [nq][T + 1][C] and must be present; bp is [nq][T][C].
constexpr int kStepCols = 16;
__global__ void __launch_bounds__(kPlanThreads) dp_step_kernel(const float* __restrict__ W, int T, int C, int t,
                                                               float* __restrict__ F, int32_t* __restrict__ bp)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red_val[kPlanThreads];
    __shared__ int red_arg[kPlanThreads];
    float* f_prev = reinterpret_cast<float*>(smem);  // [C]
    constexpr int kGroups = kPlanThreads / kStepCols;
    const int q = blockIdx.y;
    const int x = (int)threadIdx.x & (kStepCols - 1);
    const int g = (int)threadIdx.x / kStepCols;
    const int c2 = (int)blockIdx.x * kStepCols + x;
    float* Fq = F + (int64_t)q * (T + 1) * C;
    const float* Wt = W + ((int64_t)q * T + t) * C * C;
    for (int c = threadIdx.x; c < C; c += blockDim.x) f_prev[c] = (t == 0) ? 0.0f : Fq[(int64_t)t * C + c];
    if (t == 0 && g == 0 && c2 < C) Fq[c2] = 0.0f;  // F_0 for the caller
    __syncthreads();
    const int rpg = (C + kGroups - 1) / kGroups;
    const int r0 = g * rpg;
    const int r1 = r0 + rpg < C ? r0 + rpg : C;
    float best = kNegInf;
    int arg = -1;
    if (c2 < C) scan_rows_memory(Wt, C, c2, r0, r1, f_prev, best, arg);
    red_val[threadIdx.x] = best;
    red_arg[threadIdx.x] = arg;
    __syncthreads();
    if (g == 0 && c2 < C) {
        float cur = kNegInf;
        int a = -1;
        for (int gg = 0; gg < kGroups; ++gg) {
            const float v = red_val[gg * kStepCols + x];
            if (v > cur) {
                cur = v;
                a = red_arg[gg * kStepCols + x];
            }
        }
        Fq[(int64_t)(t + 1) * C + c2] = cur;
        bp[((int64_t)q * T + t) * C + c2] = a;
    }
}

// Final arg-max and walk back for the stepwise path (one thread per query does the walk).
__global__ void __launch_bounds__(64) dp_finish_kernel(int nq, int T, int C, const int32_t* __restrict__ valid,
                                                       const float* __restrict__ F, const int32_t* __restrict__ bp,
                                                       int32_t* __restrict__ plan, int32_t* __restrict__ start,
                                                       float* __restrict__ objective, int32_t* __restrict__ status,
                                                       int einval, int einfeasible)
{
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nq) return;
    finish_plan(q, T, C, F + ((int64_t)q * (T + 1) + T) * C, bp + (int64_t)q * T * C, nullptr, plan, start, objective,
                status, valid ? valid[q] != 0 : true, einval, einfeasible);
}

}  // namespace parcae
