// Look-ahead dynamic program (Eq. 6) for candidate lists of at most 64 entries, built around one wavefront
// per query: candidate c lives on lane c, so a step of the recurrence needs no workgroup barrier and no atomics.
//
// The chain of T dependent steps is the only sequential part of the plan, so everything that does not depend on
// the value function is taken off it:
//   phase A (all threads, before the chain): the weights of the same-depth transitions of a chunk of steps, from
//           the histogram tails, into local memory (Eq. 4 with the rule of section 6.2); they do not depend on F;
//   chain   (one wave): F_{t+1}[c'] = max(max over same-depth c of F_t[c] + W_t[c][c'],
//                                          (max over other-depth c of F_t[c]) + R[c']),
//           values only.  All transitions into c' from another depth carry the same weight R[c'] (re-partition), and
//           a rounded addition is monotone, so the largest sum is the sum with the largest F_t[c]: one prefix and one
//           suffix maximum over the lanes serve every target at once;
//   phase C (all threads, after the chain): the back-pointer of every (step, target) is the smallest source whose
//           sum equals the new value bit for bit, which is what an ascending scan with a strict comparison keeps.
// Steps are processed in chunks whose rows fit local memory; the rows of the next chunk are read into registers
// while the current chunk is worked on, so memory latency is paid once.
#pragma once

#include "plan_kernels.hpp"

namespace parcae {

constexpr int kWaveMaxConfigs = 64;
constexpr int kWaveRowRegs = 8;  // histogram words per thread and histogram that hold the rows of the next chunk

// The candidate table as the kernel takes it (by value, as a kernel argument): the candidates, and per candidate
// its depth group [lo, hi), the slot of the group in the group-aligned layout and the first cell of the group.
struct WaveTable {
    CfgRec rec[kWaveMaxConfigs];
    uint32_t span[kWaveMaxConfigs];  // lo | hi << 8 | slot of the group's first candidate << 16
    uint32_t cell0[kWaveMaxConfigs]; // index of the group's first (source, target) pair in the cell list
};

// How the wave planner lays a candidate list out (the host sizes local memory with it, the kernel indexes with it).
struct WaveGeom {
    int gp;      // size of the largest depth group, rounded up to a multiple of 4
    int ws;      // floats per target row of the same-depth weights: gp + 4 (keeps 16-byte reads of neighbouring rows on different banks)
    int cpad;    // slots of the value function in its group-aligned layout, with gp slots of padding at the end
    int ncells;  // same-depth (source, target) pairs of one step
    uint32_t inv_ncells, inv_C;  // floor(2^32 / d) + 1: (x * inv) >> 32 == x / d for the index ranges of the kernel
};

__host__ __device__ inline int round_up4(int x) { return (x + 3) & ~3; }

__host__ __device__ inline WaveGeom wave_geometry(const CfgRec* rec, int C)
{
    WaveGeom g{0, 0, 0, 0, 0u, 0u};
    int widest = 0, slots = 0;
    for (int i = 0; i < C;) {
        int j = i + 1;
        while (j < C && rec[j].P == rec[i].P) ++j;
        const int size = j - i;
        widest = size > widest ? size : widest;
        slots += round_up4(size);
        g.ncells += size * size;
        i = j;
    }
    g.gp = round_up4(widest);
    g.ws = g.gp + 4;
    g.cpad = slots + g.gp;
    // exact for x < 2^18 and 2 <= d <= 2^12 (x * d < 2^32): at most 63 steps of 4096 pairs or 64 candidates per
    // chunk; d = 1 has no 32-bit reciprocal and is divided by directly (see fast_div)
    g.inv_ncells = g.ncells > 1 ? (uint32_t)(((uint64_t)1 << 32) / (uint32_t)g.ncells) + 1u : 0u;
    g.inv_C = C > 1 ? (uint32_t)(((uint64_t)1 << 32) / (uint32_t)C) + 1u : 0u;
    return g;
}

// x / d by the reciprocal above (inv == 0 stands for d == 1).
__device__ __forceinline__ int fast_div(int x, uint32_t inv) { return inv ? (int)__umulhi((uint32_t)x, inv) : x; }

inline void wave_fill_table(const CfgRec* rec, int C, WaveTable& tb)
{
    int slot = 0, cells = 0;
    for (int i = 0; i < C;) {
        int j = i + 1;
        while (j < C && rec[j].P == rec[i].P) ++j;
        for (int c = i; c < j; ++c) {
            tb.rec[c] = rec[c];
            tb.span[c] = (uint32_t)i | ((uint32_t)j << 8) | ((uint32_t)slot << 16);
            tb.cell0[c] = (uint32_t)cells;
        }
        slot += round_up4(j - i);
        cells += (j - i) * (j - i);
        i = j;
    }
    for (int c = C; c < kWaveMaxConfigs; ++c) {
        tb.rec[c] = CfgRec{1, 1, 0, 0};
        tb.span[c] = 0u;
        tb.cell0[c] = 0u;
    }
}

// Local memory of one workgroup, in bytes: fixed part and the part per step of a chunk.
__host__ __device__ inline size_t wave_fixed_lds(int C, int T, const WaveGeom& g, bool bp_in_lds)
{
    size_t o = sizeof(CfgRec) * (size_t)C;         // cfg
    o += 16 * (size_t)C;                            // target record: full, e[3]
    o += 4 * (size_t)C * 8;                         // full, e[3], rnd[3], R
    o += 4 * (size_t)C * 2;                         // group span, slot of the candidate
    o += 4 * (((size_t)T + 3) & ~(size_t)1);        // availability (even count: the cell list needs 8-byte alignment)
    o += 8 * (size_t)g.ncells;                      // cell list
    o += (size_t)round_up4(g.cpad);                 // candidate of every slot
    o = (o + 15) & ~(size_t)15;
    if (bp_in_lds) o += (2 * (size_t)T * (size_t)C + 15) & ~(size_t)15;
    return o + 32;  // alignment of the per-chunk arrays
}
// `packed`: the two tails of a bin share a word (scenario counts below 2^16, see plan_wave_kernel)
__host__ __device__ inline size_t wave_step_lds(int C, int L, const WaveGeom& g, bool packed)
{
    return (packed ? 4 : 8) * (size_t)L + 4 * (size_t)C * g.ws + 4 * (size_t)g.cpad + 4 * (size_t)C +
           (size_t)round_up4(C);
}

struct WaveShared {
    PlanShared ps;       // cfg, full, e, rnd and the tails: what same_depth_weight() reads
    float* R;            // [C] weight of reaching c from another depth (or from nothing)
    uint32_t* span;      // [C] candidates of the depth of c: first | (one past last) << 8 | slot of the first << 16
    int* slot;           // [C] slot of candidate c in the group-aligned layout of the value function
    int* av;             // [T + 1] availability, clamped to [0, N]
    float4* tgt;         // [C] what a weight needs of its target: full throughput, max(0, tau - cost) of the three classes
    uint2* cell;         // [ncells] same-depth pairs (source c, target c2), ready-made indices:
                         //   x = bin of c's row at the width of c2 (off + min(D2, D)) | first bin of c's row << 16
                         //   y = c2 | (c2 * ws + c - lo) << 8 | c << 24 | (D2 <= D) << 31
    uint8_t* cand;       // [cpad] candidate of every slot of the group-aligned layout, 0xff for padding
    uint16_t* bp16;      // [T][C] back-pointers, or null
    uint32_t* tail_int;  // [Tc][L]
    uint32_t* tail_min;  // [Tc][L]
    float* wsame;        // [Tc][C][ws]
    float* feff;         // [Tc][cpad]
    float* fnew;         // [Tc][C]
    uint8_t* oflag;      // [Tc][C] the new value is reached from another depth (possibly among others)
};

__device__ __forceinline__ void wave_carve(unsigned char* smem, int C, int L, int T, int Tc, const WaveGeom& g,
                                           bool bp_in_lds, bool packed, WaveShared& w)
{
    size_t o = 0;
    w.ps.cfg = reinterpret_cast<CfgRec*>(smem + o); o += sizeof(CfgRec) * (size_t)C;
    w.tgt = reinterpret_cast<float4*>(smem + o); o += 16 * (size_t)C;
    w.ps.full = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)C;
    w.ps.e = reinterpret_cast<float*>(smem + o); o += 12 * (size_t)C;
    w.ps.rnd = reinterpret_cast<float*>(smem + o); o += 12 * (size_t)C;
    w.R = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)C;
    w.span = reinterpret_cast<uint32_t*>(smem + o); o += 4 * (size_t)C;
    w.slot = reinterpret_cast<int*>(smem + o); o += 4 * (size_t)C;
    w.av = reinterpret_cast<int*>(smem + o); o += 4 * (((size_t)T + 3) & ~(size_t)1);
    w.cell = reinterpret_cast<uint2*>(smem + o); o += 8 * (size_t)g.ncells;
    w.cand = reinterpret_cast<uint8_t*>(smem + o); o += (size_t)round_up4(g.cpad);
    o = (o + 15) & ~(size_t)15;
    w.bp16 = nullptr;
    if (bp_in_lds) {
        w.bp16 = reinterpret_cast<uint16_t*>(smem + o);
        o += (2 * (size_t)T * (size_t)C + 15) & ~(size_t)15;
    }
    w.tail_int = reinterpret_cast<uint32_t*>(smem + o); o += 4 * (size_t)Tc * L;  // packed: both tails, int | min << 16
    w.tail_min = reinterpret_cast<uint32_t*>(smem + o); o += packed ? 0 : 4 * (size_t)Tc * L;
    o = (o + 15) & ~(size_t)15;
    w.wsame = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)Tc * C * g.ws;
    w.feff = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)Tc * g.cpad;
    w.fnew = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)Tc * C;
    w.oflag = smem + o;
    w.ps.from_ok = w.ps.to_ok = w.ps.chunk_start = nullptr;
    w.ps.F = w.ps.Feff = w.ps.R = nullptr;
    w.ps.gspan = nullptr;
    w.ps.key = nullptr;
    w.ps.tail_int = w.tail_int;
    w.ps.tail_min = w.tail_min;
    w.ps.bp16 = nullptr;
    w.ps.n_chunks = 1;
    w.ps.tile_log2 = 0;
    w.ps.cold = 0;
}

// The value function holds -inf or non-negative floats (sums of non-negative weights), and on those the signed
// order of the bit patterns is the order of the floats: the cross-lane maxima below are integer maxima, which the
// data-parallel primitives (DPP) feed directly.
constexpr int kNegInfBits = (int)0xff800000u;
constexpr int kIntMin = (int)0x80000000u;

// max(v, value of another lane); lanes without a source lane see the identity of max and keep v.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int dpp_max(int v)
{
    const int moved = __builtin_amdgcn_update_dpp(kIntMin, v, kCtrl, kRowMask, 0xf, false);
    return moved > v ? moved : v;
}

// Inclusive prefix maximum over the 64 lanes: lane i gets the maximum of lanes 0..i.
__device__ __forceinline__ int wave_prefix_max(int v)
{
    v = dpp_max<0x111, 0xf>(v);  // row_shr:1
    v = dpp_max<0x112, 0xf>(v);  // row_shr:2
    v = dpp_max<0x114, 0xf>(v);  // row_shr:4
    v = dpp_max<0x118, 0xf>(v);  // row_shr:8
    v = dpp_max<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    v = dpp_max<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

// Inclusive suffix maximum: lane i gets the maximum of lanes i..63.  Inside a row of 16 lanes by shifts; the rows
// above a lane's own row come in through three lane reads (the data-parallel primitives broadcast upwards only).
__device__ __forceinline__ int wave_suffix_max(int v, int lane)
{
    v = dpp_max<0x101, 0xf>(v);  // row_shl:1
    v = dpp_max<0x102, 0xf>(v);  // row_shl:2
    v = dpp_max<0x104, 0xf>(v);  // row_shl:4
    v = dpp_max<0x108, 0xf>(v);  // row_shl:8
    const int r1 = __builtin_amdgcn_readlane(v, 16), r2 = __builtin_amdgcn_readlane(v, 32);
    const int r3 = __builtin_amdgcn_readlane(v, 48);
    const int r23 = r2 > r3 ? r2 : r3, r123 = r1 > r23 ? r1 : r23;
    const int above = lane < 16 ? r123 : (lane < 32 ? r23 : (lane < 48 ? r3 : kIntMin));
    return above > v ? above : v;
}

__device__ __forceinline__ int lane_value(int v, int src_lane)
{
    return __builtin_amdgcn_ds_bpermute(src_lane << 2, v);
}

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Suffix sums inside a histogram row of D + 1 bins that starts at bin o (slot 0 keeps the raw bin 0), eight bins at
// a time with every load before the first use; the last, partial batch runs on clamped indices with its updates
// predicated, so that there is no one-bin-at-a-time tail.
__device__ __forceinline__ void suffix_row_batched(uint32_t* tail_int, uint32_t* tail_min, int o, int D)
{
    uint32_t ri = 0u, rm = 0u;
    for (int j = D; j >= 1; j -= 8) {
        uint32_t vi[8], vm[8];
        static_for<8>([&](auto x) {
            const int at = j - x.value >= 1 ? j - x.value : 1;
            vi[x.value] = tail_int[o + at];
            vm[x.value] = tail_min[o + at];
        });
        static_for<8>([&](auto x) {
            if (j - x.value >= 1) {
                ri += vi[x.value];
                rm += vm[x.value];
                tail_int[o + j - x.value] = ri;
                tail_min[o + j - x.value] = rm;
            }
        });
    }
}

// The same on rows whose words hold both histograms, hist_int | hist_min << 16: while a unit has fewer than 2^16
// scenarios no partial sum of either half reaches 2^16, so one 32-bit addition adds both halves.
__device__ __forceinline__ void suffix_row_batched_packed(uint32_t* tail, int o, int D)
{
    uint32_t r = 0u;
    for (int j = D; j >= 1; j -= 8) {
        uint32_t v[8];
        static_for<8>([&](auto x) {
            const int at = j - x.value >= 1 ? j - x.value : 1;
            v[x.value] = tail[o + at];
        });
        static_for<8>([&](auto x) {
            if (j - x.value >= 1) {
                r += v[x.value];
                tail[o + j - x.value] = r;
            }
        });
    }
}

// The liveput tables a launch of the planner may write along the way (all null: none).
struct TablesOut {
    float* liveput;
    float* teff;
    float* gain;
};

// One workgroup (1 to 8 waves) per query.  Workgroups past the last query write the liveput tables, one thread per
// unit: they need the finished histograms just as the plan does, and as part of this launch they cost no launch of
// their own.
// kPacked (without transfer rounds, fewer than 2^16 scenarios): the two tails of a bin share a word of local memory,
// which halves the suffix sums and the room the rows of a step take, so that more steps fit a chunk.
template <bool kRounds, bool kPacked>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 8))) plan_wave_kernel(
    Batch b, WaveTable table, WaveGeom g, int Tc, int bp_in_lds, const uint32_t* __restrict__ hist_int,
    const uint32_t* __restrict__ hist_min, float* __restrict__ F, int32_t* __restrict__ bp,
    int32_t* __restrict__ plan, int32_t* __restrict__ start, float* __restrict__ objective,
    int32_t* __restrict__ status, int einval, int einfeasible, TablesOut tables)
{
    if ((int)blockIdx.x >= b.nq) {
        finalise_unit(b, table.rec, ((int64_t)blockIdx.x - b.nq) * blockDim.x + threadIdx.x, hist_int, hist_min,
                      tables.liveput, tables.teff, tables.gain);
        return;
    }
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int bad_inputs;
    WaveShared w;
    const int C = b.C, T = b.T, L = b.L;
    static_assert(!(kRounds && kPacked), "the weights by transfer rounds read the tails one histogram at a time");
    wave_carve(smem, C, L, T, Tc, g, bp_in_lds != 0, kPacked, w);
    const int q = blockIdx.x;
    const int tid = (int)threadIdx.x, nthreads = (int)blockDim.x;
    const int lane = tid & (kWave - 1);
    // the chain runs on one wave; which one rotates with the query, so that the chains of the workgroups that share a
    // compute unit do not all sit on the same SIMD
    const int n_waves = nthreads / kWave;
    const int chain_first = (q % n_waves) * kWave;
    const bool chain_wave = tid >= chain_first && tid < chain_first + kWave;
    const int64_t hist_base = (int64_t)q * T * L;

    // rows of a chunk: n * L consecutive words of each histogram; thread x holds words x, x + nthreads, ...
    uint32_t next_int[kWaveRowRegs], next_min[kWaveRowRegs];
    auto fetch_rows = [&](int t0) __attribute__((always_inline)) {
        const int n = T - t0 < Tc ? T - t0 : Tc;
        const int words = n * L;
        const int64_t base = hist_base + (int64_t)t0 * L;
        static_for<kWaveRowRegs>([&](auto x) {
            const int i = x.value * nthreads + tid;
            const int at = i < words ? i : 0;  // unconditional loads on clamped indices travel together
            next_int[x.value] = hist_int[base + at];
            next_min[x.value] = hist_min[base + at];
        });
    };
    auto stash_rows = [&](int t0) __attribute__((always_inline)) {
        const int n = T - t0 < Tc ? T - t0 : Tc;
        const int words = n * L;
        static_for<kWaveRowRegs>([&](auto x) {
            const int i = x.value * nthreads + tid;
            if (i < words) {
                if constexpr (kPacked) {
                    w.tail_int[i] = next_int[x.value] | (next_min[x.value] << 16);
                } else {
                    w.tail_int[i] = next_int[x.value];
                    w.tail_min[i] = next_min[x.value];
                }
            }
        });
    };
    fetch_rows(0);

    // ---- per-query tables
    if (tid == 0) bad_inputs = 0;
    for (int p = tid; p < g.cpad; p += nthreads) w.cand[p] = 0xffu;  // padding slots hold no candidate
    __syncthreads();
    for (int c = tid; c < C; c += nthreads) {
        const CfgRec cr = table.rec[c];
        w.ps.cfg[c] = cr;
        const float full = b.thr[(int64_t)q * L + cr.off + cr.D];
        const float* co = b.cost + ((int64_t)q * C + c) * 3;
        const float e0 = max0(__fsub_rn(b.tau, co[0])), e1 = max0(__fsub_rn(b.tau, co[1]));
        const float e2 = max0(__fsub_rn(b.tau, co[2]));
        w.tgt[c] = make_float4(full, e0, e1, e2);
        w.ps.full[c] = full;
        w.ps.e[3 * c + 0] = e0;
        w.ps.e[3 * c + 1] = e1;
        w.ps.e[3 * c + 2] = e2;
        w.ps.rnd[3 * c + 0] = co[1];
        w.ps.rnd[3 * c + 1] = co[2];
        w.ps.rnd[3 * c + 2] = b.cost_round ? b.cost_round[(int64_t)q * C + c] : 0.0f;
        w.R[c] = __fmul_rn(full, e2);
        // depth group of c (candidates are sorted by depth): its pairs in the cell list, its slot
        const uint32_t sp = table.span[c];
        const int lo = (int)(sp & 0xffu), hi = (int)((sp >> 8) & 0xffu);
        const int slot = (int)(sp >> 16) + c - lo;
        w.span[c] = sp;
        w.slot[c] = slot;
        w.cand[slot] = (uint8_t)c;
        const int size = hi - lo, cells = (int)table.cell0[c];
        for (int i = 0; i < size; ++i) {
            const int c2 = lo + i, D2 = table.rec[c2].D;
            const uint32_t x = (uint32_t)(cr.off + (D2 <= cr.D ? D2 : cr.D)) | ((uint32_t)cr.off << 16);
            const uint32_t y = (uint32_t)c2 | ((uint32_t)(c2 * g.ws + c - lo) << 8) | ((uint32_t)c << 24) |
                               (D2 <= cr.D ? 0x80000000u : 0u);
            w.cell[cells + (c - lo) * size + i] = make_uint2(x, y);
        }
    }
    for (int t = tid; t <= T; t += nthreads) w.av[t] = clampi(b.avail[(int64_t)q * b.avail_stride + t], 0, b.N);
    for (int i = tid; i < Tc * C * g.ws; i += nthreads) w.wsame[i] = kNegInf;  // padding of the weight rows stays -inf
    for (int i = tid; i < Tc * g.cpad; i += nthreads) w.feff[i] = kNegInf;      // padding slots of the value function too
    const int cur = b.cur_config ? b.cur_config[q] : -1;
    const bool cold = cur == -2;

    // ---- lane state of the chain (lane = candidate)
    const int lc = lane < C ? lane : C - 1;  // lanes past the list compute on the last candidate and store nothing
    const bool is_cand = chain_wave && lane < C;
    const CfgRec mine = table.rec[lc];
    const int used = mine.D * mine.P;
    const bool deep = mine.P >= b.p_min;
    float Fcur = 0.0f;
    float* Fq = F ? F + (int64_t)q * (T + 1) * C : nullptr;
    int32_t* bpq = bp ? bp + (int64_t)q * T * C : nullptr;
    if (Fq && is_cand) Fq[lane] = 0.0f;
    __syncthreads();
    // the input checks wait on memory: the waves that do not carry the chain run them while the first chain runs
    // (a workgroup of one wave runs them here)
    auto check_inputs = [&](int rank, int count) __attribute__((always_inline)) {
        if (query_inputs_bad(b, w.ps.cfg, q, rank, count)) atomicOr(&bad_inputs, 1);
    };
    if (n_waves == 1) check_inputs(tid, nthreads);

    for (int t0 = 0; t0 < T; t0 += Tc) {
        const int n = T - t0 < Tc ? T - t0 : Tc;
        stash_rows(t0);
        __syncthreads();
        if (t0 + Tc < T) fetch_rows(t0 + Tc);
        // suffix sums inside every row of the chunk
        for (int row = tid; row < n * C; row += nthreads) {
            const int ti = fast_div(row, g.inv_C);
            const CfgRec cr = w.ps.cfg[row - ti * C];
            if constexpr (kPacked) suffix_row_batched_packed(w.tail_int, ti * L + cr.off, cr.D);
            else suffix_row_batched(w.tail_int, w.tail_min, ti * L + cr.off, cr.D);
        }
        __syncthreads();
        // phase A: weights of the same-depth transitions, four pairs per thread at a time (the loads of the four
        // travel together); what is left for a last round of at most two per thread is done two at a time
        const int n_pairs = n * g.ncells;
        auto weights_of = [&](auto width, int e0) __attribute__((always_inline)) {
            constexpr int kW = decltype(width)::value;
            int ti[kW];
            uint2 cell[kW];
            bool live[kW];
            static_for<kW>([&](auto k) {
                const int e = e0 + k.value * nthreads;
                live[k.value] = e < n_pairs;
                const int ec = live[k.value] ? e : e0;
                ti[k.value] = fast_div(ec, g.inv_ncells);
                cell[k.value] = w.cell[ec - ti[k.value] * g.ncells];
            });
            float wt[kW];
            if constexpr (kRounds) {
                static_for<kW>([&](auto k) {
                    PlanShared ps = w.ps;
                    ps.tail_int = w.tail_int + ti[k.value] * L;
                    ps.tail_min = w.tail_min + ti[k.value] * L;
                    wt[k.value] = same_depth_weight<true>(b, ps, 0, (int)((cell[k.value].y >> 24) & 0x3fu),
                                                          (int)(cell[k.value].y & 0xffu));
                });
            } else {
                uint32_t t_int[kW], t_min[kW], h0[kW];
                float4 tg[kW];
                static_for<kW>([&](auto k) {
                    const uint32_t* ri = w.tail_int + ti[k.value] * L;
                    if constexpr (kPacked) {
                        t_int[k.value] = ri[cell[k.value].x & 0xffffu];  // both tails; taken apart below
                        h0[k.value] = ri[cell[k.value].x >> 16];
                    } else {
                        const uint32_t* rm = w.tail_min + ti[k.value] * L;
                        t_int[k.value] = ri[cell[k.value].x & 0xffffu];
                        t_min[k.value] = rm[cell[k.value].x & 0xffffu];
                        h0[k.value] = rm[cell[k.value].x >> 16];
                    }
                    tg[k.value] = w.tgt[cell[k.value].y & 0xffu];
                });
                if constexpr (kPacked) {
                    static_for<kW>([&](auto k) {
                        t_min[k.value] = t_int[k.value] >> 16;
                        t_int[k.value] &= 0xffffu;
                        h0[k.value] >>= 16;
                    });
                }
                static_for<kW>([&](auto k) {
                    // a target wider than the source keeps nothing (the width of a target is at least 1)
                    const bool keep = (cell[k.value].y & 0x80000000u) != 0u;
                    const uint32_t n0 = keep ? t_int[k.value] : 0u, n01 = keep ? t_min[k.value] : 0u;
                    wt[k.value] = __fmul_rn(tg[k.value].x, teff_from_counts(n0, n01, h0[k.value], 1, (uint32_t)b.S, b.tau,
                                                                            tg[k.value].y, tg[k.value].z, tg[k.value].w));
                });
            }
            static_for<kW>([&](auto k) {
                if (live[k.value]) w.wsame[ti[k.value] * C * g.ws + (int)((cell[k.value].y >> 8) & 0xffffu)] = wt[k.value];
            });
        };
        {
            int e0 = tid;
            for (; e0 + 2 * nthreads < n_pairs; e0 += 4 * nthreads) weights_of(std::integral_constant<int, 4>{}, e0);
            if (e0 < n_pairs) weights_of(std::integral_constant<int, 2>{}, e0);
        }
        __syncthreads();
        // chain: values only
        if (chain_wave) {
            const uint32_t sp = w.span[lc];
            const int lo = (int)(sp & 0xffu), hi = (int)((sp >> 8) & 0xffu);
            const int gslot = (int)(sp >> 16);
            const float reach = w.R[lc];
            const int n4 = g.gp / 4;
            // whether this lane's candidate may be left / entered at each step of the chunk (constraint D * P <= N of
            // Eq. 6, memory floor, the current configuration at t = 0), one bit per step, before the dependent steps
            uint32_t from_bits = 0u, to_bits = 0u;  // a chunk has at most 32 steps
            for (int ti = 0; ti < n; ++ti) {
                const int t = t0 + ti;
                const bool from = used <= b.group * w.av[t] && deep && (t > 0 || cur < 0 || lane == cur);
                const bool to = used <= b.group * w.av[t + 1] && deep;
                from_bits |= (uint32_t)(from && is_cand) << ti;
                to_bits |= (uint32_t)to << ti;
            }
            for (int ti = 0; ti < n; ++ti) {
                const int t = t0 + ti;
                const bool from = (from_bits >> ti) & 1u;
                const bool to = (to_bits >> ti) & 1u;
                const float fe = from ? Fcur : kNegInf;
                float* frow = w.feff + ti * g.cpad;
                if (is_cand) frow[gslot + lane - lo] = fe;
                float fn, other;
                if (t == 0 && cold) {
                    other = __fadd_rn(0.0f, reach);  // nothing is running: c' comes up from nothing at its re-partition cost
                    fn = other;
                } else {
                    wave_sync();  // the values of this step are in local memory
                    // same depth, first 16 sources: the loads go out before anything else (indices clamped: a source
                    // taken twice does not change a maximum)
                    const float4* f4 = reinterpret_cast<const float4*>(frow + gslot);
                    const float4* w4 = reinterpret_cast<const float4*>(w.wsame + (ti * C + lc) * g.ws);
                    float4 f[4], x[4];
                    static_for<4>([&](auto k) {
                        const int i = k.value < n4 ? k.value : n4 - 1;
                        f[k.value] = f4[i];
                        x[k.value] = w4[i];
                    });
                    // largest value among the candidates of other depths: those before the group and those after it
                    const int fb = __float_as_int(fe);
                    const int pm = wave_prefix_max(fb);
                    const int sm = wave_suffix_max(fb, lane);
                    const int before = lane_value(pm, lo > 0 ? lo - 1 : 0);
                    const int after = lane_value(sm, hi < kWave ? hi : 0);
                    const int ob = lo > 0 ? before : kNegInfBits, oa = hi < kWave ? after : kNegInfBits;
                    other = __fadd_rn(__int_as_float(ob > oa ? ob : oa), reach);
                    // the maximum as a tree (a maximum does not depend on the order): the step waits for the deepest
                    // path of dependent instructions, not for their number
                    float m[4];
                    static_for<4>([&](auto k) {
                        const float s0 = __fadd_rn(f[k.value].x, x[k.value].x), s1 = __fadd_rn(f[k.value].y, x[k.value].y);
                        const float s2 = __fadd_rn(f[k.value].z, x[k.value].z), s3 = __fadd_rn(f[k.value].w, x[k.value].w);
                        m[k.value] = __builtin_fmaxf(__builtin_fmaxf(s0, s1), __builtin_fmaxf(s2, s3));
                    });
                    fn = __builtin_fmaxf(__builtin_fmaxf(__builtin_fmaxf(m[0], m[1]), __builtin_fmaxf(m[2], m[3])), other);
                    for (int i0 = 4; i0 < n4; i0 += 4) {  // depth groups of more than 16 candidates
                        static_for<4>([&](auto k) {
                            const int i = i0 + k.value < n4 ? i0 + k.value : n4 - 1;
                            f[k.value] = f4[i];
                            x[k.value] = w4[i];
                        });
                        static_for<4>([&](auto k) {
                            const float s0 = __fadd_rn(f[k.value].x, x[k.value].x), s1 = __fadd_rn(f[k.value].y, x[k.value].y);
                            const float s2 = __fadd_rn(f[k.value].z, x[k.value].z), s3 = __fadd_rn(f[k.value].w, x[k.value].w);
                            fn = __builtin_fmaxf(__builtin_fmaxf(fn, s0), s1);
                            fn = __builtin_fmaxf(__builtin_fmaxf(fn, s2), s3);
                        });
                    }
                }
                const bool from_other = to && other == fn;
                fn = to ? fn : kNegInf;
                if (is_cand) {
                    w.fnew[ti * C + lane] = fn;
                    w.oflag[ti * C + lane] = from_other ? 1u : 0u;
                    if (Fq) Fq[(int64_t)(t + 1) * C + lane] = fn;
                }
                Fcur = fn;
            }
        } else if (t0 == 0 && n_waves > 1) {
            check_inputs(tid < chain_first ? tid : tid - kWave, nthreads - kWave);
        }
        __syncthreads();
        // phase C: back-pointers.  The sources sit in slot order, which is candidate order, so the smallest matching
        // slot is the smallest matching candidate; scans run downwards and keep the last match.
        for (int item0 = 0; item0 < n * C; item0 += nthreads) {
            const int item = item0 + tid;
            const bool live = item < n * C;
            const int it = live ? item : 0;
            const int ti = fast_div(it, g.inv_C), c2 = it - ti * C;
            const int t = t0 + ti;
            const float fn = w.fnew[it];
            const bool reached = live && fn > kNegInf;
            const bool cold_step = t == 0 && cold;
            const uint32_t sp = w.span[c2];
            const int gslot = (int)(sp >> 16);
            const int gsize4 = round_up4((int)((sp >> 8) & 0xffu) - (int)(sp & 0xffu));
            const float4* frow4 = reinterpret_cast<const float4*>(w.feff + ti * g.cpad);
            int best = 0x7fffffff;
            // other depths: only where the chain saw the new value come from another depth (rare after the first step)
            const bool want_other = reached && !cold_step && w.oflag[it] != 0u;
            if (__any(want_other)) {
                const float reach = w.R[c2];
                const int n_blocks = (g.cpad - g.gp) / 4;
                for (int p0 = n_blocks - 1; p0 >= 0; p0 -= 4) {
                    float4 f[4];
                    static_for<4>([&](auto k) { f[k.value] = frow4[p0 - k.value >= 0 ? p0 - k.value : 0]; });
                    static_for<4>([&](auto k) {
                        const int p = (p0 - k.value >= 0 ? p0 - k.value : 0) * 4;
                        const bool own = (unsigned)(p - gslot) < (unsigned)gsize4;  // blocks of four slots never straddle groups
                        if (!own) {
                            if (__fadd_rn(f[k.value].w, reach) == fn) best = p + 3;
                            if (__fadd_rn(f[k.value].z, reach) == fn) best = p + 2;
                            if (__fadd_rn(f[k.value].y, reach) == fn) best = p + 1;
                            if (__fadd_rn(f[k.value].x, reach) == fn) best = p;
                        }
                    });
                }
                best = want_other ? best : 0x7fffffff;
            }
            // same depth
            {
                const float4* fg4 = frow4 + gslot / 4;
                const float4* wr4 = reinterpret_cast<const float4*>(w.wsame + (ti * C + c2) * g.ws);
                int best_in = 0x7fffffff;
                for (int i0 = g.gp / 4 - 1; i0 >= 0; i0 -= 4) {
                    float4 f[4], x[4];
                    static_for<4>([&](auto k) {
                        const int i = i0 - k.value >= 0 ? i0 - k.value : 0;
                        f[k.value] = fg4[i];
                        x[k.value] = wr4[i];
                    });
                    static_for<4>([&](auto k) {
                        const int i = (i0 - k.value >= 0 ? i0 - k.value : 0) * 4;
                        if (__fadd_rn(f[k.value].w, x[k.value].w) == fn) best_in = i + 3;
                        if (__fadd_rn(f[k.value].z, x[k.value].z) == fn) best_in = i + 2;
                        if (__fadd_rn(f[k.value].y, x[k.value].y) == fn) best_in = i + 1;
                        if (__fadd_rn(f[k.value].x, x[k.value].x) == fn) best_in = i;
                    });
                }
                if (best_in != 0x7fffffff && gslot + best_in < best) best = gslot + best_in;
            }
            int arg = -1;
            if (reached) {
                if (cold_step) arg = c2;
                else if (best != 0x7fffffff) arg = (int)w.cand[best];
            }
            if (live) {
                if (bpq) bpq[(int64_t)t * C + c2] = arg;
                if (w.bp16) w.bp16[t * C + c2] = arg < 0 ? kNoPred16 : (uint16_t)arg;
            }
        }
        __syncthreads();
    }

    // ---- final arg-max (smallest index on ties) and walk back
    if (chain_wave) {
        const float fl = is_cand ? Fcur : kNegInf;
        const float top = __int_as_float(lane_value(wave_prefix_max(__float_as_int(fl)), kWave - 1));
        const unsigned long long at_top = __ballot(is_cand && fl == top && top > kNegInf);
        int last = at_top ? (int)__builtin_ctzll(at_top) : -1;  // the same in every lane
        int32_t* pl = plan + (int64_t)q * T;
        int st = 0;
        if (last < 0) {
            for (int t = lane; t < T; t += kWave) pl[t] = -1;
            if (lane == 0 && start) start[q] = -1;
            st = einfeasible;
        } else if (w.bp16) {
            // walk back with the back-pointers of a step spread over the lanes (lane = candidate): following a
            // pointer is one lane read, the row of the next step is loaded while the current one is followed, and
            // lane t collects plan[t] so that the plan goes out in whole rows
            for (int hi = T; hi > 0; hi -= kWave) {          // steps [lo, hi) at a time, latest first
                const int lo = hi > kWave ? hi - kWave : 0;
                int mine = -1;
                for (int t = hi - 1; t >= lo; t -= 4) {      // four rows per round of loads
                    int row[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) row[j] = (int)w.bp16[(t - j > 0 ? t - j : 0) * C + lc];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (t - j < lo) break;
                        mine = lane == t - j - lo ? last : mine;  // plan[t] = the candidate the walk is at
                        const int prev = __builtin_amdgcn_readlane(row[j], last);
                        last = prev == (int)kNoPred16 ? 0 : prev;  // cannot happen on a finite path; keeps the walk in bounds
                    }
                }
                if (lo + lane < hi) pl[lo + lane] = mine;
            }
            if (lane == 0 && start) start[q] = last;
        } else if (lane == 0) {
            pl[T - 1] = last;
            for (int t = T - 1; t >= 0; --t) {
                int prev = bpq[(int64_t)t * C + last];
                if (prev < 0) prev = 0;  // cannot happen on a finite path; keeps the walk in bounds
                if (t >= 1) pl[t - 1] = prev;
                else if (start) start[q] = prev;
                last = prev;
            }
        }
        if (lane == 0) {
            if (objective) objective[q] = top;
            if (status) status[q] = bad_inputs ? einval : st;
        }
    }
}

}  // namespace parcae
