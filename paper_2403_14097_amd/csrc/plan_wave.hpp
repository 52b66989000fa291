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
constexpr int kWaveRowRegs = 24;  // histogram words per thread and histogram that hold the rows of the next chunk

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
};

__host__ __device__ inline int round_up4(int x) { return (x + 3) & ~3; }

__host__ __device__ inline WaveGeom wave_geometry(const CfgRec* rec, int C)
{
    WaveGeom g{0, 0, 0, 0};
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
    return g;
}

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
    o += 4 * (size_t)C * 8;                         // full, e[3], rnd[3], R
    o += 4 * (size_t)C * 2;                         // group span, slot of the candidate
    o += 4 * ((size_t)T + 2);                       // availability
    o += 2 * (size_t)round_up4(g.ncells);           // cell list
    o = (o + 15) & ~(size_t)15;
    if (bp_in_lds) o += (2 * (size_t)T * (size_t)C + 15) & ~(size_t)15;
    return o + 32;  // alignment of the per-chunk arrays
}
__host__ __device__ inline size_t wave_step_lds(int C, int L, const WaveGeom& g)
{
    return 8 * (size_t)L + 4 * (size_t)C * g.ws + 4 * (size_t)g.cpad + 4 * (size_t)C;
}

struct WaveShared {
    PlanShared ps;       // cfg, full, e, rnd and the tails: what same_depth_weight() reads
    float* R;            // [C] weight of reaching c from another depth (or from nothing)
    uint32_t* span;      // [C] candidates of the depth of c: first | (one past last) << 8 | slot of the first << 16
    int* slot;           // [C] slot of candidate c in the group-aligned layout of the value function
    int* av;             // [T + 1] availability, clamped to [0, N]
    uint16_t* cell;      // [ncells] same-depth pairs: source | target << 8
    uint16_t* bp16;      // [T][C] back-pointers, or null
    uint32_t* tail_int;  // [Tc][L]
    uint32_t* tail_min;  // [Tc][L]
    float* wsame;        // [Tc][C][ws]
    float* feff;         // [Tc][cpad]
    float* fnew;         // [Tc][C]
};

__device__ __forceinline__ void wave_carve(unsigned char* smem, int C, int L, int T, int Tc, const WaveGeom& g,
                                           bool bp_in_lds, WaveShared& w)
{
    size_t o = 0;
    w.ps.cfg = reinterpret_cast<CfgRec*>(smem + o); o += sizeof(CfgRec) * (size_t)C;
    w.ps.full = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)C;
    w.ps.e = reinterpret_cast<float*>(smem + o); o += 12 * (size_t)C;
    w.ps.rnd = reinterpret_cast<float*>(smem + o); o += 12 * (size_t)C;
    w.R = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)C;
    w.span = reinterpret_cast<uint32_t*>(smem + o); o += 4 * (size_t)C;
    w.slot = reinterpret_cast<int*>(smem + o); o += 4 * (size_t)C;
    w.av = reinterpret_cast<int*>(smem + o); o += 4 * ((size_t)T + 2);
    w.cell = reinterpret_cast<uint16_t*>(smem + o); o += 2 * (size_t)round_up4(g.ncells);
    o = (o + 15) & ~(size_t)15;
    w.bp16 = nullptr;
    if (bp_in_lds) {
        w.bp16 = reinterpret_cast<uint16_t*>(smem + o);
        o += (2 * (size_t)T * (size_t)C + 15) & ~(size_t)15;
    }
    w.tail_int = reinterpret_cast<uint32_t*>(smem + o); o += 4 * (size_t)Tc * L;
    w.tail_min = reinterpret_cast<uint32_t*>(smem + o); o += 4 * (size_t)Tc * L;
    o = (o + 15) & ~(size_t)15;
    w.wsame = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)Tc * C * g.ws;
    w.feff = reinterpret_cast<float*>(smem + o); o += 4 * (size_t)Tc * g.cpad;
    w.fnew = reinterpret_cast<float*>(smem + o);
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
// data-parallel primitives (DPP) can feed directly.
constexpr int kNegInfBits = (int)0xff800000u;

// max(v, value of another lane); lanes without a source lane keep v.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int dpp_max(int v)
{
    const int moved = __builtin_amdgcn_update_dpp(v, v, kCtrl, kRowMask, 0xf, false);
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

__device__ __forceinline__ int lane_value(int v, int src_lane)
{
    return __builtin_amdgcn_ds_bpermute(src_lane << 2, v);
}

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// One workgroup (1 to 8 waves) per query.
template <bool kRounds>
__global__ void __launch_bounds__(512) plan_wave_kernel(
    Batch b, WaveTable table, WaveGeom g, int Tc, int bp_in_lds, const uint32_t* __restrict__ hist_int,
    const uint32_t* __restrict__ hist_min, float* __restrict__ F, int32_t* __restrict__ bp,
    int32_t* __restrict__ plan, int32_t* __restrict__ start, float* __restrict__ objective,
    int32_t* __restrict__ status, int einval, int einfeasible)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int bad_inputs;
    WaveShared w;
    const int C = b.C, T = b.T, L = b.L;
    wave_carve(smem, C, L, T, Tc, g, bp_in_lds != 0, w);
    const int q = blockIdx.x;
    const int tid = (int)threadIdx.x, nthreads = (int)blockDim.x;
    const int lane = tid & (kWave - 1);
    const bool chain_wave = tid < kWave;
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
                w.tail_int[i] = next_int[x.value];
                w.tail_min[i] = next_min[x.value];
            }
        });
    };
    fetch_rows(0);

    // ---- per-query tables
    if (tid == 0) bad_inputs = 0;
    for (int c = tid; c < C; c += nthreads) {
        const CfgRec cr = table.rec[c];
        w.ps.cfg[c] = cr;
        const float full = b.thr[(int64_t)q * L + cr.off + cr.D];
        const float* co = b.cost + ((int64_t)q * C + c) * 3;
        const float e2 = max0(__fsub_rn(b.tau, co[2]));
        w.ps.full[c] = full;
        w.ps.e[3 * c + 0] = max0(__fsub_rn(b.tau, co[0]));
        w.ps.e[3 * c + 1] = max0(__fsub_rn(b.tau, co[1]));
        w.ps.e[3 * c + 2] = e2;
        w.ps.rnd[3 * c + 0] = co[1];
        w.ps.rnd[3 * c + 1] = co[2];
        w.ps.rnd[3 * c + 2] = b.cost_round ? b.cost_round[(int64_t)q * C + c] : 0.0f;
        w.R[c] = __fmul_rn(full, e2);
        // depth group of c (candidates are sorted by depth): its pairs in the cell list
        const uint32_t sp = table.span[c];
        const int lo = (int)(sp & 0xffu), hi = (int)((sp >> 8) & 0xffu);
        w.span[c] = sp;
        w.slot[c] = (int)(sp >> 16) + c - lo;
        const int size = hi - lo, cells = (int)table.cell0[c];
        for (int i = 0; i < size; ++i) w.cell[cells + (c - lo) * size + i] = (uint16_t)(c | ((lo + i) << 8));
    }
    for (int t = tid; t <= T; t += nthreads) w.av[t] = clampi(b.avail[(int64_t)q * b.avail_stride + t], 0, b.N);
    for (int i = tid; i < Tc * C * g.ws; i += nthreads) w.wsame[i] = kNegInf;  // padding of the weight rows stays -inf
    for (int i = tid; i < Tc * g.cpad; i += nthreads) w.feff[i] = kNegInf;      // padding slots of the value function too
    __syncthreads();
    if (query_inputs_bad(b, w.ps.cfg, q, tid, nthreads)) atomicOr(&bad_inputs, 1);
    const int cur = b.cur_config ? b.cur_config[q] : -1;
    const bool cold = cur == -2;

    // ---- lane state of the chain (wave 0; lane = candidate)
    const int lc = lane < C ? lane : C - 1;  // lanes past the list compute on the last candidate and store nothing
    const bool is_cand = chain_wave && lane < C;
    const CfgRec mine = table.rec[lc];
    const int used = mine.D * mine.P;
    const bool deep = mine.P >= b.p_min;
    float Fcur = 0.0f;
    float* Fq = F ? F + (int64_t)q * (T + 1) * C : nullptr;
    int32_t* bpq = bp ? bp + (int64_t)q * T * C : nullptr;
    if (Fq && is_cand) Fq[lane] = 0.0f;

    for (int t0 = 0; t0 < T; t0 += Tc) {
        const int n = T - t0 < Tc ? T - t0 : Tc;
        stash_rows(t0);
        __syncthreads();
        if (t0 + Tc < T) fetch_rows(t0 + Tc);
        // suffix sums inside every row of the chunk
        for (int row = tid; row < n * C; row += nthreads) {
            const int ti = row / C;
            const CfgRec cr = w.ps.cfg[row - ti * C];
            suffix_row(w.ps, cr, ti * L + cr.off);
        }
        __syncthreads();
        // phase A: weights of the same-depth transitions
        for (int e = tid; e < n * g.ncells; e += nthreads) {
            const int ti = e / g.ncells;
            const uint32_t pair = w.cell[e - ti * g.ncells];
            const int c = (int)(pair & 0xffu), c2 = (int)(pair >> 8);
            PlanShared ps = w.ps;
            ps.tail_int = w.tail_int + ti * L;
            ps.tail_min = w.tail_min + ti * L;
            const float wt = same_depth_weight<kRounds>(b, ps, 0, c, c2);
            w.wsame[(ti * C + c2) * g.ws + (c - (int)(w.span[c2] & 0xffu))] = wt;
        }
        __syncthreads();
        // chain: values only
        if (chain_wave) {
            const uint32_t sp = w.span[lc];
            const int lo = (int)(sp & 0xffu), hi = (int)((sp >> 8) & 0xffu);
            const int gslot = (int)(sp >> 16);
            const float reach = w.R[lc];
            const int n4 = g.gp / 4;
            const int av_mine = w.av[t0 + lane <= T ? t0 + lane : T];  // lane i holds the availability of step t0 + i
            for (int ti = 0; ti < n; ++ti) {
                const int t = t0 + ti;
                const int a_prev = b.group * __builtin_amdgcn_readlane(av_mine, ti);
                const int a_next = b.group * __builtin_amdgcn_readlane(av_mine, ti + 1);
                const bool from = is_cand && used <= a_prev && deep && (t > 0 || cur < 0 || lane == cur);
                const bool to = used <= a_next && deep;
                const float fe = from ? Fcur : kNegInf;
                float* frow = w.feff + ti * g.cpad;
                if (is_cand) frow[gslot + lane - lo] = fe;
                float fn;
                if (t == 0 && cold) {
                    fn = __fadd_rn(0.0f, reach);  // nothing is running: c' comes up from nothing at its re-partition cost
                } else {
                    // largest value among the candidates of other depths: those before the group and those after it
                    const int fb = __float_as_int(fe);
                    const int pm = wave_prefix_max(fb);
                    const int sm = wave_prefix_max(lane_value(fb, kWave - 1 - lane));
                    const int before = lane_value(pm, lo > 0 ? lo - 1 : 0);
                    const int after = lane_value(sm, hi < kWave ? kWave - 1 - hi : 0);
                    const int ob = lo > 0 ? before : kNegInfBits, oa = hi < kWave ? after : kNegInfBits;
                    fn = __fadd_rn(__int_as_float(ob > oa ? ob : oa), reach);
                    wave_sync();  // the group's values are in local memory
                    // same depth: 16 sources at a time, every load before the first use (indices clamped: a source
                    // taken twice does not change a maximum)
                    const float4* f4 = reinterpret_cast<const float4*>(frow + gslot);
                    const float4* w4 = reinterpret_cast<const float4*>(w.wsame + (ti * C + lc) * g.ws);
                    for (int i0 = 0; i0 < n4; i0 += 4) {
                        float4 f[4], x[4];
                        static_for<4>([&](auto k) {
                            const int i = i0 + k.value < n4 ? i0 + k.value : n4 - 1;
                            f[k.value] = f4[i];
                            x[k.value] = w4[i];
                        });
                        static_for<4>([&](auto k) {
                            const float s0 = __fadd_rn(f[k.value].x, x[k.value].x), s1 = __fadd_rn(f[k.value].y, x[k.value].y);
                            const float s2 = __fadd_rn(f[k.value].z, x[k.value].z), s3 = __fadd_rn(f[k.value].w, x[k.value].w);
                            fn = __builtin_fmaxf(fn, __builtin_fmaxf(s0, s1));
                            fn = __builtin_fmaxf(fn, __builtin_fmaxf(s2, s3));
                        });
                    }
                }
                fn = to ? fn : kNegInf;
                if (is_cand) {
                    w.fnew[ti * C + lane] = fn;
                    if (Fq) Fq[(int64_t)(t + 1) * C + lane] = fn;
                }
                Fcur = fn;
            }
        }
        __syncthreads();
        // phase C: back-pointers
        for (int item = tid; item < n * C; item += nthreads) {
            const int ti = item / C, c2 = item - ti * C;
            const int t = t0 + ti;
            const float fn = w.fnew[ti * C + c2];
            int arg = -1;
            if (fn > kNegInf) {
                if (t == 0 && cold) {
                    arg = c2;
                } else {
                    const uint32_t sp = w.span[c2];
                    const int lo = (int)(sp & 0xffu), hi = (int)((sp >> 8) & 0xffu);
                    const float reach = w.R[c2];
                    const float* frow = w.feff + ti * g.cpad;
                    int best = kWaveMaxConfigs;
                    // other depths, descending: the last match kept is the smallest
                    for (int c = C - 1; c >= 0; --c) {
                        const float v = __fadd_rn(frow[w.slot[c]], reach);
                        if ((c < lo || c >= hi) && v == fn) best = c;
                    }
                    // same depth
                    const float* fg = frow + (int)(sp >> 16);
                    const float* wr = w.wsame + (ti * C + c2) * g.ws;
                    int best_in = kWaveMaxConfigs;
                    for (int i = hi - lo - 1; i >= 0; --i)
                        if (__fadd_rn(fg[i], wr[i]) == fn) best_in = lo + i;
                    best = best_in < best ? best_in : best;
                    arg = best < kWaveMaxConfigs ? best : -1;
                }
            }
            if (bpq) bpq[(int64_t)t * C + c2] = arg;
            if (w.bp16) w.bp16[t * C + c2] = arg < 0 ? kNoPred16 : (uint16_t)arg;
        }
        __syncthreads();
    }

    // ---- final arg-max (smallest index on ties) and walk back
    if (chain_wave) {
        const float fl = is_cand ? Fcur : kNegInf;
        const float top = __int_as_float(lane_value(wave_prefix_max(__float_as_int(fl)), kWave - 1));
        const unsigned long long at_top = __ballot(is_cand && fl == top && top > kNegInf);
        if (lane == 0) {
            int last = at_top ? (int)__builtin_ctzll(at_top) : -1;
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
                    if (w.bp16) {
                        const uint16_t v = w.bp16[t * C + last];
                        prev = v == kNoPred16 ? -1 : (int)v;
                    } else {
                        prev = bpq[(int64_t)t * C + last];
                    }
                    if (prev < 0) prev = 0;  // cannot happen on a finite path; keeps the walk in bounds
                    if (t >= 1) pl[t - 1] = prev;
                    else if (start) start[q] = prev;
                    last = prev;
                }
            }
            if (objective) objective[q] = top;
            if (status) status[q] = bad_inputs ? einval : st;
        }
    }
}

}  // namespace parcae
