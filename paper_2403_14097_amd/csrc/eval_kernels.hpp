// Scenario sampler, survivor reducer and histogram kernels (section 6.3, section 5.2).
//
// One lane owns one scenario: Floyd's subset loop carries a dependence on the
// growing set, so it cannot be spread over lanes, but all 64 lanes of a wave
// work on the same unit (q, t, c), which keeps D, P, M, k and every loop trip
// count in scalar registers.  A 256-bit preemption mask lives in NW 32-bit
// vector registers per lane (NW = 1, 2, 4 or 8 by the unit's size).
#pragma once

#include <utility>

#include "device_common.hpp"

namespace parcae {

// ------------------------------------------------------------------ Philox4x32-10

struct Philox4 {
    uint32_t x[4];
};

// The ten round keys of a query (key bumped by the Weyl constants of Salmon et al., SC'11), held in
// vector registers: on gfx950 a bitwise VALU instruction with a scalar-register operand issues at half
// the rate of one whose operands are all vector registers, and the round keys are used by every block.
struct PhiloxKeys {
    uint32_t a[10];
    uint32_t b[10];
};

__device__ __forceinline__ uint32_t in_vgpr(uint32_t uniform_value)
{
    uint32_t v;
    asm volatile("v_mov_b32 %0, %1" : "=v"(v) : "s"(uniform_value));
    return v;
}

__device__ __forceinline__ PhiloxKeys philox_keys(uint32_t k0, uint32_t k1)
{
    PhiloxKeys ks;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        ks.a[r] = in_vgpr(k0 + (uint32_t)r * 0x9E3779B9u);
        ks.b[r] = in_vgpr(k1 + (uint32_t)r * 0xBB67AE85u);
    }
    return ks;
}

// a ^ b ^ c in one instruction
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// One block: counter (c0..c3), ten rounds with multipliers 0xD2511F53 and 0xCD9E8D57.
__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 const PhiloxKeys& ks)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t pa = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = xor3((uint32_t)(pb >> 32), c1, ks.a[round]);
        const uint32_t n2 = xor3((uint32_t)(pa >> 32), c3, ks.b[round]);
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
    }
    Philox4 r;
    r.x[0] = c0; r.x[1] = c1; r.x[2] = c2; r.x[3] = c3;
    return r;
}

// ------------------------------------------------------------------ bit set in registers

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

template <int NW>
struct Mask {
    uint32_t w[NW];

    __device__ __forceinline__ void clear()
    {
        static_for<NW>([&](auto i) { w[i.value] = 0u; });
    }
    // bit b (per-lane value) set?
    __device__ __forceinline__ bool test(uint32_t b) const
    {
        const uint32_t sel = b >> 5;
        uint32_t word = w[0];
        static_for<NW>([&](auto i) {
            if constexpr (i.value > 0) word = (sel == (uint32_t)i.value) ? w[i.value] : word;
        });
        return (word >> (b & 31u)) & 1u;
    }
    __device__ __forceinline__ void set(uint32_t b)
    {
        const uint32_t sel = b >> 5;
        const uint32_t bit = 1u << (b & 31u);
        static_for<NW>([&](auto i) { w[i.value] |= (sel == (uint32_t)i.value) ? bit : 0u; });
    }
    // keep bits [0, M) of the complement
    __device__ __forceinline__ void complement(int M)
    {
        static_for<NW>([&](auto i) {
            constexpr int lo = i.value * 32;
            const uint32_t valid = (M >= lo + 32) ? 0xffffffffu : (M <= lo ? 0u : ((1u << (M - lo)) - 1u));
            w[i.value] = ~w[i.value] & valid;
        });
    }
};

// ------------------------------------------------------------------ sampler

// Floyd's step on a set held in registers, written without selects: setting bit r always happens; if r
// was already present the step also sets bit j (never present before: j exceeds every earlier draw).
// `hit` is all-ones or zero, the bit of j is the same in every lane.

// Preempted set of scenario s of a unit with M <= 32 (one word).
__device__ __forceinline__ void sample_mask(Mask<1>& mask, int M, int k, uint32_t s, uint32_t unit,
                                            uint32_t stream_id, const PhiloxKeys& ks)
{
    const int m = (k < M - k) ? k : (M - k);
    uint32_t w = 0u;
    for (int i0 = 0; i0 < m; i0 += 4) {
        const Philox4 blk = philox4x32_10(s, (uint32_t)(i0 >> 2), unit, stream_id, ks);
        static_for<4>([&](auto x) {
            const int i = i0 + x.value;
            if (i < m) {
                const uint32_t j = (uint32_t)(M - m + i);
                const uint32_t r = __umulhi(blk.x[x.value], j + 1u);
                const uint32_t hit = (uint32_t)__builtin_amdgcn_sbfe((int)w, r, 1u);  // all ones if bit r is set
                w |= 1u << r;
                w |= hit & (1u << j);
            }
        });
    }
    mask.w[0] = w;
    if (k > M - k) mask.complement(M);
}

// M <= 64 (two words, handled as one 64-bit value).
__device__ __forceinline__ void sample_mask(Mask<2>& mask, int M, int k, uint32_t s, uint32_t unit,
                                            uint32_t stream_id, const PhiloxKeys& ks)
{
    const int m = (k < M - k) ? k : (M - k);
    uint64_t w = 0ull;
    for (int i0 = 0; i0 < m; i0 += 4) {
        const Philox4 blk = philox4x32_10(s, (uint32_t)(i0 >> 2), unit, stream_id, ks);
        static_for<4>([&](auto x) {
            const int i = i0 + x.value;
            if (i < m) {
                const uint32_t j = (uint32_t)(M - m + i);
                const uint32_t r = __umulhi(blk.x[x.value], j + 1u);
                const uint32_t hit = 0u - ((uint32_t)(w >> r) & 1u);
                const uint64_t bj = 1ull << j;  // uniform
                const uint64_t br = 1ull << r;
                const uint32_t lo = (uint32_t)w | (uint32_t)br | (hit & (uint32_t)bj);
                const uint32_t hi = (uint32_t)(w >> 32) | (uint32_t)(br >> 32) | (hit & (uint32_t)(bj >> 32));
                w = ((uint64_t)hi << 32) | lo;
            }
        });
    }
    mask.w[0] = (uint32_t)w;
    mask.w[1] = (uint32_t)(w >> 32);
    if (k > M - k) mask.complement(M);
}

// M > 64: the set lives in LDS while it is drawn, word x of this lane at lds[x * stride + lane slot]
// (conflict-free: the bank depends on the lane only).  One LDS read and two LDS ORs per step whatever the
// mask width; the finished words are then loaded into registers for the reducer.
template <int NW>
__device__ __forceinline__ void sample_mask_lds(Mask<NW>& mask, uint32_t* lds_col, int stride, int M, int k,
                                                uint32_t s, uint32_t unit, uint32_t stream_id, const PhiloxKeys& ks)
{
    const int m = (k < M - k) ? k : (M - k);
    static_for<NW>([&](auto i) { lds_col[i.value * stride] = 0u; });
    for (int i0 = 0; i0 < m; i0 += 4) {
        const Philox4 blk = philox4x32_10(s, (uint32_t)(i0 >> 2), unit, stream_id, ks);
        static_for<4>([&](auto x) {
            const int i = i0 + x.value;
            if (i < m) {
                const uint32_t j = (uint32_t)(M - m + i);
                const uint32_t r = __umulhi(blk.x[x.value], j + 1u);
                uint32_t* pr = lds_col + (r >> 5) * (uint32_t)stride;
                const uint32_t old = *pr;
                const uint32_t hit = (uint32_t)__builtin_amdgcn_sbfe((int)old, r & 31u, 1u);  // all ones if bit r is set
                *pr = old | (1u << (r & 31u));
                uint32_t* pj = lds_col + (j >> 5) * (uint32_t)stride;  // the same word in every lane
                atomicOr(pj, hit & (1u << (j & 31u)));                  // LDS operations of a wave stay in order
            }
        });
    }
    static_for<NW>([&](auto i) { mask.w[i.value] = lds_col[i.value * stride]; });
    if (k > M - k) mask.complement(M);
}

// ------------------------------------------------------------------ reducer

// Bits at multiples of P inside a 32-bit word (P a power of two <= 32).
__device__ __forceinline__ uint32_t comb32(int log2P)
{
    // 0xffffffff / (2^P - 1) for P < 32, 1 for P == 32
    switch (log2P) {
        case 0: return 0xffffffffu;
        case 1: return 0x55555555u;
        case 2: return 0x11111111u;
        case 3: return 0x01010101u;
        case 4: return 0x00010001u;
        default: return 0x00000001u;
    }
}

// Vertical (bit-sliced) counters: plane p holds bit p of one counter per bit position.
template <int NP>
struct Planes {
    uint32_t p[NP];
    __device__ __forceinline__ void clear()
    {
        static_for<NP>([&](auto i) { p[i.value] = 0u; });
    }
    // add one to the counter of every position whose bit is set in x
    __device__ __forceinline__ void add(uint32_t x)
    {
        uint32_t carry = x;
        static_for<NP>([&](auto i) {
            const uint32_t t = p[i.value] & carry;
            p[i.value] ^= carry;
            carry = t;
        });
    }
    // largest counter over all positions
    __device__ __forceinline__ int max() const
    {
        uint32_t cand = 0xffffffffu;
        int result = 0;
        static_for<NP>([&](auto i) {
            constexpr int bit = NP - 1 - i.value;
            const uint32_t x = cand & p[bit];
            if (x != 0u) {
                cand = x;
                result |= (1 << bit);
            }
        });
        return result;
    }
};

// n_int (pipelines without a preempted instance) and d_min (fewest survivors in any stage)
// of a D x P grid whose preempted instances are the set bits of mask; instance j = d * P + s.
template <int NW>
__device__ __forceinline__ void reduce_mask(const Mask<NW>& mask, int D, int P, int log2P, int& n_int, int& d_min)
{
    if (log2P >= 0 && P <= 32) {
        // pipelines: OR-fold every aligned P-bit group onto its lowest bit
        const uint32_t comb = comb32(log2P);
        int broken = 0;
        static_for<NW>([&](auto i) {
            uint32_t y = mask.w[i.value];
            for (int sh = 1; sh < P; sh <<= 1) y |= y >> sh;
            broken += __popc(y & comb);
        });
        n_int = D - broken;
        if (P <= 16) {
            // stages: popcount of the stride-P comb shifted to the stage
            int worst = 0;
            for (int s = 0; s < P; ++s) {
                const uint32_t cs = comb << s;
                int cnt = 0;
                static_for<NW>([&](auto i) { cnt += __popc(mask.w[i.value] & cs); });
                worst = cnt > worst ? cnt : worst;
            }
            d_min = D - worst;
        } else {
            // P == 32: one word per pipeline (D <= 8), add the words as vertical counters
            Planes<4> pl;
            pl.clear();
            static_for<NW>([&](auto i) { pl.add(mask.w[i.value]); });
            d_min = D - pl.max();
        }
    } else if (log2P >= 6) {
        // P in {64, 128, 256}: a pipeline is P/32 whole words, D <= 4
        int broken = 0, worst = 0;
        if constexpr (NW >= 2) {
            const int wpr = P >> 5;  // words per pipeline
            uint32_t acc_or = 0u;
            static_for<NW>([&](auto i) {
                acc_or |= mask.w[i.value];
                if (((i.value + 1) & (wpr - 1)) == 0) {  // last word of a pipeline
                    broken += (acc_or != 0u) ? 1 : 0;
                    acc_or = 0u;
                }
            });
            // stage counts: for each word column x in [0, wpr) add words x, x + wpr, x + 2 wpr, ...
            for (int x = 0; x < wpr; ++x) {
                Planes<3> pl;
                pl.clear();
                static_for<NW>([&](auto i) {
                    if ((i.value & (wpr - 1)) == x) pl.add(mask.w[i.value]);
                });
                const int cm = pl.max();
                worst = cm > worst ? cm : worst;
            }
        }
        n_int = D - broken;
        d_min = D - worst;
    } else {
        // any other depth: walk the grid bit by bit (the bit index is the same in every lane)
        int intact = 0;
        for (int d = 0; d < D; ++d) {
            bool hit = false;
            for (int s = 0; s < P; ++s) hit = hit || mask.test((uint32_t)(d * P + s));
            intact += hit ? 0 : 1;
        }
        int least = D;
        for (int s = 0; s < P; ++s) {
            int alive = 0;
            for (int d = 0; d < D; ++d) alive += mask.test((uint32_t)(d * P + s)) ? 0 : 1;
            least = alive < least ? alive : least;
        }
        n_int = intact;
        d_min = least;
    }
}

// ------------------------------------------------------------------ histogram update

// One LDS atomic per lane.  Lanes that hit the same bin are serialised by the LDS bank, not by the
// vector ALU, which is the unit this kernel is bound by.
__device__ __forceinline__ void hist_add(uint32_t* bins, int val, bool active)
{
    if (active) atomicAdd(&bins[val], 1u);
}

// ------------------------------------------------------------------ kernels

constexpr int kEvalThreads = 256;

// Clears the histograms and writes the closed-form bins of units that need no sampling:
// k == 0 puts all S scenarios in bin D, k == M in bin 0 (of both histograms).
__global__ void __launch_bounds__(256) prep_hist_kernel(Batch b, uint32_t* __restrict__ hist_int,
                                                        uint32_t* __restrict__ hist_min)
{
    const int64_t total = (int64_t)b.nq * b.T * b.L;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int pos = (int)(e % b.L);
        const int64_t qt = e / b.L;
        const int t = (int)(qt % b.T);
        const int q = (int)(qt / b.T);
        // candidate whose row holds pos: last c with off[c] <= pos
        int lo = 0, hi = b.C - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (b.cfg[mid].off <= pos) lo = mid; else hi = mid - 1;
        }
        const CfgRec cr = b.cfg[lo];
        const int j = pos - cr.off;
        int M, k;
        unit_pool(cr.D, cr.P, b.avail[(int64_t)q * (b.T + 1) + t + 1], b.N, M, k);
        uint32_t v = 0u;
        if (k == 0) v = (j == cr.D) ? (uint32_t)b.S : 0u;
        else if (k == M) v = (j == 0) ? (uint32_t)b.S : 0u;
        hist_int[e] = v;
        hist_min[e] = v;
    }
}

// Draws scenario s of a unit into registers, by the path that fits the unit's size.
template <int NW>
__device__ __forceinline__ void draw_scenario(Mask<NW>& mask, uint32_t* lds_col, int M, int k, uint32_t s,
                                              uint32_t unit, uint32_t stream_id, const PhiloxKeys& ks)
{
    if constexpr (NW <= 2) {
        sample_mask(mask, M, k, s, unit, stream_id, ks);
    } else {
        sample_mask_lds<NW>(mask, lds_col, kEvalThreads, M, k, s, unit, stream_id, ks);
    }
}

template <int NW>
__device__ __forceinline__ void eval_unit_chunk(const CfgRec cr, int M, int k, uint32_t unit, uint32_t stream_id,
                                                const PhiloxKeys& ks, uint32_t s_begin, uint32_t s_end,
                                                uint32_t* lds_col, uint32_t* bins_int, uint32_t* bins_min)
{
    const uint32_t span = s_end - s_begin;
    for (uint32_t x = threadIdx.x; x < span; x += blockDim.x) {
        int n_int, d_min;
        Mask<NW> mask;
        draw_scenario<NW>(mask, lds_col, M, k, s_begin + x, unit, stream_id, ks);
        reduce_mask<NW>(mask, cr.D, cr.P, cr.log2P, n_int, d_min);
        hist_add(bins_int, n_int, true);
        hist_add(bins_min, d_min, true);
    }
}

// Block b handles scenarios [chunk * chunk_len, ...) of unit b / n_chunks.
__global__ void __launch_bounds__(kEvalThreads) eval_hist_kernel(Batch b, int n_chunks, int chunk_len,
                                                                 uint32_t* __restrict__ hist_int,
                                                                 uint32_t* __restrict__ hist_min)
{
    __shared__ uint32_t bins[2 * (kMaxInstances + 1)];
    __shared__ uint32_t lmask[8 * kEvalThreads];  // sets of units with more than 64 instances, [word][lane]
    const uint32_t unit_global = blockIdx.x / (uint32_t)n_chunks;  // q * T * C + t * C + c
    const int chunk = (int)(blockIdx.x % (uint32_t)n_chunks);
    const int tc = (int)(unit_global % (uint32_t)(b.T * b.C));
    const int q = (int)(unit_global / (uint32_t)(b.T * b.C));
    const int t = tc / b.C;
    const int c = tc - t * b.C;
    const CfgRec cr = b.cfg[c];
    int M, k;
    unit_pool(cr.D, cr.P, b.avail[(int64_t)q * (b.T + 1) + t + 1], b.N, M, k);
    if (k == 0 || k == M) return;  // closed form, written by prep_hist_kernel

    const int nb = cr.D + 1;
    uint32_t* bins_int = bins;
    uint32_t* bins_min = bins + nb;
    for (int i = threadIdx.x; i < 2 * nb; i += blockDim.x) bins[i] = 0u;
    __syncthreads();

    const uint64_t seed = b.seed[q];
    const PhiloxKeys ks = philox_keys((uint32_t)(seed & 0xffffffffull), (uint32_t)(seed >> 32));
    const uint32_t stream_id = b.stream_id ? b.stream_id[q] : 0u;
    const uint32_t s_begin = (uint32_t)chunk * (uint32_t)chunk_len;
    uint32_t s_end = s_begin + (uint32_t)chunk_len;
    s_end = s_end > (uint32_t)b.S ? (uint32_t)b.S : s_end;
    uint32_t* lds_col = lmask + threadIdx.x;

    if (M <= 32) eval_unit_chunk<1>(cr, M, k, (uint32_t)tc, stream_id, ks, s_begin, s_end, lds_col, bins_int, bins_min);
    else if (M <= 64) eval_unit_chunk<2>(cr, M, k, (uint32_t)tc, stream_id, ks, s_begin, s_end, lds_col, bins_int, bins_min);
    else if (M <= 128) eval_unit_chunk<4>(cr, M, k, (uint32_t)tc, stream_id, ks, s_begin, s_end, lds_col, bins_int, bins_min);
    else eval_unit_chunk<8>(cr, M, k, (uint32_t)tc, stream_id, ks, s_begin, s_end, lds_col, bins_int, bins_min);
    __syncthreads();

    const int64_t base = ((int64_t)q * b.T + t) * b.L + cr.off;
    for (int i = threadIdx.x; i < nb; i += blockDim.x) {
        const uint32_t vi = bins_int[i], vm = bins_min[i];
        if (n_chunks == 1) {
            hist_int[base + i] = vi;
            hist_min[base + i] = vm;
        } else {
            if (vi) atomicAdd(&hist_int[base + i], vi);
            if (vm) atomicAdd(&hist_min[base + i], vm);
        }
    }
}

// One scenario through the same code path the histogram kernel takes for a unit of this size.
template <int NW>
__device__ __forceinline__ void debug_one(const CfgRec cr, uint32_t* lds_col, int M, int k, uint32_t s, uint32_t unit,
                                          uint32_t stream_id, const PhiloxKeys& ks, uint32_t* mask_out, int& n_int,
                                          int& d_min)
{
    Mask<NW> mask;
    draw_scenario<NW>(mask, lds_col, M, k, s, unit, stream_id, ks);
    reduce_mask<NW>(mask, cr.D, cr.P, cr.log2P, n_int, d_min);
    static_for<8>([&](auto i) {
        if constexpr (i.value < NW) mask_out[i.value] = mask.w[i.value];
        else mask_out[i.value] = 0u;
    });
}

// Scenarios one by one, for inspection: masks [ns][8], n_int [ns], d_min [ns].
__global__ void __launch_bounds__(kEvalThreads) debug_sample_kernel(Batch b, int q, int t, int c, uint32_t s0,
                                                                    uint32_t ns, uint32_t* __restrict__ masks,
                                                                    int32_t* __restrict__ n_int_out,
                                                                    int32_t* __restrict__ d_min_out)
{
    __shared__ uint32_t lmask[8 * kEvalThreads];
    const uint32_t x = blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= ns) return;
    const CfgRec cr = b.cfg[c];
    int M, k;
    unit_pool(cr.D, cr.P, b.avail[(int64_t)q * (b.T + 1) + t + 1], b.N, M, k);
    const uint64_t seed = b.seed[q];
    const PhiloxKeys ks = philox_keys((uint32_t)(seed & 0xffffffffull), (uint32_t)(seed >> 32));
    const uint32_t stream_id = b.stream_id ? b.stream_id[q] : 0u;
    const uint32_t unit = (uint32_t)(t * b.C + c);
    uint32_t* lds_col = lmask + threadIdx.x;
    uint32_t* out = masks + (size_t)x * 8;
    int n_int, d_min;
    if (M <= 32) debug_one<1>(cr, lds_col, M, k, s0 + x, unit, stream_id, ks, out, n_int, d_min);
    else if (M <= 64) debug_one<2>(cr, lds_col, M, k, s0 + x, unit, stream_id, ks, out, n_int, d_min);
    else if (M <= 128) debug_one<4>(cr, lds_col, M, k, s0 + x, unit, stream_id, ks, out, n_int, d_min);
    else debug_one<8>(cr, lds_col, M, k, s0 + x, unit, stream_id, ks, out, n_int, d_min);
    n_int_out[x] = n_int;
    d_min_out[x] = d_min;
}

}  // namespace parcae
