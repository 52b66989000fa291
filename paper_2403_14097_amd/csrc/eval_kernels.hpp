// Scenario sampler, survivor reducer and histogram kernels (section 6.3, section 5.2).
//
// One lane owns one scenario: Floyd's subset loop carries a dependence on the
// growing set, so it cannot be spread over lanes, but all 64 lanes of a wave
// work on the same unit (q, t, c), which keeps D, P, M, k and every loop trip
// count in scalar registers.  A 256-bit preemption mask lives in NW 32-bit
// vector registers per lane (NW = 1, 2, 4 or 8 by the unit's size).
#pragma once

#include "device_common.hpp"
#include "eval_launch.hpp"

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
    // drop bits at and above M
    __device__ __forceinline__ void keep_below(int M)
    {
        static_for<NW>([&](auto i) {
            constexpr int lo = i.value * 32;
            const uint32_t valid = (M >= lo + 32) ? 0xffffffffu : (M <= lo ? 0u : ((1u << (M - lo)) - 1u));
            w[i.value] &= valid;
        });
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

// ------------------------------------------------------------------ non-uniform preemption (zones)

// Zones of the pool of one unit, built once per work item by the wave that owns it (section 5.1: the
// equal-probability assumption may be replaced; here instances fall into zones of unequal hazard weight and
// leave by successive weighted sampling without replacement).
struct ZoneCtx {
    const uint8_t* perm;    // LDS [kMaxZones][256]: perm[z * 256 + r] = pool index of the r-th member of zone z
    const uint32_t* zmask;  // LDS [kMaxZones][8]: members of zone z among the pool as a bit set
    int size[kMaxZones];    // members of zone z in the pool
    uint32_t weight[kMaxZones];
};

// All 64 lanes of the wave must be active.  perm and zmask are this wave's LDS tables.
__device__ __forceinline__ ZoneCtx zone_setup(const Batch& b, int q, int M, uint8_t* perm, uint32_t* zmask)
{
    const int lane = lane_id();
    const uint8_t* zq = b.zone + (int64_t)q * b.N;
    ZoneCtx zc;
    zc.perm = perm;
    zc.zmask = zmask;
    static_for<kMaxZones>([&](auto z) {
        zc.size[z.value] = 0;
        zc.weight[z.value] = z.value < b.n_zones ? b.zone_weight[(int64_t)q * kMaxZones + z.value] : 0u;
    });
    if (lane < kMaxZones * 8) zmask[lane] = 0u;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int j0 = 0; j0 < M; j0 += kWave) {
        const int j = j0 + lane;
        const int zj = j < M ? (int)zq[j] : -1;
        static_for<kMaxZones>([&](auto z) {
            const unsigned long long votes = __ballot(zj == z.value);
            if (zj == z.value) perm[z.value * 256 + zc.size[z.value] + __popcll(votes & below)] = (uint8_t)j;
            if (lane == 0) {
                zmask[z.value * 8 + (j0 >> 5)] = (uint32_t)votes;
                zmask[z.value * 8 + (j0 >> 5) + 1] = (uint32_t)(votes >> 32);
            }
            zc.size[z.value] += __popcll(votes);
        });
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return zc;
}

// Preempted set of scenario s when preemption is not uniform.  Part 1 draws the zones of the k departures
// (word sequence 0xFFFF): per lane the products weight * instances left of every zone, one compare chain
// per draw.  Part 2 draws, per zone, which members go: Floyd's method on the ranks of the zone's members
// (word sequence z), the smaller side, ranks mapped to pool indices through perm; lanes differ in how many
// members of a zone go, so the loop runs to the largest count in the wave with the other lanes masked off.
// The set is built in LDS ([word][lane], as in sample_mask_lds) whatever the pool size.
template <int NW>
__device__ __forceinline__ void sample_mask_zoned(Mask<NW>& mask, uint32_t* lds_col, int stride, const ZoneCtx& zc,
                                                  int k, uint32_t s, uint32_t unit, uint32_t stream_id,
                                                  const PhiloxKeys& ks)
{
    // Part 1 without compares or selects (selects through the condition register are slow on this chip):
    // all quantities stay below 2^31, so the sign of r - c is the outcome of r < c as an all-ones mask.
    // below[j] counts the draws that fell into zones 0..j.
    uint32_t left_w[kMaxZones], below[kMaxZones - 1], wv[kMaxZones];
    static_for<kMaxZones>([&](auto z) {
        left_w[z.value] = zc.weight[z.value] * (uint32_t)zc.size[z.value];
        wv[z.value] = in_vgpr(zc.weight[z.value]);
    });
    static_for<kMaxZones - 1>([&](auto z) { below[z.value] = 0u; });
    for (int i0 = 0; i0 < k; i0 += 4) {
        const Philox4 blk = philox4x32_10(s, 0xFFFF0000u + (uint32_t)(i0 >> 2), unit, stream_id, ks);
        static_for<4>([&](auto x) {
            if (i0 + x.value < k) {
                const uint32_t c0 = left_w[0], c1 = c0 + left_w[1], c2 = c1 + left_w[2], total = c2 + left_w[3];
                const uint32_t r = __umulhi(blk.x[x.value], total);
                const uint32_t m0 = (uint32_t)((int32_t)(r - c0) >> 31);  // all ones if r < c0
                const uint32_t m1 = (uint32_t)((int32_t)(r - c1) >> 31);
                const uint32_t m2 = (uint32_t)((int32_t)(r - c2) >> 31);
                below[0] -= m0;
                below[1] -= m1;
                below[2] -= m2;
                left_w[0] -= m0 & wv[0];
                left_w[1] -= (m1 ^ m0) & wv[1];  // m0 implies m1 implies m2
                left_w[2] -= (m2 ^ m1) & wv[2];
                left_w[3] -= ~m2 & wv[3];
            }
        });
    }
    const uint32_t gone[kMaxZones] = {below[0], below[1] - below[0], below[2] - below[1], (uint32_t)k - below[2]};
    static_for<NW>([&](auto i) { lds_col[i.value * stride] = 0u; });
    static_for<kMaxZones>([&](auto zi) {
        constexpr int z = zi.value;
        const int Mz = zc.size[z];
        if (Mz > 0) {
            const int kz = (int)gone[z];
            const int rest = Mz - kz;
            const int mz = kz < rest ? kz : rest;
            const uint8_t* perm = zc.perm + z * 256;
            for (int i0 = 0; __any(i0 < mz); i0 += 4) {
                const Philox4 blk = philox4x32_10(s, ((uint32_t)z << 16) + (uint32_t)(i0 >> 2), unit, stream_id, ks);
                static_for<4>([&](auto x) {
                    const int i = i0 + x.value;
                    if (i < mz) {
                        const uint32_t j = (uint32_t)(Mz - mz + i);
                        const uint32_t r = __umulhi(blk.x[x.value], j + 1u);
                        const uint32_t pr = perm[r], pj = perm[j];
                        const uint32_t old = lds_col[(pr >> 5) * (uint32_t)stride];
                        const uint32_t put = ((old >> (pr & 31u)) & 1u) ? pj : pr;  // r already there: j goes in
                        atomicOr(lds_col + (put >> 5) * (uint32_t)stride, 1u << (put & 31u));
                    }
                });
            }
            if (kz > rest) static_for<NW>([&](auto w) { lds_col[w.value * stride] ^= zc.zmask[z * 8 + w.value]; });
        }
    });
    static_for<NW>([&](auto i) { mask.w[i.value] = lds_col[i.value * stride]; });
}

// ------------------------------------------------------------------ a hazard weight per instance

// How a unit's scenarios are drawn: every instance equally likely, zones of unequal hazard, or a weight per instance.
enum DrawKind { kDrawUniform = 0, kDrawZoned = 1, kDrawWeighted = 2 };

// Weights of the pool of one unit, staged once per work item by the wave that owns it (section 5.1: the
// equal-probability assumption replaced by an estimate per instance).
struct WeightCtx {
    const uint8_t* bytes;   // LDS [272], 16-byte aligned: the weights, one per instance, 0 beyond the pool
    uint32_t word_sum[8];   // sum of the weights of instances 32 W .. 32 W + 31 (the same in every lane)
    uint32_t total;         // sum over the pool
};

// All 64 lanes of the wave must be active.  A weight of 0 (refused by the input checks) counts as 1.
__device__ __forceinline__ WeightCtx weight_setup(const Batch& b, int q, int M, uint8_t* bytes)
{
    const int lane = lane_id();
    const uint8_t* wq = b.inst_weight + (int64_t)q * b.N;
    WeightCtx wc;
    wc.bytes = bytes;
    uint32_t sum = 0u;
    static_for<4>([&](auto x) {  // lane L stages instances 4 L .. 4 L + 3
        const int j = 4 * lane + x.value;
        uint32_t w = 0u;
        if (j < M) {
            w = wq[j];
            w = w < 1u ? 1u : w;
        }
        bytes[j] = (uint8_t)w;
        sum += w;
    });
    if (lane < 4) bytes[256 + lane] = 0u;  // a look-up one past the pool (cannot happen for valid input) finds 0
    for (int sh = 1; sh < 8; sh <<= 1) sum += __shfl_xor(sum, sh);  // eight lanes hold a word of 32 instances
    static_for<8>([&](auto W) { wc.word_sum[W.value] = (uint32_t)__builtin_amdgcn_readlane((int)sum, 8 * W.value); });
    for (int sh = 8; sh < kWave; sh <<= 1) sum += __shfl_xor(sum, sh);
    wc.total = sum;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return wc;
}

// Preempted set of scenario s by successive weighted sampling without replacement: k times, word i of sequence
// 0xFFFE scaled to the weight still there picks a point, and the first instance (ascending) at which the running
// sum of the weights still there exceeds the point goes.  Every lane has its own set and walks the pool in three
// passes; running sums never decrease, so in each pass the number of parts whose running sum does not exceed the
// point is the part that holds the instance: (1) the words of 32 instances, by the weight still there per word,
// which the lane keeps up to date; (2) the eight groups of four instances of that word (the four "still there"
// bits spread to bytes, one dot product with the four weights per group); (3) the four instances of that group.
template <int NW>
__device__ __forceinline__ void sample_mask_weighted(Mask<NW>& mask, const WeightCtx& wc, int M, int k, uint32_t s,
                                                     uint32_t unit, uint32_t stream_id, const PhiloxKeys& ks)
{
    mask.clear();
    uint32_t total = wc.total;
    uint32_t left[NW];  // weight still there, per word
    static_for<NW>([&](auto W) { left[W.value] = wc.word_sum[W.value]; });
    const uint4* by_sixteen = reinterpret_cast<const uint4*>(wc.bytes);
    const uint32_t* by_four = reinterpret_cast<const uint32_t*>(wc.bytes);
    for (int i0 = 0; i0 < k; i0 += 4) {
        const Philox4 blk = philox4x32_10(s, 0xFFFE0000u + (uint32_t)(i0 >> 2), unit, stream_id, ks);
        static_for<4>([&](auto x) {
            if (i0 + x.value < k) {
                const uint32_t point = __umulhi(blk.x[x.value], total);
                uint32_t running = 0u, word = 0u, before = 0u;
                static_for<NW - 1>([&](auto W) {  // the last word takes what the others leave
                    running += left[W.value];
                    const bool below = running <= point;
                    word += below ? 1u : 0u;
                    before = below ? running : before;
                });
                uint32_t there = 0u;
                static_for<NW>([&](auto W) { there = word == (uint32_t)W.value ? ~mask.w[W.value] : there; });
                // the 32 weights of that word, four to a register
                const uint4 lo = by_sixteen[2u * word], hi = by_sixteen[2u * word + 1u];
                const uint32_t fours[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                uint32_t group = 0u;
                running = before;
                static_for<8>([&](auto p) {
                    // bits 4p .. 4p + 3 of `there`, one per byte: b0 + 2 b1 + 4 b2 + 8 b3 times (1 + 2^7 + 2^14 + 2^21)
                    const uint32_t nibble = (there >> (4 * p.value)) & 0xfu;
                    const uint32_t ones = (nibble * 0x00204081u) & 0x01010101u;
                    running = __builtin_amdgcn_udot4(fours[p.value], ones, running, false);
                    const bool below = running <= point;
                    group += below ? 1u : 0u;
                    before = below ? running : before;
                });
                // the four instances of that group (a group past the word cannot come out of weights that add up)
                group = group < 8u ? group : 7u;
                const uint32_t four = by_four[8u * word + group];
                const uint32_t nibble = (there >> (4u * group)) & 0xfu;
                uint32_t inside = 0u, went = 0u;
                running = before;
                static_for<4>([&](auto y) {
                    const uint32_t w = (four >> (8 * y.value)) & 0xffu;
                    const uint32_t on = 0u - ((nibble >> y.value) & 1u);
                    running += on & w;
                    const bool below = running <= point;
                    inside += below ? 1u : 0u;
                    went = (below || went != 0u) ? went : w;  // the weight at which the running sum first exceeds the point
                });
                mask.set(32u * word + 4u * group + inside);
                total -= went;
                static_for<NW>([&](auto W) { left[W.value] -= word == (uint32_t)W.value ? went : 0u; });
            }
        });
    }
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

// Vertical (bit-sliced) counters: plane i holds bit i of one counter per bit position.
template <int NP>
struct Planes {
    uint32_t p[NP];
    __device__ __forceinline__ void clear()
    {
        static_for<NP>([&](auto i) { p[i.value] = 0u; });
    }
    // add one to the counter of every position whose bit is set in x; the carry ripples through the
    // lowest N planes (the caller knows the counters stay below 2^N)
    template <int N = NP>
    __device__ __forceinline__ void add(uint32_t x)
    {
        uint32_t carry = x;
        static_for<N>([&](auto i) {
            const uint32_t t = p[i.value] & carry;
            p[i.value] ^= carry;
            carry = t;
        });
    }
    // counters of position b += counters of position b + sh, for N-plane inputs; the result has N + 1 planes
    template <int N>
    __device__ __forceinline__ void fold(int sh)
    {
        static_assert(N + 1 <= NP, "no room for the carry plane");
        uint32_t carry = 0u;
        static_for<N>([&](auto i) {
            const uint32_t a = p[i.value];
            const uint32_t b = a >> sh;
            if constexpr (i.value == 0) {
                p[0] = a ^ b;
                carry = a & b;
            } else {
                p[i.value] = __builtin_amdgcn_bitop3_b32(a, b, carry, 0x96);   // a ^ b ^ carry
                carry = __builtin_amdgcn_bitop3_b32(a, b, carry, 0xE8);        // majority
            }
        });
        p[N] = carry;
    }
    // largest counter over the positions selected by keep
    __device__ __forceinline__ int max(uint32_t keep = 0xffffffffu) const
    {
        uint32_t cand = keep;
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

// Largest number of preempted instances in any stage, P a power of two in [8, 32]: the words are added
// as vertical counters (rows of different words are aligned because P divides 32), then the rows inside
// the word are folded onto the lowest row.
template <int NW>
__device__ __forceinline__ int worst_stage_tree(const Mask<NW>& mask, int P)
{
    constexpr int NP0 = (NW == 1) ? 1 : (NW == 2) ? 2 : (NW == 4) ? 3 : 4;  // planes that hold a count of NW
    Planes<NP0 + 2> pl;
    pl.clear();
    static_for<NW>([&](auto i) { pl.template add<NP0>(mask.w[i.value]); });
    if (P <= 16) pl.template fold<NP0>(16);
    if (P <= 8) pl.template fold<NP0 + 1>(8);
    const uint32_t keep = (P >= 32) ? 0xffffffffu : ((1u << P) - 1u);
    return pl.max(keep);
}

// ---- depths that are not powers of two: pipeline rows do not line up with the 32-bit words ----

// Bits at multiples of P below 32.
__device__ __forceinline__ uint32_t period_comb(int P)
{
    uint32_t q = 0u;
    for (int b = 0; b < 32; b += P) q |= 1u << b;
    return q;
}

// Bits b of word i with (32 i + b) mod P == s, given q = period_comb(P).
__device__ __forceinline__ uint32_t stage_comb(uint32_t q, int P, int s, int i)
{
    int r = (s - 32 * i) % P;
    r = r < 0 ? r + P : r;
    return q << r;
}

// 2 <= P <= 8, not a power of two (3, 5, 6, 7): windows and combs.
// Intact pipelines: OR of every window of P consecutive bits (built by doubling, shifts cross word
// boundaries), sampled at the positions where a pipeline starts.  Stage occupancy: popcount of the
// period-P comb of every stage.
template <int NW>
__device__ __forceinline__ void reduce_small_depth(const Mask<NW>& mask, int D, int P, int& n_int, int& d_min)
{
    const uint32_t q = period_comb(P);
    uint32_t y[NW];
    static_for<NW>([&](auto i) { y[i.value] = mask.w[i.value]; });
    for (int cover = 1; cover < P;) {
        const int sh = cover < P - cover ? cover : P - cover;
        static_for<NW>([&](auto i) {  // ascending: word i + 1 still holds its old value
            uint32_t next = 0u;
            if constexpr (i.value + 1 < NW) next = y[i.value + 1];
            y[i.value] |= __builtin_amdgcn_alignbit(next, y[i.value], (uint32_t)sh);
        });
        cover += sh;
    }
    int broken = 0;
    static_for<NW>([&](auto i) { broken += __popc(y[i.value] & stage_comb(q, P, 0, i.value)); });
    n_int = D - broken;
    int worst = 0;
    for (int s = 0; s < P; ++s) {
        int cnt = 0;
        static_for<NW>([&](auto i) { cnt += __popc(mask.w[i.value] & stage_comb(q, P, s, i.value)); });
        worst = cnt > worst ? cnt : worst;
    }
    d_min = D - worst;
}

// 8 < P < 32, not a power of two: every pipeline row is cut out of the two words it touches (the word
// index is a compile-time constant, the shift is the same in every lane) and added to vertical counters.
template <int NW, int NP>
__device__ __forceinline__ void reduce_medium_depth(const Mask<NW>& mask, int D, int P, int& n_int, int& d_min)
{
    const uint32_t pmask = (1u << P) - 1u;
    Planes<NP> pl;
    pl.clear();
    int broken = 0;
    static_for<NW>([&](auto i) {
        uint32_t hi = 0u;
        if constexpr (i.value + 1 < NW) hi = mask.w[i.value + 1];
        const uint32_t lo = mask.w[i.value];
        // pipelines whose first bit lies in word i
        int d = (32 * i.value + P - 1) / P;
        for (; d < D && d * P < 32 * (i.value + 1); ++d) {
            const uint32_t row = __builtin_amdgcn_alignbit(hi, lo, (uint32_t)(d * P - 32 * i.value)) & pmask;
            pl.add(row);
            broken += row != 0u ? 1 : 0;
        }
    });
    n_int = D - broken;
    d_min = D - pl.max();
}

// P > 32, not a power of two (D <= 7): a pipeline row spans several words; word c of every row is added to
// its own set of vertical counters.
template <int NW>
__device__ __forceinline__ void reduce_large_depth(const Mask<NW>& mask, int D, int P, int& n_int, int& d_min)
{
    const int rw = (P + 31) >> 5;                                         // words per row
    const uint32_t last = (P & 31) ? ((1u << (P & 31)) - 1u) : 0xffffffffu;  // valid bits of a row's last word
    Planes<3> pl[NW];
    static_for<NW>([&](auto c) { pl[c.value].clear(); });
    int broken = 0;
    static_for<NW>([&](auto i) {
        // at most one pipeline starts in word i
        const int d = (32 * i.value + P - 1) / P;
        if (d < D && d * P < 32 * (i.value + 1)) {
            const uint32_t sh = (uint32_t)(d * P - 32 * i.value);
            uint32_t any = 0u;
            static_for<NW>([&](auto c) {
                if constexpr (i.value + c.value < NW) {
                    if (c.value < rw) {
                        uint32_t hi = 0u;
                        if constexpr (i.value + c.value + 1 < NW) hi = mask.w[i.value + c.value + 1];
                        uint32_t x = __builtin_amdgcn_alignbit(hi, mask.w[i.value + c.value], sh);
                        if (c.value == rw - 1) x &= last;
                        pl[c.value].add(x);
                        any |= x;
                    }
                }
            });
            broken += any != 0u ? 1 : 0;
        }
    });
    int worst = 0;
    static_for<NW>([&](auto c) {
        if (c.value < rw) {
            const int m = pl[c.value].max();
            worst = m > worst ? m : worst;
        }
    });
    n_int = D - broken;
    d_min = D - worst;
}

// Which reducer a grid shape takes.  The choice depends on the unit only, so the sampling loop is compiled once
// per kind: each copy then carries only its own loop-invariant masks in scalar registers (with all kinds inside
// one loop the invariants of every kind were live at once and spilled).
enum ReducerKind {
    kPow2Narrow = 0,   // P in {1, 2, 4}: stage counts by popcounts of stride-P combs
    kPow2Tree = 1,     // P in {8, 16, 32}: stage counts by vertical counters
    kPow2Words = 2,    // P in {64, 128, 256}: a pipeline is whole words
    kAnySmall = 3,     // other P <= 8: windows and period-P combs
    kAnyMediumFew = 4, // other P < 32, at most 7 pipelines
    kAnyMedium = 5,    // other P < 32, more pipelines
    kAnyLarge = 6,     // other P > 32
};

__device__ __forceinline__ int reducer_kind(int D, int P, int log2P)
{
    if (log2P >= 0 && P <= 32) return P <= 4 ? kPow2Narrow : kPow2Tree;
    if (log2P >= 6) return kPow2Words;
    if (P <= 8) return kAnySmall;
    if (P < 32) return D <= 7 ? kAnyMediumFew : kAnyMedium;
    return kAnyLarge;
}

// n_int (pipelines without a preempted instance) and d_min (fewest survivors in any stage)
// of a D x P grid whose preempted instances are the set bits of mask; instance j = d * P + s.
template <int NW, int KIND>
__device__ __forceinline__ void reduce_kind(const Mask<NW>& mask, int D, int P, int log2P, int& n_int, int& d_min)
{
    if constexpr (KIND == kPow2Narrow || KIND == kPow2Tree) {
        // pipelines: OR-fold every aligned P-bit group onto its lowest bit
        const uint32_t comb = comb32(log2P);
        int broken = 0;
        static_for<NW>([&](auto i) {
            uint32_t y = mask.w[i.value];
            for (int sh = 1; sh < P; sh <<= 1) y |= y >> sh;
            broken += __popc(y & comb);
        });
        n_int = D - broken;
        if constexpr (KIND == kPow2Narrow) {
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
            d_min = D - worst_stage_tree<NW>(mask, P);
        }
    } else if constexpr (KIND == kPow2Words) {
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
    } else if constexpr (KIND == kAnySmall) {
        reduce_small_depth<NW>(mask, D, P, n_int, d_min);
    } else if constexpr (KIND == kAnyMediumFew) {
        reduce_medium_depth<NW, 3>(mask, D, P, n_int, d_min);
    } else if constexpr (KIND == kAnyMedium) {
        reduce_medium_depth<NW, 5>(mask, D, P, n_int, d_min);
    } else {
        if constexpr (NW >= 2) reduce_large_depth<NW>(mask, D, P, n_int, d_min);
        else { n_int = D; d_min = D; }  // unreachable: more than 32 stages need more than one word
    }
}

// Calls f(integral_constant<int, kind>) for the reducer kind of the grid shape.
template <typename F>
__device__ __forceinline__ void with_reducer_kind(int D, int P, int log2P, F&& f)
{
    switch (reducer_kind(D, P, log2P)) {
        case kPow2Narrow: f(std::integral_constant<int, kPow2Narrow>{}); break;
        case kPow2Tree: f(std::integral_constant<int, kPow2Tree>{}); break;
        case kPow2Words: f(std::integral_constant<int, kPow2Words>{}); break;
        case kAnySmall: f(std::integral_constant<int, kAnySmall>{}); break;
        case kAnyMediumFew: f(std::integral_constant<int, kAnyMediumFew>{}); break;
        case kAnyMedium: f(std::integral_constant<int, kAnyMedium>{}); break;
        default: f(std::integral_constant<int, kAnyLarge>{}); break;
    }
}

template <int NW>
__device__ __forceinline__ void reduce_mask(const Mask<NW>& mask, int D, int P, int log2P, int& n_int, int& d_min)
{
    with_reducer_kind(D, P, log2P, [&](auto kind) {
        reduce_kind<NW, decltype(kind)::value>(mask, D, P, log2P, n_int, d_min);
    });
}

// ------------------------------------------------------------------ stage-occupancy statistic

// For a scenario in which every stage kept a survivor (d_min >= 1): one count per stage into the bin of its number
// of survivors (section 8.4: what an inter-stage migration costs depends on how many instances must receive state,
// and that follows from these counts for every target width).  Works for any depth: stage s owns the bits
// s, s + P, s + 2 P, ... of the mask; first[i] = first such bit of word i for the current stage, kept in step.
// The wave keeps 2, 4 or 8 copies of these bins (copy = lane mod copies, bin v of copy r at (v << shift) + r): most
// lanes of a wave hit the same one or two bins, a stage at a time, and the local memory takes lanes that add to one
// address one after the other; with a single copy those adds, one per stage and scenario, kept the local memory of
// the compute unit busy for longer than the vector units need for the rest of the scenario.
// Words of local memory per wave for the copies: as many as leave the kernel variant its resident waves.
__host__ __device__ constexpr int occ_words(int draw) { return draw == kDrawUniform ? 384 : (draw == kDrawZoned ? 520 : 768); }
__device__ __forceinline__ int occ_copies_shift(int nb, int words)
{
    return (nb << 3) <= words ? 3 : ((nb << 2) <= words ? 2 : ((nb << 1) <= words ? 1 : 0));
}

template <int NW>
__device__ __forceinline__ void stage_occupancy_add(const Mask<NW>& mask, int rows, int P, int group, int d_min,
                                                    uint32_t* bins_occ, int shift)
{
    // bin of a stage with `gone` lost instances, in this lane's copy: top - gone * step
    const uint32_t step = (uint32_t)group << shift;
    const uint32_t top = (uint32_t)rows * step + (uint32_t)(lane_id() & ((1 << shift) - 1));
    if ((P & (P - 1)) == 0 && P <= 32) {
        // the depth divides 32: stage s owns the same bits s, s + P, ... of every word
        uint32_t comb = period_comb(P);
        for (int s = 0; s < P; ++s, comb <<= 1) {
            uint32_t gone = 0u;
            static_for<NW>([&](auto i) { gone += (uint32_t)__popc(mask.w[i.value] & comb); });
            if (d_min >= 1) atomicAdd(&bins_occ[top - gone * step], 1u);
        }
        return;
    }
    const uint32_t period = P < 32 ? period_comb(P) : 1u;
    int first[NW];
    static_for<NW>([&](auto i) {
        int r = (-32 * i.value) % P;
        first[i.value] = r < 0 ? r + P : r;
    });
    for (int s = 0; s < P; ++s) {
        uint32_t gone = 0u;
        static_for<NW>([&](auto i) {
            const uint32_t comb = first[i.value] < 32 ? period << first[i.value] : 0u;
            gone += (uint32_t)__popc(mask.w[i.value] & comb);
            first[i.value] = first[i.value] + 1 == P ? 0 : first[i.value] + 1;
        });
        if (d_min >= 1) atomicAdd(&bins_occ[top - gone * step], 1u);
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

// Work queue of the sampling kernel, in the workspace.  The items are dealt to kQueueShards shards (item g
// belongs to shard g mod kQueueShards), each with its own claim counter: atomics on ONE address complete at a
// fixed, low rate (about 86 per microsecond on this chip), which a single counter would turn into the
// bottleneck of small launches.
constexpr int kQueueShards = 32;
// Claims a wave makes over a launch if all waves take equal shares (measured: 8 leaves a 4 % longer tail on a
// 1024-query batch, 128 is no better).
constexpr uint32_t kClaimsPerWave = 32;
constexpr int kShardStride = 64;  // counters sit 256 bytes apart: atomics on one cache line serialise too
struct WorkQueue {
    uint32_t* list;   // [n_units] global unit indices (q * T * C + t * C + c) that need sampling, any order
    uint32_t* count;  // number of entries of list
    uint32_t* next;   // [kQueueShards * kShardStride] items handed out so far in shard i at next[i * kShardStride]
};

// Clears the histograms, writes the single bin of the units that need no sampling, resets the work queue.
__global__ void __launch_bounds__(256) prep_hist_kernel(Batch b, WorkQueue wq, uint32_t* __restrict__ hist_int,
                                                        uint32_t* __restrict__ hist_min)
{
    if (blockIdx.x == 0 && threadIdx.x < kQueueShards) {
        if (threadIdx.x == 0) *wq.count = 0u;
        wq.next[threadIdx.x * kShardStride] = 0u;
    }
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
        unit_pool(b, q, t, cr.D, cr.P, M, k);
        int bin;
        const bool single = unit_closed_form(cr.D / b.group, cr.P, M, k, bin) && j == bin * b.group;
        const uint32_t v = single ? (uint32_t)b.S : 0u;
        hist_int[e] = v;
        hist_min[e] = v;
        // stage-occupancy statistic of such a unit: every stage of every scenario has `bin` survivors, and a unit
        // that lost a stage (bin 0) counts nothing
        if (b.hist_occ) b.hist_occ[e] = (single && bin >= 1) ? (uint32_t)b.S * (uint32_t)cr.P : 0u;
    }
}

// Appends every unit that needs sampling to the work list: one thread per unit, positions inside the
// block by ballot + LDS prefix, ONE global atomic per block of 1024 units (atomics on one address are slow).
constexpr int kBuildThreads = 1024;
__global__ void __launch_bounds__(kBuildThreads) build_work_kernel(Batch b, WorkQueue wq)
{
    constexpr int kWaves = kBuildThreads / kWave;
    __shared__ uint32_t wave_count[kWaves];
    __shared__ uint32_t wave_base[kWaves];
    const int64_t n_units = (int64_t)b.nq * b.T * b.C;
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool need = false;
    if (u < n_units) {
        const int tc = (int)(u % ((int64_t)b.T * b.C));
        const int q = (int)(u / ((int64_t)b.T * b.C));
        const int t = tc / b.C;
        const CfgRec cr = b.cfg[tc - t * b.C];
        int M, k, bin;
        unit_pool(b, q, t, cr.D, cr.P, M, k);
        need = !unit_closed_form(cr.D / b.group, cr.P, M, k, bin);
    }
    const unsigned long long votes = __ballot(need);
    const int lane = lane_id();
    const int wave = (int)threadIdx.x / kWave;
    if (lane == 0) wave_count[wave] = (uint32_t)__popcll(votes);
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t sum = 0u;
        for (int w = 0; w < kWaves; ++w) {
            wave_base[w] = sum;
            sum += wave_count[w];
        }
        const uint32_t base = sum ? atomicAdd(wq.count, sum) : 0u;
        for (int w = 0; w < kWaves; ++w) wave_base[w] += base;
    }
    __syncthreads();
    if (need) wq.list[wave_base[wave] + (uint32_t)__popcll(votes & ((1ull << lane) - 1ull))] = (uint32_t)u;
}

// Small problems: everything that has to happen before the sampling kernel, in ONE workgroup and one launch.  The
// candidate table arrives in the kernel's arguments and is written to the workspace for the kernels that follow; a
// thread per unit clears the unit's histogram rows (or writes their single bin), and the units that need sampling
// are appended to the work list by ballot and prefix inside the workgroup, so no counter has to be reset first.
constexpr int kStageThreads = 1024;
constexpr int kStageMaxConfigs = 64;
constexpr int64_t kStageMaxUnits = 2 * kStageThreads;
constexpr int64_t kStageMaxBins = 32 * kStageThreads;  // histogram words a thread writes one by one: few, or the launches pay
struct StageTable {
    CfgRec rec[kStageMaxConfigs];
};

__global__ void __launch_bounds__(kStageThreads) stage_small_kernel(Batch b, StageTable table, CfgRec* __restrict__ cfg_out,
                                                                    WorkQueue wq, uint32_t* __restrict__ hist_int,
                                                                    uint32_t* __restrict__ hist_min)
{
    constexpr int kWaves = kStageThreads / kWave;
    __shared__ CfgRec cfg[kStageMaxConfigs];
    __shared__ uint32_t wave_count[kWaves];
    __shared__ uint32_t wave_base[kWaves];
    __shared__ uint32_t listed;
    const int tid = (int)threadIdx.x;
    const int lane = lane_id();
    const int wave = tid / kWave;
    if (tid < b.C) {
        cfg[tid] = table.rec[tid];
        cfg_out[tid] = table.rec[tid];
    }
    if (tid < kQueueShards) wq.next[tid * kShardStride] = 0u;
    if (tid == 0) listed = 0u;
    __syncthreads();
    const int64_t n_units = (int64_t)b.nq * b.T * b.C;
    for (int64_t first = 0; first < n_units; first += kStageThreads) {
        const int64_t u = first + tid;
        bool need = false;
        if (u < n_units) {
            const int c = (int)(u % b.C);
            const int64_t qt = u / b.C;
            const int t = (int)(qt % b.T);
            const int q = (int)(qt / b.T);
            const CfgRec cr = cfg[c];
            int M, k, bin;
            unit_pool(b, q, t, cr.D, cr.P, M, k);
            const bool closed = unit_closed_form(cr.D / b.group, cr.P, M, k, bin);
            need = !closed;
            const int at = closed ? bin * b.group : -1;
            const int64_t row = qt * b.L + cr.off;
            for (int j = 0; j <= cr.D; ++j) {
                const uint32_t v = j == at ? (uint32_t)b.S : 0u;
                hist_int[row + j] = v;
                hist_min[row + j] = v;
                if (b.hist_occ) b.hist_occ[row + j] = (j == at && bin >= 1) ? (uint32_t)b.S * (uint32_t)cr.P : 0u;
            }
        }
        const unsigned long long votes = __ballot(need);
        if (lane == 0) wave_count[wave] = (uint32_t)__popcll(votes);
        __syncthreads();
        if (tid == 0) {
            uint32_t sum = listed;
            for (int w = 0; w < kWaves; ++w) {
                wave_base[w] = sum;
                sum += wave_count[w];
            }
            listed = sum;
        }
        __syncthreads();
        if (need) wq.list[wave_base[wave] + (uint32_t)__popcll(votes & ((1ull << lane) - 1ull))] = (uint32_t)u;
    }
    __syncthreads();
    if (tid == 0) *wq.count = listed;
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

// One wave, scenarios [s_begin, s_end) of one unit, 64 at a time.  zc / wc: zones or weights of the pool for the
// draws that are not uniform.  kMoves adds the stage-occupancy statistic (bins_occ).
template <int NW, int kDraw, bool kMoves, int KIND>
__device__ __forceinline__ void eval_unit_chunk(const CfgRec cr, int group, int M, int k, uint32_t unit,
                                                uint32_t stream_id, const PhiloxKeys& ks, uint32_t s_begin,
                                                uint32_t s_end, uint32_t* lds_col, uint32_t* bins_int,
                                                uint32_t* bins_min, uint32_t* bins_occ, int occ_shift,
                                                const ZoneCtx* zc, const WeightCtx* wc)
{
    const int rows = cr.D / group;  // pipelines of the instance grid
    for (uint32_t s = s_begin + (uint32_t)lane_id(); s < s_end; s += kWave) {
        int n_int, d_min;
        Mask<NW> mask;
        if constexpr (kDraw == kDrawZoned) sample_mask_zoned<NW>(mask, lds_col, kEvalThreads, *zc, k, s, unit, stream_id, ks);
        else if constexpr (kDraw == kDrawWeighted) sample_mask_weighted<NW>(mask, *wc, M, k, s, unit, stream_id, ks);
        else draw_scenario<NW>(mask, lds_col, M, k, s, unit, stream_id, ks);
        if (M > rows * cr.P) mask.keep_below(rows * cr.P);  // idle instances of the pool are not on the grid
        reduce_kind<NW, KIND>(mask, rows, cr.P, cr.log2P, n_int, d_min);
        hist_add(bins_int, n_int * group, true);
        hist_add(bins_min, d_min * group, true);
        if constexpr (kMoves) stage_occupancy_add<NW>(mask, rows, cr.P, group, d_min, bins_occ, occ_shift);
    }
}

// Persistent kernel: every wave pulls (unit, chunk) items from the work queue until it is empty, so waves never
// wait for each other and units without sampling cost nothing here.  Item i is chunk i % n_chunks of
// list[i / n_chunks]; a chunk is chunk_len consecutive scenarios.  Each wave owns a slice of the LDS bins.
// kDraw selects how scenarios are drawn and kMoves adds the stage-occupancy statistic (kernels of their own, so
// the plain one keeps its registers).
template <int kDraw, bool kMoves>
__global__ void __launch_bounds__(kEvalThreads) __attribute__((amdgpu_waves_per_eu(kDraw != kDrawUniform ? 5 : 7, 8))) eval_hist_kernel(Batch b, WorkQueue wq, int n_resident_waves,
                                                                 uint32_t* __restrict__ hist_int,
                                                                 uint32_t* __restrict__ hist_min)
{
    constexpr int kWaves = kEvalThreads / kWave;
    constexpr bool kZoned = kDraw == kDrawZoned;
    constexpr bool kWeighted = kDraw == kDrawWeighted;
    __shared__ uint32_t bins_all[kWaves][2 * (kMaxInstances + 1) + (kMoves ? occ_words(kDraw) : 0)];
    __shared__ uint32_t lmask[8 * kEvalThreads];  // sets of units with more than 64 instances, [word][lane]
    __shared__ uint8_t zone_perm[kZoned ? kWaves : 1][kMaxZones * 256];
    __shared__ uint32_t zone_mask[kZoned ? kWaves : 1][kMaxZones * 8];
    __shared__ __align__(16) uint8_t weight_bytes[kWeighted ? kWaves : 1][272];
    const int lane = lane_id();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // the same in every lane
    uint32_t* bins = bins_all[wave];
    uint32_t* lds_col = lmask + threadIdx.x;
    // the length of an item follows from the number of units on the list (the same value in every wave)
    const uint32_t n_listed = *wq.count;
    const int chunk_len = pick_chunk_len((int64_t)n_listed, b.S, b.N, (int64_t)n_resident_waves);
    const int n_chunks = (b.S + chunk_len - 1) / chunk_len;
    const uint32_t total = n_listed * (uint32_t)n_chunks;
    // Shard s holds the items g with g mod kQueueShards == s (neighbouring items cost about the same, whole ranges of
    // the list do not: interleaving gives every shard the same mix).  A wave claims `batch` items of its current
    // shard at a time; that is its home shard until it runs dry.  Then the wave looks at all shard counters AT ONCE
    // (one load per lane, one round trip) and moves to one of the shards that still have items, a different one for
    // different waves; a walk over the shards one probe after the other would cost a memory round trip per shard in
    // every wave at the end of the launch.  A wave leaves when no shard has items left; counters only grow, so that
    // point is reached.
    // The first item of a wave is the one with the wave's own index: nothing to claim, so a launch with no more items
    // than waves touches no counter at all (claims of single items by thousands of waves at once would queue up at
    // the few counters).  The shards hand out the items past those.
    const uint32_t n_waves = (uint32_t)gridDim.x * kWaves;
    auto shard_size = [&](uint32_t s) { return s < total ? (total - s + kQueueShards - 1u) / kQueueShards : 0u; };
    auto shard_first = [&](uint32_t s) { return s < n_waves ? (n_waves - s + kQueueShards - 1u) / kQueueShards : 0u; };
    uint32_t batch = total / (n_waves * kClaimsPerWave);
    batch = batch < 1u ? 1u : (batch > 64u ? 64u : batch);
    const uint32_t wave_id = (uint32_t)blockIdx.x * kWaves + wave;
    uint32_t shard = wave_id % kQueueShards;
    uint32_t slot = 0u, slot_end = 0u;  // position inside the shard: item = slot * kQueueShards + shard
    bool own_item = wave_id < total;

    for (;;) {
        bool drained = false;
        while (!own_item && slot == slot_end) {
            const uint32_t size = shard_size(shard);
            const uint32_t skip = shard_first(shard);
            if (size > skip) {
                uint32_t got = 0u;
                if (lane == 0) got = atomicAdd(&wq.next[shard * kShardStride], batch);
                const uint32_t first = __builtin_amdgcn_readfirstlane(got) + skip;
                if (first < size) {
                    slot = first;
                    slot_end = first + batch < size ? first + batch : size;
                    break;
                }
            }
            bool has_items = false;
            if (lane < kQueueShards) {
                const uint32_t taken =
                    __hip_atomic_load(&wq.next[lane * kShardStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                has_items = taken + shard_first((uint32_t)lane) < shard_size((uint32_t)lane);
            }
            const unsigned long long open = __ballot(has_items);
            if (open == 0ull) {
                drained = true;
                break;
            }
            const uint32_t pick = wave_id % (uint32_t)__popcll(open);
            unsigned long long rest = open;
            for (uint32_t i = 0; i < pick; ++i) rest &= rest - 1ull;  // drop the lowest set bit
            shard = (uint32_t)__builtin_ctzll(rest);
        }
        if (drained) break;
        uint32_t item;
        if (own_item) {
            item = wave_id;
            own_item = false;
        } else {
            item = slot * kQueueShards + shard;
            ++slot;
        }
        const uint32_t unit_global = wq.list[item / (uint32_t)n_chunks];
        const int chunk = (int)(item % (uint32_t)n_chunks);
        const int tc = (int)(unit_global % (uint32_t)(b.T * b.C));
        const int q = (int)(unit_global / (uint32_t)(b.T * b.C));
        const int t = tc / b.C;
        const int c = tc - t * b.C;
        const CfgRec cr = b.cfg[c];
        int M, k;
        unit_pool(b, q, t, cr.D, cr.P, M, k);

        const int nb = cr.D + 1;
        uint32_t* bins_int = bins;
        uint32_t* bins_min = bins + nb;
        uint32_t* bins_occ = bins + 2 * nb;  // used with kMoves only: (1 << occ_shift) copies of nb bins
        const int occ_shift = occ_copies_shift(nb, occ_words(kDraw));
        for (int i = lane; i < 2 * nb + (kMoves ? nb << occ_shift : 0); i += kWave) bins[i] = 0u;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        const uint64_t seed = b.seed[q];
        const PhiloxKeys ks = philox_keys((uint32_t)(seed & 0xffffffffull), (uint32_t)(seed >> 32));
        const uint32_t stream_id = (b.stream_id ? b.stream_id[q] : 0u) + b.stream_offset;
        const uint32_t s_begin = (uint32_t)chunk * (uint32_t)chunk_len;
        uint32_t s_end = s_begin + (uint32_t)chunk_len;
        s_end = s_end > (uint32_t)b.S ? (uint32_t)b.S : s_end;

        ZoneCtx zc;
        WeightCtx wc;
        if constexpr (kZoned) zc = zone_setup(b, q, M, zone_perm[wave], zone_mask[wave]);
        if constexpr (kWeighted) wc = weight_setup(b, q, M, weight_bytes[wave]);
        with_reducer_kind(cr.D / b.group, cr.P, cr.log2P, [&](auto kind) {
            constexpr int K = decltype(kind)::value;
            // kinds that need more than 32 stages cannot meet a one-word pool
            if (M <= 32) {
                if constexpr (K != kPow2Words && K != kAnyLarge)
                    eval_unit_chunk<1, kDraw, kMoves, K>(cr, b.group, M, k, (uint32_t)tc, stream_id, ks, s_begin, s_end, lds_col, bins_int, bins_min, bins_occ, occ_shift, &zc, &wc);
            } else if (M <= 64) {
                eval_unit_chunk<2, kDraw, kMoves, K>(cr, b.group, M, k, (uint32_t)tc, stream_id, ks, s_begin, s_end, lds_col, bins_int, bins_min, bins_occ, occ_shift, &zc, &wc);
            } else if (M <= 128) {
                eval_unit_chunk<4, kDraw, kMoves, K>(cr, b.group, M, k, (uint32_t)tc, stream_id, ks, s_begin, s_end, lds_col, bins_int, bins_min, bins_occ, occ_shift, &zc, &wc);
            } else {
                eval_unit_chunk<8, kDraw, kMoves, K>(cr, b.group, M, k, (uint32_t)tc, stream_id, ks, s_begin, s_end, lds_col, bins_int, bins_min, bins_occ, occ_shift, &zc, &wc);
            }
        });
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        const int64_t base = ((int64_t)q * b.T + t) * b.L + cr.off;
        for (int i = lane; i < nb; i += kWave) {
            const uint32_t vi = bins_int[i], vm = bins_min[i];
            if (n_chunks == 1) {
                hist_int[base + i] = vi;
                hist_min[base + i] = vm;
            } else {
                if (vi) atomicAdd(&hist_int[base + i], vi);
                if (vm) atomicAdd(&hist_min[base + i], vm);
            }
            if constexpr (kMoves) {
                uint32_t vo = 0u;
                for (int r = 0; r < (1 << occ_shift); ++r) vo += bins_occ[(i << occ_shift) + r];
                if (n_chunks == 1) b.hist_occ[base + i] = vo;
                else if (vo) atomicAdd(&b.hist_occ[base + i], vo);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// One scenario through the same code path the histogram kernel takes for a unit of this size.
template <int NW>
__device__ __forceinline__ void debug_one(const CfgRec cr, int group, uint32_t* lds_col, int M, int k, uint32_t s, uint32_t unit,
                                          uint32_t stream_id, const PhiloxKeys& ks, const ZoneCtx* zc, const WeightCtx* wc,
                                          uint32_t* mask_out, int& n_int, int& d_min)
{
    Mask<NW> mask;
    if (wc) sample_mask_weighted<NW>(mask, *wc, M, k, s, unit, stream_id, ks);
    else if (zc) sample_mask_zoned<NW>(mask, lds_col, kEvalThreads, *zc, k, s, unit, stream_id, ks);
    else draw_scenario<NW>(mask, lds_col, M, k, s, unit, stream_id, ks);
    static_for<8>([&](auto i) {
        if constexpr (i.value < NW) mask_out[i.value] = mask.w[i.value];
        else mask_out[i.value] = 0u;
    });
    const int rows = cr.D / group;
    if (M > rows * cr.P) mask.keep_below(rows * cr.P);
    reduce_mask<NW>(mask, rows, cr.P, cr.log2P, n_int, d_min);
    n_int *= group;
    d_min *= group;
}

// Scenarios one by one, for inspection: masks [ns][8], n_int [ns], d_min [ns].
__global__ void __launch_bounds__(kEvalThreads) debug_sample_kernel(Batch b, int q, int t, int c, uint32_t s0,
                                                                    uint32_t ns, uint32_t* __restrict__ masks,
                                                                    int32_t* __restrict__ n_int_out,
                                                                    int32_t* __restrict__ d_min_out)
{
    __shared__ uint32_t lmask[8 * kEvalThreads];
    __shared__ uint8_t zone_perm[kEvalThreads / kWave][kMaxZones * 256];
    __shared__ uint32_t zone_mask[kEvalThreads / kWave][kMaxZones * 8];
    __shared__ __align__(16) uint8_t weight_bytes[kEvalThreads / kWave][272];
    const uint32_t x = blockIdx.x * blockDim.x + threadIdx.x;
    const CfgRec cr = b.cfg[c];
    int M, k;
    unit_pool(b, q, t, cr.D, cr.P, M, k);
    ZoneCtx zones;
    WeightCtx weights;
    const ZoneCtx* zc = nullptr;
    const WeightCtx* wc = nullptr;
    const int wave = (int)threadIdx.x / kWave;
    if (b.inst_weight) {  // every lane takes part in building the tables, also those past the last scenario
        weights = weight_setup(b, q, M, weight_bytes[wave]);
        wc = &weights;
    } else if (b.n_zones > 0) {
        zones = zone_setup(b, q, M, zone_perm[wave], zone_mask[wave]);
        zc = &zones;
    }
    // No lane leaves early: the weighted draw reads the weights out of other lanes' registers, so every lane runs
    // the draw (lanes past the last scenario redo scenario s0) and only the stores are predicated.
    const bool live = x < ns;
    const uint32_t xs = live ? x : 0u;
    const uint64_t seed = b.seed[q];
    const PhiloxKeys ks = philox_keys((uint32_t)(seed & 0xffffffffull), (uint32_t)(seed >> 32));
    const uint32_t stream_id = (b.stream_id ? b.stream_id[q] : 0u) + b.stream_offset;
    const uint32_t unit = (uint32_t)(t * b.C + c);
    uint32_t* lds_col = lmask + threadIdx.x;
    uint32_t out[8];
    int n_int, d_min;
    if (M <= 32) debug_one<1>(cr, b.group, lds_col, M, k, s0 + xs, unit, stream_id, ks, zc, wc, out, n_int, d_min);
    else if (M <= 64) debug_one<2>(cr, b.group, lds_col, M, k, s0 + xs, unit, stream_id, ks, zc, wc, out, n_int, d_min);
    else if (M <= 128) debug_one<4>(cr, b.group, lds_col, M, k, s0 + xs, unit, stream_id, ks, zc, wc, out, n_int, d_min);
    else debug_one<8>(cr, b.group, lds_col, M, k, s0 + xs, unit, stream_id, ks, zc, wc, out, n_int, d_min);
    if (live) {
        static_for<8>([&](auto i) { masks[(size_t)x * 8 + i.value] = out[i.value]; });
        n_int_out[x] = n_int;
        d_min_out[x] = d_min;
    }
}

}  // namespace parcae
