// Shared device-side definitions of the liveput kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace parcae {

constexpr int kWave = 64;
constexpr int kMaxInstances = 256;

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
    float tau;
    const CfgRec* cfg;          // [C]
    const int32_t* avail;       // [nq][T+1]
    const float* thr;           // [nq][L]
    const float* cost;          // [nq][C][3]
    const uint64_t* seed;       // [nq]
    const uint32_t* stream_id;  // [nq] or null
    const int32_t* cur_config;  // [nq] or null
};

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

// Instances used (M) and preempted (k) when configuration (D, P) meets availability a (section 4.2).
__device__ __forceinline__ void unit_pool(int D, int P, int a, int N, int& M, int& k)
{
    M = D * P;
    a = clampi(a, 0, N);
    k = M - a;
    k = k < 0 ? 0 : k;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

}  // namespace parcae
