// Receding-horizon replay: the per-step bookkeeping between two planner calls (algorithm 1's loop,
// section 7 "parallelization adaptation", reactive baseline of section 9.4).
#pragma once

#include "device_common.hpp"

namespace parcae {

constexpr int kReplayProactive = 0;
constexpr int kReplayReactive = 1;
constexpr int kNothingRunning = -2;  // state value: training is suspended / not started

__device__ __forceinline__ bool replay_fits(const Batch& b, int c, int a) { return b.cfg[c].D * b.cfg[c].P <= b.group * a; }

// Widest candidate of depth `depth` that fits a instances, -1 if none.
__device__ __forceinline__ int replay_widest(const Batch& b, int depth, int a)
{
    int arg = -1, width = 0;
    for (int c = 0; c < b.C; ++c) {
        const CfgRec cr = b.cfg[c];
        if (cr.P == depth && replay_fits(b, c, a) && cr.D > width) {
            width = cr.D;
            arg = c;
        }
    }
    return arg;
}

// state[q] = configuration running now, total[q] = 0.  Negative inputs mean nothing is running; an index past the
// candidate list (flagged as invalid input by the checks) is treated the same way, so that no later kernel indexes
// the candidate table with it.
__global__ void __launch_bounds__(256) replay_init_kernel(int nq, int C, const int32_t* __restrict__ cur_config,
                                                          int32_t* __restrict__ state, float* __restrict__ total)
{
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nq) return;
    const int c = cur_config ? cur_config[q] : -1;
    state[q] = (c < 0 || c >= C) ? kNothingRunning : c;
    total[q] = 0.0f;
}

// Clears valid[q] when an entry of the true walk [nq][n_steps + 1] or of a forecast window [n_steps][nq][T + 1]
// (windows may be null) lies outside [0, N].  One block per query; valid[q] was set by the input checks before.
__global__ void __launch_bounds__(256) replay_validate_kernel(int nq, int n_steps, int T, int N,
                                                              const int32_t* __restrict__ true_avail,
                                                              const int32_t* __restrict__ windows,
                                                              int32_t* __restrict__ valid)
{
    const int q = blockIdx.x;
    int bad = 0;
    for (int i = threadIdx.x; i <= n_steps; i += blockDim.x) {
        const int a = true_avail[(int64_t)q * (n_steps + 1) + i];
        bad |= (a < 0 || a > N) ? 1 : 0;
    }
    if (windows) {
        const int per_step = T + 1;
        for (int x = threadIdx.x; x < n_steps * per_step; x += blockDim.x) {
            const int i = x / per_step, t = x - i * per_step;
            const int a = windows[((int64_t)i * nq + q) * per_step + t];
            bad |= (a < 0 || a > N) ? 1 : 0;
        }
    }
    if (bad) valid[q] = 0;  // every writer stores the same value
}

// One thread per query: target of step i (first configuration of the plan, or the fastest fitting candidate
// for the reactive baseline), adaptation to the actual availability, reward of the transition from the
// histograms of the one-interval problem (true[i] -> true[i + 1]), state update.
__global__ void __launch_bounds__(256) replay_step_kernel(
    Batch b, int mode, int step, int n_steps, int plan_T, const int32_t* __restrict__ true_avail,
    const int32_t* __restrict__ window, const int32_t* __restrict__ plan, const uint32_t* __restrict__ hist_int,
    const uint32_t* __restrict__ hist_min, int32_t* __restrict__ state, int32_t* __restrict__ chosen,
    float* __restrict__ reward, float* __restrict__ total)
{
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= b.nq) return;
    const int a = clampi(true_avail[(int64_t)q * (n_steps + 1) + step + 1], 0, b.N);
    const int cur = state[q];
    const float* thr = b.thr + (int64_t)q * b.L;
    const float* cost = b.cost + (int64_t)q * b.C * 3;

    int target, forecast;
    if (mode == kReplayProactive) {
        target = plan[(int64_t)q * plan_T];
        if (target < 0) target = cur;  // no feasible plan: keep what runs
        forecast = clampi(window[(int64_t)q * (plan_T + 1) + 1], 0, b.N);
    } else {
        float best = -1.0f;
        target = -1;
        for (int c = 0; c < b.C; ++c) {
            const CfgRec cr = b.cfg[c];
            const float f = thr[cr.off + cr.D];
            if (cr.P >= b.p_min && replay_fits(b, c, a) && f > best) {
                best = f;
                target = c;
            }
        }
        forecast = a;
    }

    // adaptation: keep the depth, add or drop pipelines; fewer stages if no pipeline of that depth fits
    int next = -1;
    if (target >= 0) {
        if (a == forecast && replay_fits(b, target, a)) {
            next = target;
        } else {
            const int depth = b.cfg[target].P;
            next = replay_widest(b, depth, a);
            if (next < 0) {
                // candidates are sorted by depth: walk the shallower depths from the deepest down
                int last_depth = depth;
                for (int c = b.C - 1; c >= 0 && next < 0; --c) {
                    const int d = b.cfg[c].P;
                    if (d >= last_depth || d < b.p_min) continue;
                    last_depth = d;
                    next = replay_widest(b, d, a);
                }
            }
        }
    }

    // reward: expected committed samples of cur -> next (transition weight with the class rule)
    float r = 0.0f;
    if (next >= 0) {
        const CfgRec z = b.cfg[next];
        const float full = thr[z.off + z.D];
        const float e0 = fmaxf(0.0f, __fsub_rn(b.tau, cost[3 * next + 0]));
        const float e1 = fmaxf(0.0f, __fsub_rn(b.tau, cost[3 * next + 1]));
        const float e2 = fmaxf(0.0f, __fsub_rn(b.tau, cost[3 * next + 2]));
        if (cur < 0 || b.cfg[cur].P != z.P) {
            r = __fmul_rn(full, e2);
        } else {
            const CfgRec s = b.cfg[cur];
            const uint32_t* hi = hist_int + (int64_t)q * b.L + s.off;
            const uint32_t* hm = hist_min + (int64_t)q * b.L + s.off;
            uint32_t n0 = 0u, n01 = 0u;
            for (int j = z.D; j <= s.D; ++j) {
                n0 += hi[j];
                n01 += hm[j];
            }
            const uint32_t n3 = hm[0];
            const uint32_t n1 = n01 - n0, n2 = (uint32_t)b.S - n01 - n3;
            const float round_sec = b.cost_round ? b.cost_round[(int64_t)q * b.C + next] : 0.0f;
            float inter;
            if (round_sec == 0.0f) {
                inter = __fmul_rn((float)n2, e1);
            } else {
                auto tail = [&](int x) {
                    uint32_t sum = 0u;
                    for (int j = x; j <= s.D; ++j) sum += hm[j];
                    return sum;
                };
                inter = inter_seconds_by_rounds(tail, z.D, b.tau, cost[3 * next + 1], cost[3 * next + 2], round_sec);
            }
            float num = __fadd_rn(__fmul_rn((float)n0, b.tau), __fmul_rn((float)n1, e0));
            num = __fadd_rn(num, inter);
            num = __fadd_rn(num, __fmul_rn((float)n3, e2));
            r = __fmul_rn(full, __fdiv_rn(num, (float)b.S));
        }
    }
    chosen[(int64_t)q * n_steps + step] = next;
    reward[(int64_t)q * n_steps + step] = r;
    total[q] = __fadd_rn(total[q], r);
    state[q] = next < 0 ? kNothingRunning : next;
}

}  // namespace parcae
