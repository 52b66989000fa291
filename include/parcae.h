/*
 * parcae.h - C ABI of the liveput optimizer's hot path on one AMD CDNA4 GPU.
 *
 * The library evaluates, for every candidate parallel configuration (D
 * data-parallel pipelines x P pipeline stages) and every look-ahead interval,
 * the Monte-Carlo statistics that liveput needs (Parcae, arXiv 2403.14097,
 * Definition 1 / Eq. 1 and section 6.3), and runs the look-ahead dynamic program
 * that picks the configuration sequence with the most committed samples net of
 * migration cost (Eq. 3-6, section 6.2).
 *
 * ------------------------------------------------------------------------
 * Conventions common to all calls
 * ------------------------------------------------------------------------
 * Memory.  A pointer is marked HOST or DEVICE.  The caller owns every buffer
 * (calls that may overlap in time need separate workspaces);
 * the library allocates nothing, frees nothing and keeps no state between
 * calls.  DEVICE buffers must be ordinary device allocations of the current
 * HIP device and must not overlap each other.  HOST data is read before the
 * call returns.
 *
 * Asynchrony.  Work is enqueued on `stream` (a hipStream_t passed as void*,
 * NULL = the null stream).  Outputs are valid once the stream has been
 * synchronised.  No call synchronises the device; a call enqueues kernels
 * only (no memset or memcpy nodes: memory is cleared by kernels and the
 * candidate table travels as kernel arguments).
 *
 * Errors.  Every call returns 0 (PARCAE_OK) or a negative code.  Shape errors
 * that the host can see (NULL pointers, sizes out of range, candidate list not
 * sorted, workspace too small) are returned at once and nothing is enqueued.
 * Errors that live in DEVICE data are found by the kernels and reported per
 * query in the DEVICE array `status` (see parcae_liveput_plan).  The library
 * never throws, never writes errno and never prints.
 *
 * ------------------------------------------------------------------------
 * The problem (one batch of nq independent planning queries)
 * ------------------------------------------------------------------------
 * All queries of a batch share N, T, the interval length, the candidate list
 * and the scenario count; each query has its own availability sequence,
 * throughput table, cost table, seed and current configuration.
 *
 * Candidate c = (D_c, P_c): D_c >= 1, P_c >= 1, D_c * P_c <= N <= 256 (D_c <= 256
 * and D_c * P_c <= g * N with multi-GPU instances, see below).  The
 * list is strictly increasing in (P, D) lexicographic order (so index order
 * prefers shallower, then narrower configurations when the planner breaks
 * ties).  off[c] = sum over c' < c of (D_c' + 1); L = off[C].
 *
 * Availability (section 4.2): avail[q][0] is the number of instances now,
 * avail[q][1 + t] is the predicted number in look-ahead interval t,
 * t = 0..T-1; every entry lies in [0, N].  Preemptions and allocations happen
 * only at interval starts.
 *
 * Throughput: thr[q][off[c] + d] = samples per second of d pipelines of depth
 * P_c, d = 0..D_c; finite, >= 0, thr[q][off[c]] == 0.  A configuration that
 * does not fit device memory is expressed by P_c < p_min (section 6.2: such a
 * configuration has no throughput and is never chosen).
 *
 * Migration cost (section 5.2, section 8.4): cost[q][c] = seconds of an
 * intra-stage migration, an inter-stage migration and a re-partition
 * (pipeline migration) INTO configuration c; finite, 0 <= intra <= inter <=
 * re-partition.
 */
#ifndef PARCAE_H
#define PARCAE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PARCAE_MAX_INSTANCES 256        /* N limit: one preemption mask is 256 bits */
#define PARCAE_MAX_SCENARIOS 16777216   /* S limit: counts stay exact in float      */
#define PARCAE_MASK_WORDS 8
#define PARCAE_MAX_ZONES 4

/* parcae_problem.flags */
#define PARCAE_POOL_USED 0u /* preemptions fall on the D * P instances the configuration uses (default) */
#define PARCAE_POOL_ALL 1u  /* preemptions fall on any of the available instances, idle ones included  */

#define PARCAE_COLD_START (-2) /* cur_config value: nothing is running, see the transition weight */

#define PARCAE_OK 0
#define PARCAE_EINVAL (-1)       /* bad argument or bad input data                       */
#define PARCAE_EWORKSPACE (-2)   /* workspace NULL, misaligned (256 B) or too small      */
#define PARCAE_EHIP (-3)         /* a HIP call or kernel launch failed                   */
#define PARCAE_EINFEASIBLE (-4)  /* per query: no configuration sequence is feasible     */

typedef struct parcae_config {
    int32_t D; /* data-parallel pipelines */
    int32_t P; /* pipeline stages         */
} parcae_config;

/*
 * Profiling hooks (HOST struct, optional).  Each member is a hipEvent_t passed as void*, or NULL.  The
 * library records the event on the call's stream at the named point; it never waits for one.
 */
typedef struct parcae_profile {
    void *event_before_sampling; /* right before the scenario sampling kernel is launched */
    void *event_after_sampling;  /* right after it                                        */
    void *event_before_plan;     /* right before the first kernel of the dynamic program  */
    void *event_after_plan;      /* right after its last kernel                           */
} parcae_profile;

typedef struct parcae_problem {
    uint32_t struct_size; /* sizeof(parcae_problem) of the caller's build: the structure only ever
                             grows at its end, a library reads no member past this size (absent
                             members count as 0 / NULL) and refuses a size below the first release's */
    int32_t n_queries;   /* nq >= 1                                                     */
    int32_t n_instances; /* N, 1..PARCAE_MAX_INSTANCES                                  */
    int32_t n_intervals; /* T >= 1 look-ahead intervals (the paper's I)                 */
    int32_t n_configs;   /* C >= 1, C * T < 2^31                                        */
    int32_t n_scenarios; /* S, 1..PARCAE_MAX_SCENARIOS Monte-Carlo scenarios per (t, c) */
    int32_t p_min;       /* smallest pipeline depth that fits device memory             */
    float interval_sec;  /* interval length in seconds (the paper's T), > 0, finite     */
    uint32_t flags;      /* PARCAE_POOL_USED or PARCAE_POOL_ALL                         */
    const parcae_config *configs; /* HOST   [C]                                         */
    const int32_t *avail;         /* DEVICE [nq][T + 1]                                 */
    const float *thr;             /* DEVICE [nq][L]                                     */
    const float *cost;            /* DEVICE [nq][C][3]                                  */
    const uint64_t *seed;         /* DEVICE [nq]  Philox key of the query               */
    const uint32_t *stream_id;    /* DEVICE [nq] or NULL (= 0): Philox counter word 3   */
    const int32_t *cur_config;    /* DEVICE [nq] or NULL (= -1): index of the
                                     configuration running now, -1 = any,
                                     PARCAE_COLD_START = nothing is running            */
    int32_t group_size;           /* g, GPUs per instance, 0 or 1 = single-GPU instances,
                                     at most 64; see "Multi-GPU instances" below         */
    int32_t n_zones;              /* 0 = every instance equally likely to be preempted;
                                     1..PARCAE_MAX_ZONES: see "Non-uniform preemption"   */
    const uint8_t *zone;          /* DEVICE [nq][N] zone of every instance (n_zones > 0)  */
    const uint32_t *zone_weight;  /* DEVICE [nq][PARCAE_MAX_ZONES] hazard weight of every
                                     zone, 1..255 for z < n_zones (n_zones > 0)           */
    const float *cost_round;      /* DEVICE [nq][C] or NULL (= 0): seconds per further
                                     state-transfer round of an inter-stage migration INTO
                                     configuration c, finite, >= 0; see "Transfer rounds"  */
    const parcae_profile *profile; /* HOST or NULL: profiling hooks, read before the call returns */
    const uint8_t *inst_weight;   /* DEVICE [nq][N] or NULL: hazard weight 1..255 of every instance; see
                                     "A weight per instance" below; not together with n_zones > 0  */
    const float *cost_move;       /* DEVICE [nq][C] or NULL (= 0): seconds per instance that must receive
                                     state in an inter-stage migration INTO configuration c; see
                                     "Moved instances" below; not together with cost_round; needs hist_occ */
    uint32_t *hist_occ;           /* DEVICE [nq][T][L] uint32, used with cost_move only: the stage-occupancy
                                     statistic, written by the evaluation, read by the planning calls    */
} parcae_problem;

/*
 * ------------------------------------------------------------------------
 * What is computed (the definitions every entry point refers to)
 * ------------------------------------------------------------------------
 * Unit (q, t, c): configuration c, running in interval t - 1 (now, for
 * t = 0), meets the boundary into interval t.  A pool of M instances loses k
 * of them; logical instance j = d * P + s < D * P is stage s of pipeline d,
 * instances D * P .. M - 1 are idle.
 *   PARCAE_POOL_USED: M = D * P, k = max(0, M - avail[q][1 + t]) (section 4.2:
 *     N- = max(0, N_{i-1} - N_i), here for the instances the job uses).
 *   PARCAE_POOL_ALL:  M = max(avail[q][t], D * P), k = max(0, M - avail[q][1 + t])
 *     (section 6.3: the N- preemptions are drawn among all N_i available
 *     instances; a configuration that does not fit avail[q][t] is never a source
 *     in the plan and keeps the pool of its own instances).
 *
 * Multi-GPU instances (section 9.2): with g = group_size > 1 an instance holds g
 * GPUs that are preempted together; pipeline parallelism runs across instances
 * only, so instance G of the grid (G < D * P / g) is stage G mod P of pipelines
 * g * (G div P) .. g * (G div P) + g - 1.  n_instances and avail then count
 * instances while D * P counts GPUs: every D must be a multiple of g, a
 * candidate needs D * P / g <= N, the plan needs D * P <= g * avail, pools and k
 * above are in instances (D * P / g in place of D * P), the drawn set is a set
 * of instances, and n_int, d_min and D* = min(D, g * ((M - k) / P)) count GPU
 * pipelines (multiples of g).
 *
 * Scenario s of a unit (section 6.3, section 5.1: every instance equally
 * likely) is a k-subset of [0, M) drawn as follows.  Random word i is output
 * word (i mod 4) of Philox4x32-10 (Salmon et al., SC'11; multipliers
 * 0xD2511F53, 0xCD9E8D57; key increments 0x9E3779B9, 0xBB67AE85) with
 * key = (seed & 0xffffffff, seed >> 32) and counter = (s, i / 4, t * C + c,
 * stream_id).  With m = min(k, M - k): start from the empty set; for
 * i = 0..m-1: j = M - m + i, r = (word(i) * (j + 1)) >> 32 (64-bit product);
 * insert j if r is already in the set, else insert r.  The preempted set is
 * that set if k <= M - k, otherwise its complement in [0, M).
 *
 * Non-uniform preemption (section 5.1 lets better estimates replace the equal
 * probabilities; section 4.1 names availability zones and instance types as
 * what drives preemptions).  With n_zones > 0 instance j of the pool belongs to
 * zone[q][j] < n_zones and the k preempted instances leave one after the other,
 * each time one of the remaining instances with probability proportional to the
 * weight of its zone (successive weighted sampling without replacement).
 * Instances of one zone are interchangeable, so the set is drawn in two parts,
 * word(x, i) being word i of the sequence with counter (s, x * 65536 + i / 4,
 * t * C + c, stream_id) (the uniform draw above uses x = 0):
 *   1. left[z] = members of zone z in [0, M), gone[z] = 0; for i = 0..k-1:
 *      total = sum_z weight[z] * left[z], r = (word(0xFFFF, i) * total) >> 32,
 *      z* = first z with r < sum_{z' <= z} weight[z'] * left[z'];
 *      left[z*] -= 1, gone[z*] += 1;
 *   2. per zone z, with its members ranked in ascending instance order: the
 *      uniform draw above with M = members, k = gone[z] and word(z, i) gives the
 *      ranks of the preempted members.
 * One zone gives the uniform draw bit for bit.  Everything downstream
 * (histograms, tables, weights, plan) is unchanged.
 *
 * A weight per instance (section 5.1 again: an estimate per instance in place of equal probabilities).
 * With inst_weight, instance j of the pool has the hazard weight inst_weight[q][j] and the k preempted
 * instances leave one after the other, each time one of those still there with probability proportional
 * to its weight (successive weighted sampling without replacement): for i = 0..k-1,
 * total = sum of the weights still there, r = (word(0xFFFE, i) * total) >> 32, and the instance that goes
 * is the first one, in ascending order, at which the running sum of the weights still there exceeds r.
 * Exactly k words per scenario.  Equal weights give every k-subset the same probability.
 *
 * Per scenario (section 5.2, section 7): occ_s = alive instances of stage s;
 * d_min = min over s of occ_s (pipelines that intra-stage re-routing can
 * complete; 0 = a stage lost every replica, only a checkpoint rollback
 * helps); n_int = pipelines that lost no instance.
 *   hist_int[q][t][off[c] + n_int] and hist_min[q][t][off[c] + d_min]
 * count the S scenarios of the unit.
 *
 * Migration class of a scenario for a same-depth target of width w:
 * none if w <= n_int; else intra-stage if w <= d_min; else rollback if
 * d_min == 0; else inter-stage.  Class costs: 0, cost[.][0], cost[.][1], and
 * cost[.][2] for a rollback.  From the histograms of a unit and a width w
 * (bins above D count as empty):
 *   n0 = sum_{j >= w} hist_int[j], n01 = sum_{j >= w} hist_min[j],
 *   n1 = n01 - n0, n3 = (w >= 1 ? hist_min[0] : 0), n2 = S - n01 - n3,
 *   e_x = max(0, tau - cost[.][x]),
 *   teff(w, cost row) = (((float)n0 * tau + (float)n1 * e_0) + (float)n2 * e_1
 *                        + (float)n3 * e_2) / (float)S
 * evaluated in float exactly in this order, every product and sum rounded
 * separately (no fused multiply-add), one correctly rounded division.
 *
 * Transfer rounds (section 8.4: the state-transfer part of the migration cost
 * varies with the preemption scenario and follows an alpha-beta model).  With
 * b = cost_round[q][c'] > 0 an inter-stage migration to width w costs
 * min(cost[.][2], cost[.][1] + b * (r - 1)), r = smallest r with d_min * 2^r >= w:
 * a stage with d_min survivors brings w instances to hold its state by
 * doubling, every holder serving one more instance per round; the stages work
 * in parallel, so the worst stage decides.  teff then replaces (float)n2 * e_1 by
 *   inter = sum over r = 1, 2, .. (ascending, from 0.0f, products and sums
 *           rounded separately) of (float)n_r * max(0, tau - cost_r),
 *   n_r = sum of hist_min[j] over 1 <= j <= D with ceil(w / 2^r) <= j < ceil(w / 2^(r-1)),
 *   cost_r = min(cost[.][2], cost[.][1] + b * (float)(r - 1)) in float,
 * and teff = (((float)n0 * tau + (float)n1 * e_0) + inter + (float)n3 * e_2) / (float)S.
 * With b == 0 (or cost_round NULL) the formula above applies unchanged.
 *
 * Moved instances (section 8.4 read the other way: the transfer cost grows with the number of instances that
 * must receive state; alpha-beta model with alpha = cost[.][1], beta = cost_move).  With b = cost_move[q][c'] > 0
 * an inter-stage migration of a scenario to width w costs cost[.][1] + b * moves, moves = sum over the stages
 * of max(0, w - occ_s): the instances that must receive a stage's state so that every stage has w holders.
 * The inputs must keep the dearest such migration, cost[.][1] + b * (D_c' - 1) * P_c', within
 * min(tau, cost[.][2]) (PARCAE_EINVAL per query otherwise): it then never costs more than a re-partition or
 * than the interval lasts, no cap or clamp binds, and the expectation is linear in the move counts.
 * The evaluation keeps a third statistic for it: hist_occ[q][t][off[c] + j] = number of stages with exactly j
 * alive instances, summed over the scenarios of the unit with d_min >= 1 (bin 0 stays empty; with multi-GPU
 * instances j counts GPU pipelines, as in the other histograms).  For a width w,
 *   total_moves = sum over 1 <= j < w, j <= D of hist_occ[j] * (w - j)     (64-bit)
 * is the number of moves over all scenarios of the unit (scenarios that need no inter-stage migration have
 * no stage below w), and teff replaces (float)n2 * e_1 by
 *   inter = (float)n2 * e_1 - b * (float)total_moves   (each product rounded, then the difference; the count
 *           converted to float with round-to-nearest-even)
 * as in the formula for transfer rounds.  The planning calls then take the route that writes the transition
 * weights to the workspace, whatever the batch size.
 *
 * Liveput tables (Eq. 1, Eq. 4), all float, sums in ascending bin order,
 * acc = acc + (float)count * thr (product and sum rounded separately):
 *   liveput[q][0][t][c] = (sum_j hist_int[j] * thr[c][j]) / S   no migration
 *   liveput[q][1][t][c] = (sum_j hist_min[j] * thr[c][j]) / S   intra-stage only
 *   liveput[q][2][t][c] = thr[c][D*], D* = min(D, (M - k) / P)  all live migrations
 *     (M - k survivors of the pool: idle instances may fill in at inter-stage cost)
 *   teff[q][t][c] = teff(D*, cost[q][c]);  gain[q][t][c] = thr[c][D*] * teff[q][t][c]
 *
 * Transition weight (Eq. 4 with the rule of section 6.2), c -> c' at step t:
 *   -inf if D*P > avail[q][t] or P < p_min or D'*P' > avail[q][1+t] or
 *        P' < p_min, or if t == 0, cur_config[q] >= 0 and c != cur_config[q];
 *   cold start, cur_config[q] == PARCAE_COLD_START and t == 0 (nothing is running,
 *        e.g. training was suspended, section 7): -inf unless c == c' and c'
 *        fits avail[q][1] and p_min, then thr[c'][D'] * max(0, tau - cost[q][c'][2]);
 *   thr[c'][D'] * max(0, tau - cost[q][c'][2])           if P' != P;
 *   thr[c'][D'] * teff(D', cost[q][c']) of unit (q,t,c)  if P' == P.
 *
 * Dynamic program (Eq. 6): F[q][0][c] = 0; F[q][t+1][c'] = max over c of
 * F[q][t][c] + W_t[c][c'] in float; bp[q][t][c'] = the smallest c reaching the
 * maximum, or -1 if it is -inf.  best = smallest arg-max of F[q][T][.];
 * objective[q] = F[q][T][best]; plan[q][T-1] = best, plan[q][t-1] =
 * bp[q][t][plan[q][t]], start[q] = bp[q][0][plan[q][0]].  plan[q][t] is the
 * configuration to run in interval t.  If objective is -inf the query is
 * infeasible (section 7: training would be suspended): plan and start are -1.
 */

/* Bytes of DEVICE workspace the calls below need for this problem (HOST out). */
int parcae_workspace_bytes(const parcae_problem *p, size_t *bytes);

/* L = sum of (D_c + 1) over the HOST candidate list, or a negative code. */
int64_t parcae_hist_len(const parcae_config *configs, int32_t n_configs);

/*
 * Monte-Carlo liveput evaluation (section 6.3, Eq. 1, Eq. 4).
 *   hist_int, hist_min  DEVICE out [nq][T][L] uint32, required, overwritten
 *   liveput             DEVICE out [nq][3][T][C] float, or NULL
 *   teff, gain          DEVICE out [nq][T][C] float, or NULL
 *   status              DEVICE out [nq] int32, or NULL: PARCAE_OK, or PARCAE_EINVAL
 *                       if the query's DEVICE inputs break the rules above (its
 *                       other outputs are then computed from clamped inputs and
 *                       carry no meaning)
 *   workspace           DEVICE, 256-byte aligned, >= parcae_workspace_bytes()
 */
int parcae_liveput_eval(const parcae_problem *p, uint32_t *hist_int, uint32_t *hist_min, float *liveput,
                        float *teff, float *gain, int32_t *status, void *workspace, size_t workspace_bytes,
                        void *stream);

/*
 * Look-ahead plan from histograms computed earlier (section 6.3 notes that the
 * sampling can be done in advance; Eq. 6).
 *   hist_int, hist_min  DEVICE in  [nq][T][L]: histograms of an evaluation with the same n_scenarios (the bins of
 *                       a unit add up to it; other contents give a plan without meaning, never a fault)
 *   F                   DEVICE out [nq][T + 1][C] float, or NULL
 *   bp                  DEVICE out [nq][T][C] int32, or NULL
 *   plan                DEVICE out [nq][T] int32, required
 *   start               DEVICE out [nq] int32, or NULL
 *   objective           DEVICE out [nq] float, or NULL
 *   status              DEVICE out [nq] int32, or NULL: PARCAE_OK, PARCAE_EINVAL
 *                       (bad DEVICE inputs) or PARCAE_EINFEASIBLE
 * Limit: the per-candidate tables of a query are kept in the local memory of one
 * workgroup, which holds about 1000 candidates; a longer list is refused with
 * PARCAE_EINVAL before anything is enqueued (parcae_liveput_eval has no such limit).
 */
int parcae_plan_from_hist(const parcae_problem *p, const uint32_t *hist_int, const uint32_t *hist_min, float *F,
                          int32_t *bp, int32_t *plan, int32_t *start, float *objective, int32_t *status,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * The whole path: parcae_liveput_eval followed by parcae_plan_from_hist on the
 * same stream (algorithm 1's LiveputOpt step: current configuration and
 * availability sequence in, configuration sequence out).  Arguments as above.
 */
int parcae_liveput_plan(const parcae_problem *p, uint32_t *hist_int, uint32_t *hist_min, float *liveput,
                        float *teff, float *gain, float *F, int32_t *bp, int32_t *plan, int32_t *start,
                        float *objective, int32_t *status, void *workspace, size_t workspace_bytes,
                        void *stream);

/*
 * parcae_liveput_plan for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is an array
 * inside the library (PARCAE_STATIC_WORKSPACE_BYTES per GPU, held until the process ends); the call
 * allocates nothing on the host or the device and calls no allocating routine.  Inputs, outputs and
 * results are those of parcae_liveput_plan, bit for bit.
 * Limits: at most PARCAE_STATIC_MAX_CONFIGS candidates (PARCAE_EINVAL beyond), and
 * parcae_workspace_bytes(p) <= PARCAE_STATIC_WORKSPACE_BYTES (PARCAE_EWORKSPACE beyond; nothing is
 * enqueued then).  All calls on one GPU share that GPU's array: calls that may overlap in time on the
 * same GPU (different streams, different threads) race and must be serialised by the caller.  The
 * array keeps the last call's contents; every call clears what it needs itself.
 */
#define PARCAE_STATIC_WORKSPACE_BYTES (16u << 20)
#define PARCAE_STATIC_MAX_CONFIGS 1024
int parcae_liveput_plan_static(const parcae_problem *p, uint32_t *hist_int, uint32_t *hist_min, float *liveput,
                               float *teff, float *gain, float *F, int32_t *bp, int32_t *plan, int32_t *start,
                               float *objective, int32_t *status, void *stream);

/*
 * Transition weights written out (Eq. 4, section 6.2).
 *   W  DEVICE out [nq][T][C][C] float; row c (source), column c' (target) contiguous
 */
int parcae_transition_weights(const parcae_problem *p, const uint32_t *hist_int, const uint32_t *hist_min,
                              float *W, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Max-plus dynamic program on transition weights held in memory (Eq. 6).
 *   W  DEVICE in [nq][T][C][C] float; entries are finite or -inf (never NaN or +inf)
 *   other arguments as in parcae_plan_from_hist, except that bp may be NULL only while
 *   2 * T * C <= 16384 (the back-pointers are then kept in the workgroup's local memory;
 *   larger problems walk back through bp in memory and PARCAE_EINVAL is returned without it);
 *   status is PARCAE_OK or PARCAE_EINFEASIBLE.  Needs no workspace.  C <= 4096.
 */
int parcae_dp_plan(const float *W, int32_t n_queries, int32_t n_intervals, int32_t n_configs, float *F,
                   int32_t *bp, int32_t *plan, int32_t *start, float *objective, int32_t *status, void *stream);

/*
 * Scenarios [s0, s0 + ns) of unit (q, t, c), one by one (section 6.3).
 *   masks  DEVICE out [ns][8] uint32: bit (j mod 32) of word (j / 32) is set
 *          iff instance j of the pool is preempted
 *   n_int, d_min  DEVICE out [ns] int32
 */
int parcae_debug_sample(const parcae_problem *p, int32_t q, int32_t t, int32_t c, uint32_t s0, uint32_t ns,
                        uint32_t *masks, int32_t *n_int, int32_t *d_min, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * Receding-horizon replay of the planner along a true availability walk (algorithm 1's scheduler loop,
 * the adaptation of section 7, and the reactive baseline of section 9.4), for every query of the batch,
 * with no host synchronisation between the steps.  State of a query: the configuration running in
 * interval i, starting from cur_config[q] (a negative value: nothing is running).  Step i = 0 .. n_steps-1:
 *   1. PARCAE_REPLAY_PROACTIVE: parcae_liveput_plan on window i (availability now + forecast) with the state
 *      as current configuration (cold start if nothing runs) and Philox stream id + 2 i; target = plan[0],
 *      or the running configuration if no plan is feasible.
 *      PARCAE_REPLAY_REACTIVE: target = the candidate with the largest thr[c][D_c] that fits the actual
 *      availability a = true_avail[q][i + 1] and p_min (smallest index on ties).
 *   2. adaptation: if a equals the forecast windows[i][q][1] (always, for the reactive mode) and the target
 *      fits, it stands; otherwise the widest candidate of the target's depth that fits a; if none, the widest
 *      candidate of the deepest shallower depth (>= p_min) that fits; if none, nothing runs (-1).
 *   3. reward = transition weight (as defined above) from the state to the new configuration for the one
 *      interval that actually happened (availability true_avail[q][i] -> a, stream id + 2 i + 1), without the
 *      feasibility test; re-partition formula if nothing was running; 0 if nothing runs afterwards.
 *      total[q] accumulates the rewards in float in step order.
 *   p->avail is ignored.  The pool flag, group_size and all tables of p apply, except that a cost per moved
 *   instance (cost_move) is refused with PARCAE_EINVAL.
 *   true_avail  DEVICE in  [nq][n_steps + 1]
 *   windows     DEVICE in  [n_steps][nq][T + 1], windows[i][q][0] = true_avail[q][i]; may be NULL for
 *               PARCAE_REPLAY_REACTIVE
 *   chosen      DEVICE out [nq][n_steps] int32: configuration of interval i + 1, -1 = none
 *   reward      DEVICE out [nq][n_steps] float;  total  DEVICE out [nq] float
 *   status      DEVICE out [nq] int32, or NULL: PARCAE_OK, or PARCAE_EINVAL if the query's tables, its
 *               cur_config (which must lie in [-2, C)), an entry of its true walk or of any of its windows
 *               breaks the rules above (its outputs are then computed from clamped inputs, a cur_config
 *               past the list counting as "nothing is running", and carry no meaning)
 *   workspace   DEVICE, 256-byte aligned, >= parcae_replay_workspace_bytes() for the same mode
 * The reactive mode never plans: it needs no planner workspace and has no limit on the candidate count.
 */
#define PARCAE_REPLAY_PROACTIVE 0
#define PARCAE_REPLAY_REACTIVE 1
int parcae_replay_workspace_bytes(const parcae_problem *p, int32_t n_steps, int32_t mode, size_t *bytes);
int parcae_replay(const parcae_problem *p, int32_t n_steps, const int32_t *true_avail, const int32_t *windows,
                  int32_t mode, int32_t *chosen, float *reward, float *total, int32_t *status, void *workspace,
                  size_t workspace_bytes, void *stream);

/* Static, NUL-terminated description of a return code (HOST). */
const char *parcae_strerror(int code);

/* Library version, major * 10000 + minor * 100 + patch. */
int parcae_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PARCAE_H */
