/*
 * CPU oracle for the liveput optimizer's hot path (Parcae, arXiv 2403.14097).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the GPU library must compute.  It shares no code with the GPU library, is
 * never linked into it, and nothing in the product path may call it.  Only
 * tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What it follows:
 *   - preemption counts per interval         section 4.2 (N+ / N- rule)
 *   - uniform preemption mapping             section 5.1
 *   - Monte-Carlo preemption-mapping sampler section 6.3
 *   - which migration a scenario needs       section 5.2, section 7 (fault tolerance)
 *   - liveput as an expectation              Definition 1, Eq. 1
 *   - committed samples of one interval      Eq. 3-4 (phi, T_eff = T - T_mig)
 *   - look-ahead dynamic program             Eq. 6 and the final max after it
 *   - transition-cost rule                   section 6.2 (depth change => pipeline migration ...)
 *
 * The paper leaves the random number generator, the subset-drawing method
 * and the number of trials open.  This oracle fixes them as follows.
 *   Random words: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel random
 *   numbers: as easy as 1, 2, 3", SC'11), key = (seed low, seed high),
 *   counter = (scenario, word index / 4, interval * C + config, stream id);
 *   word i is output lane i mod 4.
 *   Subset: R. Floyd's sampling (Bentley & Floyd, CACM 1987) of the smaller
 *   of the preempted / surviving sets, bounded integers by multiply-shift.
 *   Non-uniform preemption (optional): integer hazard weights per instance
 *   (orc_sample_preempted_weighted) or per zone of instances
 *   (orc_sample_preempted_zoned), successive weighted sampling without
 *   replacement in both cases.
 *
 * Precision: every floating-point result is produced twice, in double
 * (the reference value) and in float with one fixed operation order and no
 * fused multiply-add (what decides the integer plan; compile with
 * -ffp-contract=off).  Pinned by tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_INSTANCES 256
#define ORC_MAX_GROUP 64 /* GPUs per instance: a grid of D x P GPUs has at most ORC_MAX_INSTANCES * ORC_MAX_GROUP of them */

/* ---------------------------------------------------------------- Philox */

/* One Philox4x32 block with 10 rounds (SC'11, section 3.3 and table 2 constants). */
void orc_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4])
{
    const uint32_t mul_a = 0xD2511F53u, mul_b = 0xCD9E8D57u;
    const uint32_t weyl_a = 0x9E3779B9u, weyl_b = 0xBB67AE85u;
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod_a = (uint64_t)mul_a * (uint64_t)c0;
        uint64_t prod_b = (uint64_t)mul_b * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prod_b >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod_b;
        uint32_t n2 = (uint32_t)(prod_a >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod_a;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += weyl_a;
        k1 += weyl_b;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random word i of scenario s of unit (interval t, config c); unit = t * C + c. */
uint32_t orc_word(uint64_t seed, uint32_t stream_id, uint32_t unit, uint32_t s, uint32_t i)
{
    uint32_t ctr[4] = { s, i / 4u, unit, stream_id };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[i % 4u];
}

/* Random word i of the sequence `prefix` (0 .. 0xFFFF) of a scenario: block index = prefix * 2^16 + i / 4.
 * Sequence 0 is orc_word's. */
uint32_t orc_word_at(uint64_t seed, uint32_t stream_id, uint32_t unit, uint32_t s, uint32_t prefix, uint32_t i)
{
    uint32_t ctr[4] = { s, (prefix << 16) + i / 4u, unit, stream_id };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[i % 4u];
}

/* ---------------------------------------------------------------- sampler */

/*
 * Preempted set of one scenario (section 6.3: a vector v with exactly k ones
 * among the M instances, every instance equally likely, section 5.1).
 * preempted[j] in {0,1}, j = logical instance = pipeline * P + stage.
 * Floyd's method draws the smaller of the two sets: m = min(k, M - k) words.
 */
void orc_sample_preempted(int M, int k, uint64_t seed, uint32_t stream_id, uint32_t unit,
                          uint32_t s, uint8_t *preempted)
{
    uint8_t chosen[ORC_MAX_INSTANCES];
    int m = (k < M - k) ? k : M - k;
    memset(chosen, 0, sizeof chosen);
    for (int i = 0; i < m; ++i) {
        int j = M - m + i;
        uint32_t w = orc_word(seed, stream_id, unit, s, (uint32_t)i);
        uint32_t r = (uint32_t)(((uint64_t)w * (uint64_t)(j + 1)) >> 32); /* in [0, j] */
        if (chosen[r]) chosen[j] = 1; else chosen[r] = 1;
    }
    int complement = (k > M - k);
    for (int j = 0; j < M; ++j) preempted[j] = complement ? (uint8_t)!chosen[j] : chosen[j];
}

#define ORC_MAX_ZONES 4

/*
 * Preempted set when instances are NOT equally likely to go (section 5.1 allows the uniform assumption to
 * be replaced by better estimates; section 4.1 names availability zones and instance types as what drives
 * preemptions).  Instance j of the pool belongs to zone zone[j] < n_zones, zone z has the integer hazard
 * weight weight[z] in [1, 255].  The k preempted instances leave one after the other, each time one of the
 * remaining instances with probability proportional to its weight (successive weighted sampling without
 * replacement).  Instances of one zone are interchangeable, so the same distribution is drawn in two parts:
 *   1. the zones of the k departures: draw i takes zone z with probability weight[z] * left[z] / total,
 *      left[z] = instances of zone z still there; word i of sequence 0xFFFF, r = (word * total) >> 32,
 *      zone = first z whose running sum of weight * left exceeds r;
 *   2. which gone[z] instances of zone z: a uniform subset of the zone's members (ranks 0 .. size-1 in
 *      ascending instance order) by Floyd's method on the smaller side, exactly as orc_sample_preempted
 *      does on the whole pool, with the words of sequence z.
 * With a single zone this is orc_sample_preempted bit for bit.
 */
void orc_sample_preempted_zoned(int M, int k, int n_zones, const uint8_t *zone, const uint32_t *weight,
                                uint64_t seed, uint32_t stream_id, uint32_t unit, uint32_t s, uint8_t *preempted)
{
    int members[ORC_MAX_ZONES][ORC_MAX_INSTANCES];
    int size[ORC_MAX_ZONES] = { 0, 0, 0, 0 }, left[ORC_MAX_ZONES], gone[ORC_MAX_ZONES] = { 0, 0, 0, 0 };
    for (int j = 0; j < M; ++j) {
        int z = zone[j];
        members[z][size[z]++] = j;
    }
    for (int z = 0; z < n_zones; ++z) left[z] = size[z];
    for (int i = 0; i < k; ++i) {
        uint32_t total = 0u, running = 0u;
        for (int z = 0; z < n_zones; ++z) total += weight[z] * (uint32_t)left[z];
        uint32_t w = orc_word_at(seed, stream_id, unit, s, 0xFFFFu, (uint32_t)i);
        uint32_t r = (uint32_t)(((uint64_t)w * (uint64_t)total) >> 32); /* in [0, total) */
        for (int z = 0; z < n_zones; ++z) {
            running += weight[z] * (uint32_t)left[z];
            if (r < running) {
                left[z] -= 1;
                gone[z] += 1;
                break;
            }
        }
    }
    memset(preempted, 0, (size_t)M);
    for (int z = 0; z < n_zones; ++z) {
        uint8_t chosen[ORC_MAX_INSTANCES];
        int Mz = size[z], kz = gone[z];
        int m = (kz < Mz - kz) ? kz : Mz - kz;
        memset(chosen, 0, sizeof chosen);
        for (int i = 0; i < m; ++i) {
            int j = Mz - m + i;
            uint32_t w = orc_word_at(seed, stream_id, unit, s, (uint32_t)z, (uint32_t)i);
            uint32_t r = (uint32_t)(((uint64_t)w * (uint64_t)(j + 1)) >> 32);
            if (chosen[r]) chosen[j] = 1; else chosen[r] = 1;
        }
        int complement = (kz > Mz - kz);
        for (int rank = 0; rank < Mz; ++rank)
            preempted[members[z][rank]] = complement ? (uint8_t)!chosen[rank] : chosen[rank];
    }
}

/*
 * Preempted set when every instance has its own hazard weight (section 5.1: the equal-probability assumption can be
 * replaced by more accurate estimations when the provider tells more about preemptions).  weight[j] in [1, 255] for
 * the instances j < M of the pool.  The k preempted instances leave one after the other; each time one of the
 * instances still there goes, with probability proportional to its weight (successive weighted sampling without
 * replacement).  Draw i uses word i of sequence 0xFFFE: total = sum of the weights still there,
 * r = (word * total) >> 32 in [0, total), and the instance that goes is the first one, in ascending order, at which
 * the running sum of the weights still there exceeds r.  Exactly k words; no complement trick (the survivors of
 * such a process are not distributed like its victims).
 */
void orc_sample_preempted_weighted(int M, int k, const uint8_t *weight, uint64_t seed, uint32_t stream_id,
                                   uint32_t unit, uint32_t s, uint8_t *preempted)
{
    memset(preempted, 0, (size_t)M);
    for (int i = 0; i < k; ++i) {
        uint32_t total = 0u, running = 0u;
        for (int j = 0; j < M; ++j) if (!preempted[j]) total += weight[j];
        uint32_t w = orc_word_at(seed, stream_id, unit, s, 0xFFFEu, (uint32_t)i);
        uint32_t r = (uint32_t)(((uint64_t)w * (uint64_t)total) >> 32);
        for (int j = 0; j < M; ++j) {
            if (preempted[j]) continue;
            running += weight[j];
            if (r < running) { preempted[j] = 1; break; }
        }
    }
}

/* ---------------------------------------------------------------- reducer */

/*
 * What survives a scenario on a D x P grid (section 5.2):
 *   occ[s]  = instances of stage s still alive,
 *   d_min   = min over stages of occ[s]  (pipelines that re-routing inside
 *             stages can complete; 0 means a stage is gone, section 7),
 *   n_int   = pipelines that lost no instance (run on with no migration).
 */
void orc_reduce(int D, int P, const uint8_t *preempted, int *n_int, int *d_min, int *occ)
{
    int intact = 0, least = D;
    for (int s = 0; s < P; ++s) {
        int alive = 0;
        for (int d = 0; d < D; ++d) alive += preempted[d * P + s] ? 0 : 1;
        if (occ) occ[s] = alive;
        if (alive < least) least = alive;
    }
    for (int d = 0; d < D; ++d) {
        int hit = 0;
        for (int s = 0; s < P; ++s) hit |= preempted[d * P + s];
        intact += hit ? 0 : 1;
    }
    *n_int = intact;
    *d_min = least;
}

/* Pool size and preempted count of unit (t, c).
 * Used-instance pool (a_prev < 0): the D*P used instances lose max(0, D*P - a_next) of them when
 * availability drops to a_next (section 4.2).
 * Whole-cluster pool (a_prev >= 0, section 6.3: N- preemptions among all N_i available instances, idle
 * ones included): the pool is the a_prev available instances, of which the first D*P run the grid and the
 * rest are idle, and it loses N- = max(0, a_prev - a_next).  A configuration that does not even fit
 * a_prev (never a source in the dynamic program) falls back to a pool of its own D*P instances. */
static void unit_pool(int D, int P, int group, int a_prev, int a_next, int *M, int *k)
{
    *M = D * P / (group > 1 ? group : 1); /* instances the configuration occupies */
    if (a_prev > *M) *M = a_prev;
    *k = (*M - a_next > 0) ? (*M - a_next) : 0;
}

/*
 * Multi-GPU instances (section 9.2, "Multi-GPU instances"): an instance holds `group` GPUs that are
 * preempted together, and pipeline parallelism is used across instances only, so the GPUs of one instance
 * hold the same stage of `group` neighbouring pipelines: instance G of the grid (G < D*P/group) is stage
 * G mod P of pipelines group*(G div P) .. group*(G div P) + group - 1.  Availability then counts
 * instances.  gpu[d*P + s] = 1 if the GPU at stage s of pipeline d goes.  D must be a multiple of group.
 */
void orc_expand_groups(int D, int P, int group, const uint8_t *instance_preempted, uint8_t *gpu)
{
    memset(gpu, 0, (size_t)(D * P));
    for (int G = 0; G < D * P / group; ++G) {
        if (!instance_preempted[G]) continue;
        int block = G / P, stage = G % P;
        for (int i = 0; i < group; ++i) gpu[(block * group + i) * P + stage] = 1;
    }
}

/* One scenario of a unit: which instances of the pool go (pool_pre[M]) and what is left of the D x P grid
 * (occ[P], the survivors of every stage, may be NULL).  n_zones < 0 says that `zone` holds a hazard weight per
 * instance instead of a zone index (and `weight` is unused). */
static void scenario(int D, int P, int group, int M, int k, int n_zones, const uint8_t *zone,
                     const uint32_t *weight, uint64_t seed, uint32_t stream_id, uint32_t unit,
                     uint32_t s, uint8_t *pool_pre, int *n_int, int *d_min, int *occ)
{
    if (n_zones < 0 && zone)
        orc_sample_preempted_weighted(M, k, zone, seed, stream_id, unit, s, pool_pre);
    else if (n_zones > 0 && zone && weight)
        orc_sample_preempted_zoned(M, k, n_zones, zone, weight, seed, stream_id, unit, s, pool_pre);
    else
        orc_sample_preempted(M, k, seed, stream_id, unit, s, pool_pre);
    if (group <= 1) {
        orc_reduce(D, P, pool_pre, n_int, d_min, occ);
    } else {
        uint8_t gpu[ORC_MAX_INSTANCES * ORC_MAX_GROUP];
        orc_expand_groups(D, P, group, pool_pre, gpu);
        orc_reduce(D, P, gpu, n_int, d_min, occ);
    }
}

/* Stage-occupancy statistic of one scenario into bins_occ[D + 1]: bins_occ[j] += number of stages with exactly j
 * survivors, for scenarios in which every stage still has one (d_min >= 1: the scenarios that live migration can
 * serve; a lost stage means a rollback, section 7).  From it the number of instances that must receive the state
 * of a stage to bring every stage to w holders, sum over stages of max(0, w - occ_s), follows for every w at once:
 * summed over the scenarios it is the sum over j < w of bins_occ[j] * (w - j). */
static void count_stage_occupancy(int P, int d_min, const int *occ, uint32_t *bins_occ)
{
    if (d_min < 1) return;
    for (int s = 0; s < P; ++s) bins_occ[occ[s]] += 1u;
}

/*
 * Debug view of scenarios [s0, s0 + ns) of one unit: packed masks
 * (bit j of word j/32 = instance j of the pool preempted, 8 words per scenario;
 * instances D*P and up are idle ones) and the two per-scenario integers.
 * a_prev < 0 selects the used-instance pool.  With group > 1 the mask is over instances
 * of `group` GPUs each, n_int and d_min count GPU pipelines.  n_zones > 0 with zone[] (zone of every
 * instance of the pool) and weight[] draws by orc_sample_preempted_zoned; n_zones < 0 with zone[] holding a
 * hazard weight per instance draws by orc_sample_preempted_weighted; otherwise uniformly.
 */
void orc_debug_sample(int D, int P, int group, int a_prev, int a_next, int n_zones, const uint8_t *zone,
                      const uint32_t *weight, uint64_t seed, uint32_t stream_id, uint32_t unit,
                      uint32_t s0, uint32_t ns, uint32_t *masks, int32_t *n_int, int32_t *d_min)
{
    uint8_t pre[ORC_MAX_INSTANCES];
    int M, k;
    unit_pool(D, P, group, a_prev, a_next, &M, &k);
    for (uint32_t x = 0; x < ns; ++x) {
        int ni, dm;
        scenario(D, P, group, M, k, n_zones, zone, weight, seed, stream_id, unit, s0 + x, pre, &ni, &dm, NULL);
        for (int w = 0; w < 8; ++w) masks[x * 8u + (uint32_t)w] = 0u;
        for (int j = 0; j < M; ++j)
            if (pre[j]) masks[x * 8u + (uint32_t)(j / 32)] |= (1u << (j % 32));
        n_int[x] = ni;
        d_min[x] = dm;
    }
}

/*
 * Histograms of a single unit over scenarios [s_begin, s_end): bins [D + 1] each, overwritten
 * (bins_occ, the stage-occupancy statistic, may be NULL).
 * a_prev < 0 selects the used-instance pool.
 * unit = t * C + c is the value that enters the random-word counter.
 */
void orc_eval_unit(int D, int P, int group, int a_prev, int a_next, int n_zones, const uint8_t *zone,
                   const uint32_t *weight, uint64_t seed, uint32_t stream_id, uint32_t unit,
                   uint32_t s_begin, uint32_t s_end, uint32_t *bins_int, uint32_t *bins_min, uint32_t *bins_occ)
{
    uint8_t pre[ORC_MAX_INSTANCES];
    int occ[ORC_MAX_INSTANCES];
    int M, k;
    unit_pool(D, P, group, a_prev, a_next, &M, &k);
    for (int j = 0; j <= D; ++j) { bins_int[j] = 0u; bins_min[j] = 0u; if (bins_occ) bins_occ[j] = 0u; }
    for (uint32_t s = s_begin; s < s_end; ++s) {
        int ni, dm;
        scenario(D, P, group, M, k, n_zones, zone, weight, seed, stream_id, unit, s, pre, &ni, &dm, occ);
        bins_int[ni] += 1u;
        bins_min[dm] += 1u;
        if (bins_occ) count_stage_occupancy(P, dm, occ, bins_occ);
    }
}

/*
 * Histograms of one query over scenarios [s_begin, s_end):
 *   hist_int[t][off[c] + n_int] += 1, hist_min[t][off[c] + d_min] += 1.
 * configs = (D, P) pairs; avail[0] = availability now, avail[1 + t] = a_t.
 * Buffers are [T][off[C]] and are overwritten.  n_threads > 1 splits the
 * independent units over OpenMP threads (no effect on the integers).  pool_all != 0
 * draws the preemptions among all avail[t] instances instead of the used ones.
 * n_zones > 0: zone[N] and weight[n_zones] select the non-uniform draw.
 */
void orc_eval_hist_some(int T, int C, const int32_t *configs, const int32_t *thr_off, const int32_t *avail,
                        uint64_t seed, uint32_t stream_id, uint32_t s_begin, uint32_t s_end,
                        uint32_t *hist_int, uint32_t *hist_min, int n_threads, int pool_all, int group,
                        int n_zones, const uint8_t *zone, const uint32_t *weight, const uint8_t *want,
                        uint32_t *hist_occ);

void orc_eval_hist(int T, int C, const int32_t *configs, const int32_t *thr_off, const int32_t *avail,
                   uint64_t seed, uint32_t stream_id, uint32_t s_begin, uint32_t s_end,
                   uint32_t *hist_int, uint32_t *hist_min, int n_threads, int pool_all, int group,
                   int n_zones, const uint8_t *zone, const uint32_t *weight)
{
    orc_eval_hist_some(T, C, configs, thr_off, avail, seed, stream_id, s_begin, s_end, hist_int, hist_min, n_threads,
                       pool_all, group, n_zones, zone, weight, NULL, NULL);
}

/* The same for the units (t, c) with want[t * C + c] != 0 only (all units if want is NULL); the rows of the other
 * units are left at zero.  For checks that cover the units without preemption by their known single bin.
 * hist_occ ([T][off[C]], may be NULL): the stage-occupancy statistic, hist_occ[t][off[c] + j] = stages with j
 * survivors summed over the scenarios that lost no whole stage (see count_stage_occupancy). */
void orc_eval_hist_some(int T, int C, const int32_t *configs, const int32_t *thr_off, const int32_t *avail,
                        uint64_t seed, uint32_t stream_id, uint32_t s_begin, uint32_t s_end,
                        uint32_t *hist_int, uint32_t *hist_min, int n_threads, int pool_all, int group,
                        int n_zones, const uint8_t *zone, const uint32_t *weight, const uint8_t *want,
                        uint32_t *hist_occ)
{
    const int L = thr_off[C];
    memset(hist_int, 0, sizeof(uint32_t) * (size_t)T * (size_t)L);
    memset(hist_min, 0, sizeof(uint32_t) * (size_t)T * (size_t)L);
    if (hist_occ) memset(hist_occ, 0, sizeof(uint32_t) * (size_t)T * (size_t)L);
    (void)n_threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads > 0 ? n_threads : 1)
#endif
    for (int u = 0; u < T * C; ++u) {
        if (want && !want[u]) continue;
        int t = u / C, c = u % C;
        int D = configs[2 * c], P = configs[2 * c + 1];
        int M, k;
        uint8_t pre[ORC_MAX_INSTANCES];
        int occ[ORC_MAX_INSTANCES];
        unit_pool(D, P, group, pool_all ? avail[t] : -1, avail[t + 1], &M, &k);
        uint32_t *hi = hist_int + (size_t)t * L + thr_off[c];
        uint32_t *hm = hist_min + (size_t)t * L + thr_off[c];
        uint32_t *ho = hist_occ ? hist_occ + (size_t)t * L + thr_off[c] : NULL;
        for (uint32_t s = s_begin; s < s_end; ++s) {
            int ni, dm;
            scenario(D, P, group, M, k, n_zones, zone, weight, seed, stream_id, (uint32_t)u, s, pre, &ni, &dm, occ);
            hi[ni] += 1u;
            hm[dm] += 1u;
            if (ho) count_stage_occupancy(P, dm, occ, ho);
        }
    }
}

/* ---------------------------------------------------------------- tables */

static double dmax0(double x) { return x > 0.0 ? x : 0.0; }
static float fmax0(float x) { return x > 0.0f ? x : 0.0f; }

/*
 * Scenario counts by migration class when the unit's histograms are read for a
 * same-depth target of width `width` (section 5.2, section 6.2, section 7):
 *   n[0] no migration   : width <= n_int
 *   n[1] intra-stage    : n_int < width <= d_min
 *   n[3] rollback       : width > d_min and d_min == 0 (a stage lost every replica)
 *   n[2] inter-stage    : everything else
 */
static void class_counts(const uint32_t *hi, const uint32_t *hm, int D, int width, uint32_t S, uint32_t n[4])
{
    uint32_t none = 0, upto_intra = 0;
    for (int j = width; j <= D; ++j) { none += hi[j]; upto_intra += hm[j]; }
    n[0] = none;
    n[1] = upto_intra - none;
    n[3] = (width >= 1) ? hm[0] : 0u;
    n[2] = S - upto_intra - n[3];
}

/*
 * Expected effective seconds of a unit read at a same-depth target of width `width` with the target's cost row
 * co = (intra, inter, re-partition): interval length minus the migration cost of the scenario's class, not below
 * zero, averaged over the S scenarios (Eq. 4: T_eff = T - T_mig).
 *
 * round_sec == 0: every inter-stage migration costs co[1].
 * round_sec > 0 (section 8.4: the state-transfer part of the cost varies with the preemption scenario and follows
 * an alpha-beta communication model): a stage with j survivors has to bring `width` instances to hold its state;
 * every instance that holds it passes it on to one more per round, the stages work in parallel, so the worst
 * stage (j = d_min) sets the number of rounds r = smallest r with d_min * 2^r >= width, and the migration costs
 * co[1] + round_sec * (r - 1), capped by the re-partition cost co[2] (one can always re-partition instead).
 * Float order: ((n0 * tau + n1 * e_intra) + inter) + n3 * e_repartition, inter = sum over r = 1..8 ascending of
 * (float)count_r * e_r, each product and sum rounded separately; one division by S.
 *
 * move_sec > 0 (section 8.4 again, the other reading of "varies according to the preemptions": the transfer cost
 * grows with the number of instances that must receive state; alpha-beta with alpha = co[1], beta = move_sec): an
 * inter-stage migration of a scenario to `width` costs co[1] + move_sec * moves, moves = sum over stages of
 * max(0, width - survivors of the stage).  The caller guarantees co[1] + move_sec * (width - 1) * P <= min(tau, co[2])
 * (the dearest inter-stage migration still beats a re-partition and fits the interval), so no cap and no clamp ever
 * binds and the expectation is linear in the move counts: with ho = the stage-occupancy statistic of the unit,
 * total_moves = sum over 1 <= j < width, j <= D of ho[j] * (width - j) over all its scenarios (scenarios that need no
 * inter-stage migration contribute none), inter = n2 * e_inter - move_sec * total_moves.
 * Float: inter = (float)n2 * e_inter - move_sec * (float)total_moves (64-bit count, each operation rounded).
 * At most one of round_sec and move_sec may be non-zero.
 */
static void effective_seconds(const uint32_t *hi, const uint32_t *hm, const uint32_t *ho, int D, int width, uint32_t S,
                              float tau, const float *co, float round_sec, float move_sec, double *out_d, float *out_f)
{
    uint32_t n[4];
    class_counts(hi, hm, D, width, S, n);
    double e_d[3];
    float e_f[3];
    for (int x = 0; x < 3; ++x) {
        e_d[x] = dmax0((double)tau - (double)co[x]);
        e_f[x] = fmax0(tau - co[x]);
    }
    double inter_d;
    float inter_f;
    if (move_sec != 0.0f && ho) {
        uint64_t total_moves = 0;
        for (int j = 1; j <= D && j < width; ++j) total_moves += (uint64_t)ho[j] * (uint64_t)(width - j);
        inter_d = (double)n[2] * e_d[1] - (double)move_sec * (double)total_moves;
        float fixed = (float)n[2] * e_f[1];
        float moved = move_sec * (float)total_moves;
        inter_f = fixed - moved;
    } else if (round_sec == 0.0f) {
        inter_d = (double)n[2] * e_d[1];
        inter_f = (float)n[2] * e_f[1];
    } else {
        uint32_t by_rounds[9] = { 0, 0, 0, 0, 0, 0, 0, 0, 0 };
        for (int j = 1; j <= D && j < width; ++j) { /* inter-stage scenarios: 1 <= d_min < width */
            int r = 0;
            while ((j << r) < width) ++r;
            by_rounds[r] += hm[j];
        }
        inter_d = 0.0;
        inter_f = 0.0f;
        for (int r = 1; r <= 8; ++r) {
            double cost_d = (double)co[1] + (double)round_sec * (double)(r - 1);
            if (cost_d > (double)co[2]) cost_d = (double)co[2];
            float extra = round_sec * (float)(r - 1);
            float cost_f = co[1] + extra;
            if (cost_f > co[2]) cost_f = co[2];
            inter_d += (double)by_rounds[r] * dmax0((double)tau - cost_d);
            float term = (float)by_rounds[r] * fmax0(tau - cost_f);
            inter_f = inter_f + term;
        }
    }
    *out_d = ((double)n[0] * (double)tau + (double)n[1] * e_d[0] + inter_d + (double)n[3] * e_d[2]) / (double)S;
    float q0 = (float)n[0] * tau, q1 = (float)n[1] * e_f[0], q3 = (float)n[3] * e_f[2];
    float sum = q0 + q1;
    sum = sum + inter_f;
    sum = sum + q3;
    *out_f = sum / (float)S;
}

/*
 * Liveput tables of one query (Definition 1 / Eq. 1 and Eq. 4) from histograms
 * taken over S scenarios.  Levels: 0 = no migration (only untouched pipelines
 * run), 1 = intra-stage re-routing only, 2 = all live migrations (as many
 * pipelines as the survivors can fill, floor(survivors / P), capped at D).
 * teff = expected effective seconds (interval minus the class's migration
 * cost, not below zero) when the configuration keeps its depth through the
 * boundary; gain = throughput after migration times teff.
 * cost_round: [C] seconds per further state-transfer round of an inter-stage
 * migration into each configuration, or NULL (see effective_seconds).
 * cost_move with hist_occ: [C] seconds per instance that must receive state, and
 * the stage-occupancy statistic [T][off[C]]; or both NULL.
 * Outputs: liveput [3][T][C], teff [T][C], gain [T][C], each in double (*_d)
 * and in the fixed float order (*_f).
 */
void orc_finalise(int T, int C, const int32_t *configs, const int32_t *thr_off, const int32_t *avail,
                  const float *thr, const float *cost, const float *cost_round, float tau, uint32_t S, int pool_all,
                  int group, const uint32_t *hist_int, const uint32_t *hist_min,
                  double *liveput_d, double *teff_d, double *gain_d,
                  float *liveput_f, float *teff_f, float *gain_f, const float *cost_move, const uint32_t *hist_occ)
{
    const int L = thr_off[C];
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < C; ++c) {
            int D = configs[2 * c], P = configs[2 * c + 1];
            int M, k;
            unit_pool(D, P, group, pool_all ? avail[t] : -1, avail[t + 1], &M, &k);
            const uint32_t *hi = hist_int + (size_t)t * L + thr_off[c];
            const uint32_t *hm = hist_min + (size_t)t * L + thr_off[c];
            const uint32_t *ho = hist_occ ? hist_occ + (size_t)t * L + thr_off[c] : NULL;
            const float *th = thr + thr_off[c];
            const float *co = cost + 3 * c;

            double a_d = 0.0, b_d = 0.0;
            float a_f = 0.0f, b_f = 0.0f;
            for (int j = 0; j <= D; ++j) {
                a_d += (double)hi[j] * (double)th[j];
                b_d += (double)hm[j] * (double)th[j];
                float pa = (float)hi[j] * th[j];
                float pb = (float)hm[j] * th[j];
                a_f = a_f + pa;
                b_f = b_f + pb;
            }
            int d_cap = (group > 1 ? group : 1) * ((M - k) / P); /* surviving instances fill whole blocks of pipelines */
            int d_star = D < d_cap ? D : d_cap;
            size_t o = (size_t)t * C + c, lvl = (size_t)T * C;
            liveput_d[0 * lvl + o] = a_d / (double)S;
            liveput_d[1 * lvl + o] = b_d / (double)S;
            liveput_d[2 * lvl + o] = (double)th[d_star];
            liveput_f[0 * lvl + o] = a_f / (float)S;
            liveput_f[1 * lvl + o] = b_f / (float)S;
            liveput_f[2 * lvl + o] = th[d_star];

            double td;
            float tf;
            effective_seconds(hi, hm, ho, D, d_star, S, tau, co, cost_round ? cost_round[c] : 0.0f,
                              cost_move ? cost_move[c] : 0.0f, &td, &tf);
            teff_d[o] = td;
            teff_f[o] = tf;
            gain_d[o] = (double)th[d_star] * td;
            gain_f[o] = th[d_star] * tf;
        }
    }
}

/*
 * Transition weights W[t][c][c'] = phi of Eq. 4 for leaving configuration c
 * (run during interval t-1) for c' (run during interval t):
 *   -inf              if c does not fit avail[t] or c' does not fit avail[t+1],
 *                     if either depth is below p_min, or if t == 0 and a
 *                     current configuration is given and c is not it;
 *   cold start        cur_config == -2 and t == 0: only c == c' is allowed, at
 *                     thr(c') * max(0, tau - repartition cost of c');
 *   depth changes     thr(c') * max(0, tau - repartition cost of c')   (section 6.2);
 *   same depth        thr(c') * expected effective seconds, the expectation
 *                     taken over the unit's scenarios by migration class,
 *                     costs from the target's row.
 * Both outputs are [T][C][C], row c, column c' contiguous.
 */
void orc_transition(int T, int C, const int32_t *configs, const int32_t *thr_off, const int32_t *avail,
                    const float *thr, const float *cost, const float *cost_round, float tau, uint32_t S, int p_min,
                    int cur_config, int group, const uint32_t *hist_int, const uint32_t *hist_min, double *W_d,
                    float *W_f, const float *cost_move, const uint32_t *hist_occ)
{
    const int L = thr_off[C];
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < C; ++c) {
            int D = configs[2 * c], P = configs[2 * c + 1];
            const int gpus = group > 1 ? group : 1; /* GPUs per instance: availability counts instances */
            int from_ok = (D * P <= gpus * avail[t]) && (P >= p_min) && (t > 0 || cur_config < 0 || c == cur_config);
            const uint32_t *hi = hist_int + (size_t)t * L + thr_off[c];
            const uint32_t *hm = hist_min + (size_t)t * L + thr_off[c];
            const uint32_t *ho = hist_occ ? hist_occ + (size_t)t * L + thr_off[c] : NULL;
            for (int c2 = 0; c2 < C; ++c2) {
                int D2 = configs[2 * c2], P2 = configs[2 * c2 + 1];
                int to_ok = (D2 * P2 <= gpus * avail[t + 1]) && (P2 >= p_min);
                size_t o = ((size_t)t * C + c) * C + c2;
                const float *co = cost + 3 * c2;
                float full = thr[thr_off[c2] + D2];
                if (t == 0 && cur_config == -2) {
                    /* cold start: nothing is running (training was suspended, section 7); the first
                     * configuration is brought up from the checkpoint at the re-partition cost */
                    if (c == c2 && to_ok) {
                        W_d[o] = (double)full * dmax0((double)tau - (double)co[2]);
                        W_f[o] = full * fmax0(tau - co[2]);
                    } else {
                        W_d[o] = -INFINITY;
                        W_f[o] = -INFINITY;
                    }
                    continue;
                }
                if (!from_ok || !to_ok) {
                    W_d[o] = -INFINITY;
                    W_f[o] = -INFINITY;
                    continue;
                }
                if (P2 != P) {
                    W_d[o] = (double)full * dmax0((double)tau - (double)co[2]);
                    W_f[o] = full * fmax0(tau - co[2]);
                    continue;
                }
                /* a target wider than the source (D2 > D) sums over no bins: nothing is kept or re-routed */
                double td;
                float tf;
                effective_seconds(hi, hm, ho, D, D2, S, tau, co, cost_round ? cost_round[c2] : 0.0f,
                                  cost_move ? cost_move[c2] : 0.0f, &td, &tf);
                W_d[o] = (double)full * td;
                W_f[o] = full * tf;
            }
        }
    }
}

/* ---------------------------------------------------------------- dynamic program */

/*
 * Eq. 6 in float: F[0][c] = 0; F[t+1][c'] = max over c of F[t][c] + W[t][c][c'].
 * bp[t][c'] = smallest c reaching the max, -1 when the max is -inf.
 * Then the final max over c (smallest index on ties), and the walk back:
 * plan[T-1] = best, plan[t-1] = bp[t][plan[t]], start = bp[0][plan[0]].
 * A query with no finite path gets plan = -1 everywhere, start = -1,
 * objective = -inf.  Returns 1 if a finite plan exists, else 0.
 */
int orc_dp_f32(int T, int C, const float *W, float *F, int32_t *bp, int32_t *plan, int32_t *start,
               float *objective)
{
    for (int c = 0; c < C; ++c) F[c] = 0.0f;
    for (int t = 0; t < T; ++t) {
        for (int c2 = 0; c2 < C; ++c2) {
            float best = -INFINITY;
            int arg = -1;
            for (int c = 0; c < C; ++c) {
                float v = F[(size_t)t * C + c] + W[((size_t)t * C + c) * C + c2];
                if (v > best) { best = v; arg = c; }
            }
            F[(size_t)(t + 1) * C + c2] = best;
            bp[(size_t)t * C + c2] = arg;
        }
    }
    float top = -INFINITY;
    int last = -1;
    for (int c = 0; c < C; ++c)
        if (F[(size_t)T * C + c] > top) { top = F[(size_t)T * C + c]; last = c; }
    *objective = top;
    if (last < 0) {
        for (int t = 0; t < T; ++t) plan[t] = -1;
        *start = -1;
        return 0;
    }
    plan[T - 1] = last;
    for (int t = T - 1; t >= 1; --t) plan[t - 1] = bp[(size_t)t * C + plan[t]];
    *start = bp[plan[0]];
    return 1;
}

/* The same recurrence in double, for the value of the objective only. */
double orc_dp_f64(int T, int C, const double *W)
{
    double *cur = (double *)calloc((size_t)C, sizeof(double));
    double *nxt = (double *)calloc((size_t)C, sizeof(double));
    for (int t = 0; t < T; ++t) {
        for (int c2 = 0; c2 < C; ++c2) {
            double best = -INFINITY;
            for (int c = 0; c < C; ++c) {
                double v = cur[c] + W[((size_t)t * C + c) * C + c2];
                if (v > best) best = v;
            }
            nxt[c2] = best;
        }
        double *tmp = cur; cur = nxt; nxt = tmp;
    }
    double top = -INFINITY;
    for (int c = 0; c < C; ++c) if (cur[c] > top) top = cur[c];
    free(cur);
    free(nxt);
    return top;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
