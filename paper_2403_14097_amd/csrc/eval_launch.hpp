// Launch shape of the sampling kernel: how many scenarios a work item holds (host and device side).
#pragma once

#include <cstdint>

namespace parcae {

// Scenarios per work item of the sampling kernel (one wave processes an item, 64 scenarios at a time).  The kernel
// picks the length itself once the number of units that need sampling is known (a quarter to a third of all units;
// the count is in memory when the kernel starts), so that the choice fits the work that is really there.
//  * Short launches, with fewer than 16 rounds of 64 scenarios per resident wave: the items are cut so that there is
//    at most one per resident wave, all of the same number of rounds.  Every wave then starts on its own item
//    without claiming anything, and the launch lasts as long as one item.  (Measured on single queries: with the
//    fixed 1024 a query of 30 x 30 units on 64 instances left a third of the waves without work and took 16
//    rounds instead of 11; items of one round pay more for their table loads and for the adds into the shared
//    histogram rows than for their scenarios, so an item has at least two.)
//  * Longer launches take 1024 (long enough to pay for the claim and the table loads, short enough that the last
//    items do not leave the chip half empty); very long ones (1024 rounds or more per wave) take 4096, which is as
//    fast as 2048 or a little faster on every batch measured and makes a unit of up to 4096 scenarios a single item:
//    its bins are then stored once instead of added to memory by every item.  Pools of more than 128 instances cost
//    about twice as much per scenario, so their items are half as long.
__host__ __device__ inline int pick_chunk_len(int64_t n_sampled_units, int S, int n_instances, int64_t n_waves)
{
    const int64_t rounds_per_unit = ((int64_t)S + 63) / 64;
    const int64_t rounds_per_wave = (n_sampled_units * rounds_per_unit + n_waves - 1) / n_waves;
    int chunk;
    if (rounds_per_wave < 16) {
        int64_t rounds = rounds_per_wave < 2 ? 2 : rounds_per_wave;
        // the units do not divide evenly: lengthen the items until there is at most one per wave
        while (rounds < rounds_per_unit && n_sampled_units * ((rounds_per_unit + rounds - 1) / rounds) > n_waves) ++rounds;
        chunk = 64 * (int)rounds;
    } else {
        chunk = rounds_per_wave >= 1024 ? 4096 : 1024;
        if (n_instances > 128) chunk /= 2;
    }
    return S < chunk ? S : chunk;
}

// The most items a launch can have under the rule above (the host checks it against the range of the queue
// counters and sizes the grid with it): a short launch has at most one item per resident wave or, if that is more,
// one per unit, and never more than one per two rounds of a unit; the others have items of at least 512 scenarios.
inline int64_t max_eval_items(int64_t n_units, int S, int64_t n_waves)
{
    const int64_t rounds_per_unit = ((int64_t)S + 63) / 64;
    const int64_t long_items = n_units * (((int64_t)S + 511) / 512);
    int64_t short_items = n_waves > n_units ? n_waves : n_units;
    const int64_t finest = n_units * ((rounds_per_unit + 1) / 2);
    if (finest < short_items) short_items = finest;
    return long_items > short_items ? long_items : short_items;
}

// Waves per compute unit that stay resident at the kernel's register budget (7 per SIMD for the uniform draw,
// with or without the stage-occupancy statistic; 5 per SIMD for the zoned and the weighted draw).
constexpr int kEvalWavesPerCu = 28;
constexpr int kEvalWavesPerCuWide = 20;

// Persistent waves: enough workgroups (of four waves) to fill every compute unit, never more than there are items.
inline int64_t eval_grid_blocks(int cus, int64_t n_items)
{
    const int64_t fill = (int64_t)cus * 8;
    const int64_t max_useful = (n_items + 3) / 4;
    return fill < max_useful ? fill : max_useful;
}

}  // namespace parcae
