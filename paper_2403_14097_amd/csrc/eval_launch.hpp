// Launch shape of the sampling kernel (host side): how many scenarios a work item holds.
#pragma once

#include <cstdint>

namespace parcae {

// Scenarios per work item of the sampling kernel (one wave processes an item, 64 scenarios at a time), from
// timings over batches of 1 to 1024 queries of every workload shape: 1024 suits nearly all of them (an item has
// to be long enough to pay for its claim and its table loads, short enough that the last items do not leave the
// chip half empty); very large launches gain a little from 2048, launches that cannot even give every wave two
// rounds of 64 scenarios from 512; pools of more than 128 instances cost about twice as much per scenario, so
// their items are half as long.  About a quarter of the units need sampling at all.
inline int pick_chunk_len(int64_t n_units, int S, int n_instances, int64_t n_waves)
{
    const int64_t rounds_per_wave = n_units * (int64_t)S / 64 / 4 / n_waves;
    int chunk = rounds_per_wave >= 1024 ? 2048 : (rounds_per_wave < 2 ? 512 : 1024);
    if (n_instances > 128) chunk /= 2;
    return S < chunk ? S : chunk;
}

// Waves per compute unit that the kernel keeps resident (7 per SIMD at its register budget), for the estimate above.
constexpr int kEvalWavesPerCu = 28;

// Persistent waves: enough workgroups (of four waves) to fill every compute unit, never more than there are items.
inline int64_t eval_grid_blocks(int cus, int64_t n_items)
{
    const int64_t fill = (int64_t)cus * 8;
    const int64_t max_useful = (n_items + 3) / 4;
    return fill < max_useful ? fill : max_useful;
}

}  // namespace parcae
