"""Second, independent statements of pieces of the method, used only to pin the C oracle.

Big-integer Python and numpy array operations; nothing here is shared with
the oracle or with the GPU library.
"""
from __future__ import annotations

import itertools

import numpy as np

M32 = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    """Philox-4x32 with 10 rounds in Python integers (SC'11 definition: two
    32x32->64 multiplies per round, the high halves are xor-ed with the other
    two counter words and the round key, the key is bumped by Weyl constants)."""
    x = [int(v) & M32 for v in ctr]
    k = [int(v) & M32 for v in key]
    for _ in range(10):
        p0 = 0xD2511F53 * x[0]
        p1 = 0xCD9E8D57 * x[2]
        x = [((p1 >> 32) ^ x[1] ^ k[0]) & M32, p1 & M32, ((p0 >> 32) ^ x[3] ^ k[1]) & M32, p0 & M32]
        k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
    return x


def word(seed, stream_id, unit, s, i):
    return philox4x32_10([s, i // 4, unit, stream_id], [seed & M32, seed >> 32])[i % 4]


def floyd_preempted(M, k, seed, stream_id, unit, s):
    """k-subset of range(M) as a 0/1 vector, drawn with Floyd's method on the smaller side."""
    m = min(k, M - k)
    chosen = set()
    for i in range(m):
        j = M - m + i
        r = (word(seed, stream_id, unit, s, i) * (j + 1)) >> 32
        chosen.add(j if r in chosen else r)
    v = np.zeros(M, dtype=np.uint8)
    v[list(chosen)] = 1
    return (1 - v) if k > M - k else v


def survivors(D, P, v):
    """(n_int, d_min) from the D x P reshaping of the preemption vector."""
    g = np.asarray(v, dtype=np.int64).reshape(D, P)
    n_int = int((g.sum(axis=1) == 0).sum())
    d_min = int((D - g.sum(axis=0)).min())
    return n_int, d_min


def migration_class(n_int, d_min, width):
    if width <= n_int:
        return "none"
    if width <= d_min:
        return "intra"
    if d_min == 0:
        return "rollback"
    return "inter"


def all_subsets(M, k):
    for comb in itertools.combinations(range(M), k):
        v = np.zeros(M, dtype=np.uint8)
        v[list(comb)] = 1
        yield comb, v


def exact_histograms(D, P, k):
    """Exact counts of n_int and d_min over all C(D*P, k) subsets (brute force)."""
    hi = np.zeros(D + 1, dtype=np.int64)
    hm = np.zeros(D + 1, dtype=np.int64)
    n = 0
    for _, v in all_subsets(D * P, k):
        a, b = survivors(D, P, v)
        hi[a] += 1
        hm[b] += 1
        n += 1
    return hi, hm, n


def brute_force_plans(W):
    """All best sequences (c_0, ..., c_T) of the max-plus path problem on W[T][C][C] by enumeration.

    Sums are formed left to right in the dtype of W.  Returns (best value, list of best sequences).
    """
    T, C = W.shape[0], W.shape[1]
    best, arg = None, []
    for seq in itertools.product(range(C), repeat=T + 1):
        tot = W.dtype.type(0)
        for t in range(T):
            tot = W.dtype.type(tot + W[t, seq[t], seq[t + 1]])
        if best is None or tot > best:
            best, arg = tot, [seq]
        elif tot == best:
            arg.append(seq)
    return best, arg


def exact_histograms_pool(D, P, pool, k):
    """Exact counts of n_int and d_min when k of `pool` instances are preempted and only the first D*P run the grid."""
    hi = np.zeros(D + 1, dtype=np.int64)
    hm = np.zeros(D + 1, dtype=np.int64)
    n = 0
    for _, v in all_subsets(pool, k):
        a, b = survivors(D, P, v[: D * P])
        hi[a] += 1
        hm[b] += 1
        n += 1
    return hi, hm, n


def successive_sampling_subset_probs(w, k):
    """Exact probability of every k-subset when k items leave one after the other, each time one of the
    remaining items with probability proportional to its weight w[j] (sum over the k! orders of departure)."""
    M, total = len(w), float(sum(w))
    probs = {}
    for sub in itertools.combinations(range(M), k):
        p = 0.0
        for order in itertools.permutations(sub):
            left, q = total, 1.0
            for j in order:
                q *= w[j] / left
                left -= w[j]
            p += q
        probs[sub] = p
    return probs


def zone_count_distribution(sizes, weights, k):
    """Exact distribution of how many of the k departures fall into each zone (urn process, by dynamic programming
    over the numbers already gone per zone).  Returns {counts tuple: probability}."""
    Z = len(sizes)
    dist = {tuple([0] * Z): 1.0}
    for _ in range(k):
        nxt = {}
        for gone, p in dist.items():
            left = [sizes[z] - gone[z] for z in range(Z)]
            total = float(sum(weights[z] * left[z] for z in range(Z)))
            for z in range(Z):
                if left[z] > 0:
                    g = list(gone)
                    g[z] += 1
                    g = tuple(g)
                    nxt[g] = nxt.get(g, 0.0) + p * weights[z] * left[z] / total
        dist = nxt
    return dist


def word_at(seed, stream_id, unit, s, prefix, i):
    """Word i of sequence `prefix` of a scenario: block index prefix * 2^16 + i // 4 in counter word 1."""
    return philox4x32_10([s, ((prefix << 16) + i // 4) & M32, unit, stream_id], [seed & M32, seed >> 32])[i % 4]


def weighted_preempted(M, k, weight, seed, stream_id, unit, s):
    """k instances leave one after the other, each time one of those still there with probability proportional to
    its weight: word i of sequence 0xFFFE scaled to the remaining total weight picks a point, the instance whose
    stretch of the remaining weights (in ascending instance order) covers the point goes."""
    there = list(range(M))
    gone = np.zeros(M, dtype=np.uint8)
    for i in range(k):
        total = sum(int(weight[j]) for j in there)
        point = (word_at(seed, stream_id, unit, s, 0xFFFE, i) * total) >> 32
        for pos, j in enumerate(there):
            point -= int(weight[j])
            if point < 0:
                gone[j] = 1
                del there[pos]
                break
    return gone


def zoned_preempted(M, k, zone, zone_weight, seed, stream_id, unit, s):
    """Zones of unequal hazard: first the zone of each of the k departures (urn process, sequence 0xFFFF), then per
    zone a uniform subset of its members by Floyd's method on their ranks (sequence = zone index)."""
    Z = len(zone_weight)
    members = [[j for j in range(M) if zone[j] == z] for z in range(Z)]
    left = [len(m) for m in members]
    for i in range(k):
        total = sum(int(zone_weight[z]) * left[z] for z in range(Z))
        point = (word_at(seed, stream_id, unit, s, 0xFFFF, i) * total) >> 32
        for z in range(Z):
            point -= int(zone_weight[z]) * left[z]
            if point < 0:
                left[z] -= 1
                break
    gone = np.zeros(M, dtype=np.uint8)
    for z in range(Z):
        size, kz = len(members[z]), len(members[z]) - left[z]
        m = min(kz, size - kz)
        chosen = set()
        for i in range(m):
            j = size - m + i
            r = (word_at(seed, stream_id, unit, s, z, i) * (j + 1)) >> 32
            chosen.add(j if r in chosen else r)
        for rank, inst in enumerate(members[z]):
            hit = rank in chosen
            gone[inst] = (not hit) if kz > size - kz else hit
    return gone


def stage_occupancy(D, P, v):
    """Survivors of every stage of the D x P grid, given the preemption vector of the grid."""
    return D - np.asarray(v, dtype=np.int64).reshape(D, P).sum(axis=0)


def moves_to_width(occ, width):
    """Instances that must receive the state of a stage so that every stage has `width` holders."""
    return int(np.maximum(0, width - np.asarray(occ)).sum())
