"""Exhaustive enumeration used to pin the CPU oracle (tiny inputs only).

Nothing here is a DP: every selection is listed, its weight and value summed,
the feasible ones with the best value kept, and the canonical one picked by
its definition (smallest selection number).  Written with numpy only, shares
nothing with oracle/ or the HIP path.
"""
import numpy as np


def best_subset(w, v, cap):
    """Problem 1 by enumeration of all 2^n subsets.

    Returns (optimal value, canonical mask) where the canonical mask is the
    smallest integer sum_t x_t 2^t among optimal feasible subsets."""
    w = np.asarray(w, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    n = len(w)
    assert n <= 22
    masks = np.arange(1 << n, dtype=np.int64)
    wsum = np.zeros(1 << n, dtype=np.int64)
    vsum = np.zeros(1 << n, dtype=np.int64)
    for t in range(n):
        bit = (masks >> t) & 1
        wsum += bit * w[t]
        vsum += bit * v[t]
    feasible = wsum <= cap
    best = int(vsum[feasible].max())
    mask = int(masks[feasible & (vsum == best)].min())
    return best, mask


def sequential_fill(w, v, caps, order=None):
    """m knapsacks filled one after the other, each by enumeration on what the
    earlier ones left.  Returns (total, knap_value, knap_load, assignment)."""
    n, m = len(w), len(caps)
    order = list(range(m)) if order is None else list(order)
    assign = [-1] * n
    kv, kl = [0] * m, [0] * m
    for j in order:
        left = [i for i in range(n) if assign[i] == -1]
        val, mask = best_subset([w[i] for i in left], [v[i] for i in left], caps[j])
        for t, i in enumerate(left):
            if (mask >> t) & 1:
                assign[i] = j
                kl[j] += int(w[i])
        kv[j] = val
    return sum(kv), kv, kl, assign


def best_two_link(w1, w2, v, c1, c2):
    """Problem 2 (per-link weights) by enumeration of all 3^n placements
    a_i in {0: nowhere, 1: link 0, 2: link 1}.  Canonical = smallest
    sum_i a_i 3^i among optimal feasible placements.
    Returns (optimal value, assignment list with -1 / 0 / 1)."""
    n = len(v)
    assert n <= 13
    total = 3 ** n
    idx = np.arange(total, dtype=np.int64)
    l1 = np.zeros(total, dtype=np.int64)
    l2 = np.zeros(total, dtype=np.int64)
    val = np.zeros(total, dtype=np.int64)
    rest = idx.copy()
    for i in range(n):
        a = rest % 3
        rest //= 3
        l1 += (a == 1) * int(w1[i])
        l2 += (a == 2) * int(w2[i])
        val += (a != 0) * int(v[i])
    feasible = (l1 <= c1) & (l2 <= c2)
    best = int(val[feasible].max())
    num = int(idx[feasible & (val == best)].min())
    assign = []
    for i in range(n):
        assign.append(num % 3 - 1)
        num //= 3
    return best, assign


def recursive_prefixes(w, v, drop, remain):
    """Algorithm 1 by its meaning rather than its recursion: level d (d = 0 .. n) keeps
    the first n - d items and has remain - sum of drop over the d items left out; each
    level is solved by enumeration; the answer is the best level, and among equal levels
    the one with the most items left out (the recursion only prefers the shallower
    answer when it is strictly better).  Nothing scheduled anywhere -> level n.
    Returns (value, load, level, level's remaining time, assignment 0 / -1)."""
    n = len(w)
    best = (0, 0, n, 0, [-1] * n)
    rem = int(remain) - int(sum(drop))
    for d in range(n, -1, -1):           # deepest first; shallower must be strictly better
        if d < n:
            rem += int(drop[n - 1 - d])  # level d leaves out items n-d .. n-1 only
        k = n - d
        if k == 0 or rem < 0:
            continue
        val, mask = best_subset(w[:k], v[:k], rem)
        if val > best[0]:
            asg = [0 if (mask >> t) & 1 else -1 for t in range(k)] + [-1] * d
            load = sum(int(w[t]) for t in range(k) if (mask >> t) & 1)
            best = (val, load, d, rem, asg)
    return best
