"""The claim the bit-set kernels rest on, checked on the CPU against the oracle's DP and walk:
where every value equals its weight, the selection the exact DP walks back (strict
improvement, walk from the last item) is the chain t = best sum <= C; q = first[t]; take q;
t -= w_q, with first[t] the first offered item that made the sum t reachable - for the
capacity itself (sequential mode), for every smaller capacity read off the same sweep (the
capacity sweep) and for a prefix of the list (Algorithm 1's levels).  Python integers as bit
sets; no GPU."""
import numpy as np

from paper_2503_16815_amd import workloads as W
from tests.test_oracle_pins import make_seq


def first_reached(weights, cap):
    """first[t] for every reachable t in 1..cap, and the final set."""
    goal = (1 << (cap + 1)) - 1
    bits, first = 1, {}
    for q, w in enumerate(weights):
        new = (bits | (bits << w)) & goal
        fresh = new & ~bits
        bits = new
        while fresh:
            low = fresh & -fresh
            first[low.bit_length() - 1] = q
            fresh ^= low
    return first, bits


def chain(weights, first, bits, cap, prefix=None):
    """Items on the chain from the largest reachable sum <= cap (among the first `prefix` items)."""
    if prefix is not None:
        bits = 1
        for w in weights[:prefix]:
            bits |= bits << w
    t = (bits & ((1 << (cap + 1)) - 1)).bit_length() - 1
    value, taken = t, []
    while t > 0:
        q = first[t]
        taken.append(q)
        t -= weights[q]
    return value, sorted(taken)


def test_chain_equals_the_dp_walk_at_every_capacity(oracle):
    r = np.random.default_rng(31001)
    for _ in range(60):
        n = int(r.integers(1, 40))
        w = r.integers(1, 30, size=n).tolist()
        cap_max = int(r.integers(1, 200))
        first, bits = first_reached(w, cap_max)
        for cap in sorted({cap_max, *r.integers(0, cap_max + 1, size=4).tolist()}):
            ref = oracle.solve_batch(make_seq([w], [w], [[cap]]))
            value, taken = chain(w, first, bits, cap)
            assert value == int(ref.total_value[0])
            assert taken == np.flatnonzero(ref.assignment[0] == 0).tolist()


def test_chain_of_a_prefix_is_the_dp_walk_of_that_level(oracle):
    """first[] of the whole list serves every prefix: a sum reachable with the first q items
    was first reached by one of them."""
    r = np.random.default_rng(31002)
    for _ in range(40):
        n = int(r.integers(2, 30))
        w = r.integers(1, 25, size=n).tolist()
        cap = int(r.integers(1, 150))
        first, bits = first_reached(w, cap)
        q = int(r.integers(1, n))
        ref = oracle.solve_batch(make_seq([w[:q]], [w[:q]], [[cap]]))
        value, taken = chain(w, first, bits, cap, prefix=q)
        assert value == int(ref.total_value[0])
        assert taken == np.flatnonzero(ref.assignment[0] == 0).tolist()


def test_sweep_may_end_when_the_capacity_is_reached(oracle):
    """Once the sum C is reachable the chain from C only meets sums reached before: first[] of
    the items up to there is enough."""
    r = np.random.default_rng(31003)
    hits = 0
    for _ in range(80):
        n = int(r.integers(5, 40))
        w = r.integers(1, 12, size=n).tolist()
        cap = int(r.integers(5, 60))
        bits, stop = 1, None
        for q, x in enumerate(w):
            bits |= bits << x
            if (bits >> cap) & 1:
                stop = q + 1
                break
        if stop is None or stop == n:
            continue
        hits += 1
        first, part = first_reached(w[:stop], cap)
        ref = oracle.solve_batch(make_seq([w], [w], [[cap]]))
        value, taken = chain(w, first, part, cap)
        assert value == cap == int(ref.total_value[0])
        assert taken == np.flatnonzero(ref.assignment[0] == 0).tolist()
    assert hits > 20
