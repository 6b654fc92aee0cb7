"""Pins for the oracle of Algorithm 1 (RecursiveKnapsack, Section III.B), no GPU.
The oracle is the recursion; the checks are not: enumeration of every level and every
subset, reductions to the plain knapsack (which has pins of its own), a case worked by
hand, and the properties the recursion's answer must have."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests import bruteforce as bf


def make_rec(w, v, drop, remain):
    w = np.atleast_2d(np.asarray(w, dtype=np.int32))
    B, n = w.shape
    cap = np.zeros((B, 2), np.int32)
    cap[:, 0] = np.asarray(remain).reshape(B)
    return W.KnapsackBatch(name="t", mode=W.MODE_RECURSIVE, batch=B, item_stride=n, knap_stride=2,
                           n_items=np.full(B, n, np.int32), n_knapsacks=np.ones(B, np.int32), weights=w,
                           values=np.atleast_2d(np.asarray(v, dtype=np.int32)), capacities=cap,
                           drop_time=np.atleast_2d(np.asarray(drop, dtype=np.int32)))


def check_against_enumeration(kb, r):
    assert (r.status == 0).all()
    for b in range(kb.batch):
        n = int(kb.n_items[b])
        val, load, lvl, rem, asg = bf.recursive_prefixes(kb.weights[b, :n], kb.values[b, :n],
                                                         kb.drop_time[b, :n], kb.capacities[b, 0])
        assert r.total_value[b] == val, b
        assert r.knap_value[b].tolist() == [val, lvl], b
        assert r.knap_load[b].tolist() == [load, rem], b
        assert r.assignment[b, :n].tolist() == asg, b
        assert (r.assignment[b, n:] == -1).all()


@pytest.mark.parametrize("seed,ties", [(1, False), (2, False), (3, True), (4, True)])
def test_matches_enumeration_of_all_levels(oracle, seed, ties):
    """n <= 10: every level's knapsack by enumeration of 2^k subsets, best level by
    definition; with v == w and small weights there are many equal levels and subsets."""
    kb = W.random_recursive(seed, 48, 10, 9, 12, 40, 6, ragged=True, ties=ties)
    check_against_enumeration(kb, oracle.solve_batch(kb))


def test_worked_by_hand(oracle):
    """Three items w = v = (5, 4, 3), remaining time 7.
    drop (1,1,1): levels hold 7 over {5,4,3} -> 7; 6 over {5,4} -> 5; 5 over {5} -> 5:
      level 0 wins with {4,3}.
    drop (0,0,0) and remaining time 5: levels -> 5, 5, 5: all equal, the deepest level
      that still schedules something (2, the list {5}) is returned.
    drop (0,0,6) and remaining time 8: level 0 has 8 over {5,4,3} -> 8 = {5,3}; level 1 has
      2 -> 0; below that negative: level 0.
    weights (5,4,9), values (5,4,10), drop (0,0,1), remaining time 9: level 0 -> {9} value 10;
      level 1 has 8 over {5,4} -> 5: level 0."""
    kb = make_rec([[5, 4, 3]] * 3 + [[5, 4, 9]], [[5, 4, 3]] * 3 + [[5, 4, 10]],
                  [[1, 1, 1], [0, 0, 0], [0, 0, 6], [0, 0, 1]], [7, 5, 8, 9])
    r = oracle.solve_batch(kb)
    assert r.status.tolist() == [0, 0, 0, 0]
    assert r.assignment.tolist() == [[-1, 0, 0], [0, -1, -1], [0, -1, 0], [-1, -1, 0]]
    assert r.knap_value.tolist() == [[7, 0], [5, 2], [8, 0], [10, 0]]
    assert r.knap_load.tolist() == [[7, 7], [5, 5], [8, 8], [9, 9]]
    assert r.total_value.tolist() == [7, 5, 8, 10]


def test_reduces_to_plain_knapsack(oracle):
    """(a) Every drop time above the remaining time: only level 0 has a non-negative
    capacity, so the answer is Problem 1 on the whole list (sequential oracle, m = 1).
    (b) All drop times zero: every level has the full remaining time; a prefix can never
    beat the whole list, so the value is again Problem 1's, and the level is the largest d
    whose prefix still reaches it."""
    base = W.random_recursive(21, 40, 24, 30, 40, 200, 5, ragged=True)
    seq = W.KnapsackBatch(name="s", mode=W.MODE_SEQUENTIAL, batch=base.batch, item_stride=base.item_stride,
                          knap_stride=2, n_items=base.n_items, n_knapsacks=base.n_knapsacks,
                          weights=base.weights, values=base.values, capacities=base.capacities)
    plain = oracle.solve_batch(seq)
    # (a)
    big = make_rec(base.weights, base.values, np.full_like(base.weights, 1000), base.capacities[:, 0])
    big.n_items = base.n_items
    r = oracle.solve_batch(big)
    assert (r.status == 0).all()
    assert (r.total_value == plain.total_value).all()
    has = plain.total_value > 0
    assert (r.assignment[has] == plain.assignment[has]).all()
    assert (r.knap_value[has, 1] == 0).all() and (r.knap_value[~has, 1] == base.n_items[~has]).all()
    # (b)
    zero = make_rec(base.weights, base.values, np.zeros_like(base.weights), base.capacities[:, 0])
    zero.n_items = base.n_items
    r = oracle.solve_batch(zero)
    assert (r.total_value == plain.total_value).all()
    for b in range(base.batch):
        n, d = int(base.n_items[b]), int(r.knap_value[b, 1])
        if plain.total_value[b] == 0:
            assert d == n
            continue
        def prefix_opt(k):
            one = make_rec(base.weights[b:b + 1, :k], base.values[b:b + 1, :k], np.full((1, k), 1000),
                           base.capacities[b:b + 1, 0])
            return int(oracle.solve_batch(one).total_value[0])
        assert prefix_opt(n - d) == plain.total_value[b]
        assert d == n - 1 or prefix_opt(n - d - 1) < plain.total_value[b]
        assert (r.assignment[b, n - d:] == -1).all()


def test_properties_at_paper_shape(oracle):
    """ResNet-101-shaped backward stage (314 buckets): the answer is feasible for its own
    level, uses only that level's items, is at least as good as level 0 alone, and its
    level's remaining time follows from the drop times."""
    kb = W.backward_stage_shaped(batch=6)
    r = oracle.solve_batch(kb)
    assert (r.status == 0).all()
    lvl0 = make_rec(kb.weights, kb.values, np.full_like(kb.weights, 1 << 20), kb.capacities[:, 0])
    r0 = oracle.solve_batch(lvl0)
    for b in range(kb.batch):
        n, d = int(kb.n_items[b]), int(r.knap_value[b, 1])
        sel = r.assignment[b] == 0
        assert not sel[n - d:].any()
        rem = int(kb.capacities[b, 0]) - int(kb.drop_time[b, n - d:n].sum())
        assert r.knap_load[b, 1] == rem >= 0
        assert int(kb.weights[b][sel].sum()) == r.knap_load[b, 0] <= rem
        assert int(kb.values[b][sel].sum()) == r.knap_value[b, 0] == r.total_value[b]
        assert r.total_value[b] >= r0.total_value[b]


def test_status_codes(oracle):
    ok = make_rec([[3, 4]], [[3, 4]], [[1, 1]], [5])
    assert oracle.solve_batch(ok).status.tolist() == [0]
    for field, val in (("weights", 0), ("values", -1), ("drop_time", -1)):
        bad = make_rec([[3, 4]], [[3, 4]], [[1, 1]], [5])
        getattr(bad, field)[0, 1] = val
        assert oracle.solve_batch(bad).status.tolist() == [1]
    bad = make_rec([[3, 4]], [[3, 4]], [[1, 1]], [-1])
    assert oracle.solve_batch(bad).status.tolist() == [1]
    bad = make_rec([[3, 4]], [[3, 4]], [[1, 1]], [5]); bad.n_knapsacks[0] = 2
    assert oracle.solve_batch(bad).status.tolist() == [1]
    assert oracle.solve_batch(ok, cap_limit=4).status.tolist() == [2]
    empty = make_rec([[3, 4]], [[3, 4]], [[1, 1]], [5]); empty.n_items[0] = 0
    r = oracle.solve_batch(empty)
    assert r.status.tolist() == [0] and r.knap_value.tolist() == [[0, 0]] and (r.assignment == -1).all()
