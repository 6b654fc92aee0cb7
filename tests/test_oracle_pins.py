"""Pins for the CPU oracle (no GPU).  Each test checks the oracle against
something that is not the oracle: exhaustive enumeration, the bitset
subset-sum recurrence, closed forms, the problem's constraints, or the
paper's Table II bucket times."""
import os

import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests import bruteforce as bf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_seq(w, v, caps, order=None):
    w = np.atleast_2d(np.asarray(w))
    return W._sequential("t", w, np.atleast_2d(np.asarray(v)), np.atleast_2d(np.asarray(caps)),
                         None if order is None else np.atleast_2d(np.asarray(order)))


# ---------------------------------------------------------------- brute force
def test_tiny_bruteforce_batch_matches_enumeration(oracle):
    """Problem 1 + sequential fill: 64 instances, n=16, m=2 (the config meant
    for enumeration): value, canonical selection, loads, totals."""
    kb = W.tiny_bruteforce()
    r = oracle.solve_batch(kb)
    assert (r.status == 0).all()
    for b in range(kb.batch):
        tot, kv, kl, asg = bf.sequential_fill(kb.weights[b], kb.values[b], kb.capacities[b])
        assert r.total_value[b] == tot
        assert r.knap_value[b].tolist() == kv
        assert r.knap_load[b].tolist() == kl
        assert r.assignment[b].tolist() == asg


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_tie_heavy_value_equals_weight_canonical_mask(oracle, seed):
    """v == w with small weights: many optimal subsets; the oracle must return
    the smallest-mask one and respect a non-trivial fill order."""
    kb = W.random_sequential(seed, batch=24, n_max=14, m_max=3, w_hi=9, v_hi=9, cap_hi=40,
                             ragged=True, ties=True)
    r = oracle.solve_batch(kb)
    for b in range(kb.batch):
        n, m = int(kb.n_items[b]), int(kb.n_knapsacks[b])
        tot, kv, kl, asg = bf.sequential_fill(kb.weights[b, :n], kb.values[b, :n],
                                              kb.capacities[b, :m], kb.fill_order[b, :m])
        assert r.status[b] == 0
        assert r.total_value[b] == tot
        assert r.knap_value[b, :m].tolist() == kv
        assert r.knap_load[b, :m].tolist() == kl
        assert r.assignment[b, :n].tolist() == asg
        assert (r.assignment[b, n:] == -1).all()


def test_n20_single_knapsack_enumeration(oracle):
    kb = W.random_sequential(5, batch=3, n_max=20, m_max=1, w_hi=60, v_hi=100, cap_hi=400,
                             ragged=False, permute_order=False)
    r = oracle.solve_batch(kb)
    for b in range(kb.batch):
        val, mask = bf.best_subset(kb.weights[b], kb.values[b], kb.capacities[b, 0])
        assert r.knap_value[b, 0] == val
        got = sum(1 << t for t in range(20) if r.assignment[b, t] == 0)
        assert got == mask


@pytest.mark.parametrize("seed", [21, 22])
def test_joint_matches_3n_enumeration(oracle, seed):
    kb = W.random_joint(seed, batch=12, n_max=9, w_hi=12, v_hi=20, c1_hi=30, c2_hi=30)
    r = oracle.solve_batch(kb)
    for b in range(kb.batch):
        n = int(kb.n_items[b])
        val, asg = bf.best_two_link(kb.weights[b, 0, :n], kb.weights[b, 1, :n], kb.values[b, :n],
                                    int(kb.capacities[b, 0]), int(kb.capacities[b, 1]))
        assert r.status[b] == 0
        assert r.total_value[b] == val
        assert r.assignment[b, :n].tolist() == asg


def test_joint_ties_equal_weights_enumeration(oracle):
    """w1 == w2 == v (the paper's Problem 2 with one time per bucket): tie-heavy."""
    rng = np.random.Generator(np.random.PCG64(33))
    n, B = 10, 10
    w1 = rng.integers(1, 8, size=(B, n))
    kb = W.random_joint(33, batch=B, n_max=n, w_hi=7, v_hi=7, c1_hi=20, c2_hi=20, ragged=False)
    kb.weights = np.ascontiguousarray(np.stack([w1, w1], axis=1).astype(np.int32))
    kb.values = np.ascontiguousarray(w1.astype(np.int32))
    r = oracle.solve_batch(kb)
    for b in range(B):
        val, asg = bf.best_two_link(w1[b], w1[b], w1[b], int(kb.capacities[b, 0]), int(kb.capacities[b, 1]))
        assert r.total_value[b] == val
        assert r.total_value[b] <= kb.capacities[b].sum()
        assert r.assignment[b].tolist() == asg


# ----------------------------------------------------------- paper's own data
def _read_golden():
    d = {}
    with open(os.path.join(GOLDEN, "table2_vgg19_buckets.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            tok = line.split()
            if tok[0] == "expect":
                i = tok.index("assignment")
                d[tok[1]] = ([int(x) for x in tok[3:i]], [int(x) for x in tok[i + 1:]])
            else:
                d[tok[0]] = [int(x) for x in tok[1:]]
    return d


def test_table2_vgg19_worked_vector(oracle):
    g = _read_golden()
    c = g["comm_us"]
    # the table's printed total (257725) is 10000 above the sum of its six rows
    # (247725); the rows are used, the total is kept only to record the mismatch
    assert g["comm_total_us"][0] - sum(c) == 10000
    caps = [g["backward_total_us"][0], g["forward_total_us"][0]]
    for key, order in (("backward_then_forward", [0, 1]), ("forward_then_backward", [1, 0])):
        r = oracle.solve_batch(make_seq(c, c, caps, order))
        exp_vals, exp_asg = g[key]
        assert r.knap_value[0].tolist() == exp_vals
        assert r.assignment[0].tolist() == exp_asg
        tot, kv, kl, asg = bf.sequential_fill(c, c, caps, order)   # fixture vs enumeration
        assert kv == exp_vals and asg == exp_asg
        assert r.knap_load[0].tolist() == kl == exp_vals              # v == w: load == value


# ---------------------------------------------- subset-sum recurrence, full size
def _max_reachable(weights, cap):
    bits = 1
    for w in weights:
        bits |= bits << int(w)
    bits &= (1 << (cap + 1)) - 1
    return bits.bit_length() - 1


@pytest.mark.parametrize("maker,kw", [(W.resnet101_shaped, dict(k=2, batch=96)),
                                      (W.vgg19_shaped, dict(k=3, batch=256))])
def test_value_equals_weight_stages_match_bitset_subset_sum(oracle, maker, kw):
    """v == w: each stage's value is the largest reachable sum <= capacity of
    the items that stage was offered (textbook bitset recurrence, big ints)."""
    kb = maker(**kw)
    r = oracle.solve_batch(kb, nthreads=8)
    assert (r.status == 0).all()
    for b in range(kb.batch):
        placed_before = np.zeros(kb.item_stride, bool)
        for j in range(kb.knap_stride):        # default order 0,1,2,...
            left = kb.weights[b][~placed_before]
            assert r.knap_value[b, j] == _max_reachable(left, int(kb.capacities[b, j]))
            placed_before |= r.assignment[b] == j


# ------------------------------------------------------------------ closed forms
def test_closed_forms(oracle):
    # everything fits: all items with v > 0 are taken, value = sum v
    r = oracle.solve_batch(make_seq([3, 4, 5, 6], [7, 0, 2, 9], [18]))
    assert r.total_value[0] == 18 and r.assignment[0].tolist() == [0, -1, 0, 0]
    assert r.knap_load[0, 0] == 14
    # nothing fits
    r = oracle.solve_batch(make_seq([30, 40], [7, 8], [29, 10]))
    assert r.total_value[0] == 0 and (r.assignment[0] == -1).all() and (r.knap_load[0] == 0).all()
    # capacity 0
    r = oracle.solve_batch(make_seq([1, 1], [5, 5], [0]))
    assert r.total_value[0] == 0
    # a single item exactly at capacity is taken (constraint is inclusive)
    r = oracle.solve_batch(make_seq([10], [3], [10]))
    assert r.total_value[0] == 3 and r.assignment[0, 0] == 0
    r = oracle.solve_batch(make_seq([10], [3], [9]))
    assert r.total_value[0] == 0 and r.assignment[0, 0] == -1
    # two equal items, room for one: canonical = lower index (smaller mask)
    r = oracle.solve_batch(make_seq([5, 5], [4, 4], [5, 5]))
    assert r.assignment[0].tolist() == [0, 1] and r.knap_value[0].tolist() == [4, 4]
    # value beats weight: light valuable item preferred over heavy cheap one
    r = oracle.solve_batch(make_seq([9, 2], [3, 8], [9]))
    assert r.assignment[0].tolist() == [-1, 0] and r.total_value[0] == 8
    # fill order is honoured: knapsack 1 (big) first takes both
    r = oracle.solve_batch(make_seq([5, 5], [4, 4], [5, 10], [1, 0]))
    assert r.assignment[0].tolist() == [1, 1] and r.knap_value[0].tolist() == [0, 8]
    # empty instance / no knapsacks
    kb = make_seq([5, 5], [4, 4], [5, 10])
    kb.n_items[:] = 0
    r = oracle.solve_batch(kb)
    assert r.status[0] == 0 and r.total_value[0] == 0
    kb = make_seq([5, 5], [4, 4], [5, 10])
    kb.n_knapsacks[:] = 0
    r = oracle.solve_batch(kb)
    assert r.status[0] == 0 and r.total_value[0] == 0 and (r.assignment[0] == -1).all()


def test_joint_reductions(oracle):
    kb = W.random_joint(41, batch=16, n_max=24, w_hi=20, v_hi=50, c1_hi=80, c2_hi=80, ragged=False)
    # link 1 unusable (capacity 0, all w2 >= 1): joint == Problem 1 on link 0
    kb.capacities[:, 1] = 0
    r = oracle.solve_batch(kb)
    seq = W._sequential("s", kb.weights[:, 0], kb.values, kb.capacities[:, :1])
    rs = oracle.solve_batch(seq)
    assert (r.total_value == rs.total_value).all()
    assert (r.assignment == rs.assignment).all()
    # link 0 unusable: joint == Problem 1 on link 1, reported as knapsack 1
    kb = W.random_joint(42, batch=16, n_max=24, w_hi=20, v_hi=50, c1_hi=80, c2_hi=80, ragged=False)
    kb.capacities[:, 0] = 0
    r = oracle.solve_batch(kb)
    rs = oracle.solve_batch(W._sequential("s", kb.weights[:, 1], kb.values, kb.capacities[:, 1:]))
    assert (r.total_value == rs.total_value).all()
    assert (np.where(r.assignment == 1, 0, r.assignment) == rs.assignment).all()
    assert (r.assignment != 0).all()


def test_joint_at_least_sequential_and_bounded(oracle):
    """Joint optimum >= sequential fill of the same two knapsacks (any order);
    with w1 == w2 == v it is <= C1 + C2."""
    kb2 = W.hetero_joint(batch=24)
    kb2.weights[:, 1] = kb2.weights[:, 0]
    kb2.values[:] = kb2.weights[:, 0]
    kb2.capacities[:] = [[300, 200]]
    rj = oracle.solve_batch(kb2, nthreads=8)
    for order in ([0, 1], [1, 0]):
        seq = W._sequential("s", kb2.weights[:, 0], kb2.values, kb2.capacities,
                            np.tile(np.array([order]), (kb2.batch, 1)))
        rs = oracle.solve_batch(seq, nthreads=8)
        assert (rj.total_value >= rs.total_value).all()
    assert (rj.total_value <= 500).all()
    assert (rj.status == 0).all()


# -------------------------------------------------------------------- invariants
def check_invariants(kb, r):
    """Constraints of Problems 1 and 2 on a solved batch (any valid solution
    passes; canonical choice is pinned elsewhere)."""
    for b in range(kb.batch):
        if r.status[b] != 0:
            assert r.total_value[b] == 0 and (r.assignment[b] == -1).all()
            continue
        n, m = int(kb.n_items[b]), int(kb.n_knapsacks[b])
        asg = r.assignment[b]
        assert ((asg >= -1) & (asg < max(m, 1))).all()          # one knapsack at most
        assert (asg[n:] == -1).all()
        tot = 0
        for j in range(m):
            sel = asg[:n] == j
            wj = kb.weights[b, j, :n] if kb.mode == W.MODE_JOINT2 else kb.weights[b, :n]
            load = int(wj[sel].sum())
            val = int(kb.values[b, :n][sel].sum())
            assert load <= kb.capacities[b, j]
            assert r.knap_load[b, j] == load
            assert r.knap_value[b, j] == val
            tot += val
        assert r.total_value[b] == tot


@pytest.mark.parametrize("make", [
    lambda: W.tiny_single(), lambda: W.tiny_bruteforce(),
    lambda: W.resnet101_shaped(k=4, batch=32), lambda: W.vgg19_shaped(k=4, batch=128),
    lambda: W.gpt2_shaped(batch=8), lambda: W.hetero_joint(batch=16),
    lambda: W.random_sequential(77, 64, 40, 5, 300, 1000, 2500),
])
def test_invariants_on_paper_shaped_batches(oracle, make):
    kb = make()
    r = oracle.solve_batch(kb, nthreads=8)
    assert (r.status == 0).all()
    check_invariants(kb, r)
    if kb.mode == W.MODE_SEQUENTIAL and (kb.values == kb.weights).all():
        assert (r.knap_value == r.knap_load).all()               # v == w: value == load <= C


def test_value_monotone_in_capacity(oracle):
    kb0 = W.random_sequential(91, batch=1, n_max=30, m_max=1, w_hi=50, v_hi=200, cap_hi=10,
                              ragged=False, permute_order=False)
    caps = np.arange(0, 400)
    kb = W._sequential("mono", np.tile(kb0.weights, (len(caps), 1)), np.tile(kb0.values, (len(caps), 1)),
                       caps[:, None])
    r = oracle.solve_batch(kb, nthreads=4)
    assert (np.diff(r.total_value) >= 0).all()
    assert r.total_value[0] == 0
    # once everything fits the value stops at sum v
    assert r.total_value[-1] <= kb0.values.sum()
    big = W._sequential("all", kb0.weights, kb0.values, [[int(kb0.weights.sum())]])
    assert oracle.solve_batch(big).total_value[0] == kb0.values.sum()


def test_cell_counts_follow_their_definition(oracle):
    """touched = sum over stages and offered items of max(0, C - w + 1);
    table = offered items x (C + 1); joint = n (C1+1)(C2+1)."""
    kb = W.random_sequential(55, 20, 25, 3, 120, 50, 300)
    r = oracle.solve_batch(kb)
    for b in range(kb.batch):
        n, m = int(kb.n_items[b]), int(kb.n_knapsacks[b])
        placed = np.zeros(n, bool)
        touched = table = 0
        for s in range(m):
            j = int(kb.fill_order[b, s])
            C = int(kb.capacities[b, j])
            ws = kb.weights[b, :n][~placed]
            touched += int(np.maximum(0, C - ws + 1).sum())
            table += len(ws) * (C + 1)
            placed |= r.assignment[b, :n] == j
        assert r.touched_cells[b] == touched and r.table_cells[b] == table
    kj = W.random_joint(56, 6, 10, 9, 9, 30, 40)
    rj = oracle.solve_batch(kj)
    exp = kj.n_items.astype(np.int64) * (kj.capacities[:, 0] + 1) * (kj.capacities[:, 1] + 1)
    assert (rj.touched_cells == exp).all()


# --------------------------------------------------------------- per-instance status
def test_status_codes(oracle):
    kb = W.random_sequential(61, batch=8, n_max=6, m_max=2, w_hi=9, v_hi=9, cap_hi=20, ragged=False,
                             permute_order=False)
    kb.weights[1, 2] = 0                      # w < 1
    kb.values[2, 0] = -1                      # v < 0
    kb.capacities[3, 1] = -5                  # capacity < 0
    kb.fill_order[4] = [1, 1]                 # not a permutation
    kb.values[5, :] = 2 ** 30                 # sum v >= 2^31
    kb.capacities[6, 0] = 1000                # above the limit passed below
    kb.n_items[7] = 7                         # more items than the stride
    r = oracle.solve_batch(kb, cap_limit=100)
    assert r.status.tolist() == [0, 1, 1, 1, 1, 3, 2, 1]
    for b in range(1, 8):
        assert r.total_value[b] == 0 and (r.assignment[b] == -1).all()
        assert (r.knap_value[b] == 0).all() and (r.knap_load[b] == 0).all()
    tot, kv, kl, asg = bf.sequential_fill(kb.weights[0], kb.values[0], kb.capacities[0])
    assert r.total_value[0] == tot and r.assignment[0].tolist() == asg
    # precedence: invalid data wins over limit and overflow
    kb.weights[5, 0] = -3
    kb.weights[6, 0] = 0
    r = oracle.solve_batch(kb, cap_limit=100)
    assert r.status[5] == 1 and r.status[6] == 1
    # joint: n_knapsacks must be 2; limits per link
    kj = W.random_joint(62, 4, 5, 5, 5, 10, 10, ragged=False)
    kj.n_knapsacks[1] = 1
    kj.capacities[2, 1] = 11
    kj.weights[3, 1, 4] = 0
    rj = oracle.solve_batch(kj, c1_limit=10, c2_limit=10)
    assert rj.status.tolist() == [0, 1, 2, 1]
