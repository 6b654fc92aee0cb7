"""Pins for the oracle of the paper's greedy heuristic (Section III.C), no GPU.
A heuristic has no optimum to compare with, so the checks are: cases worked by hand
(ties in both sorts, both layouts), closed forms, what every greedy answer must satisfy
(feasible, and no item left that an earlier-or-own knapsack could still take), independence
of the input order when nothing ties, and the exact solvers (pinned elsewhere by
enumeration) as an upper bound."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W


def greedy_seq(w, v, caps):
    w = np.atleast_2d(np.asarray(w, dtype=np.int32))
    kb = W._sequential("g", w, np.atleast_2d(np.asarray(v)), np.atleast_2d(np.asarray(caps)), None)
    return W.as_greedy(kb)


def test_worked_by_hand_one_time_per_item(oracle):
    """caps (10, 7): knapsack 1 (7) goes first.  Times 6 5 4 3 2 -> order 6 5 4 3 2.
    Knapsack 1: 6 fits (left 1), nothing else.  Knapsack 0 (10): 5 (left 5), 4 (left 1).
    Items 3 and 2 stay out.
    Second instance, ties: caps (8, 8) -> knapsack 0 first; times 4 4 4 4 -> index order;
    knapsack 0 takes items 0, 1; knapsack 1 takes items 2, 3.
    Third: values differ from times; the order still goes by time: times 5 3 3, values 1 9 9,
    cap (6,): takes the 5 (value 1), then nothing fits."""
    r = oracle.solve_batch(greedy_seq([[6, 5, 4, 3, 2]], [[6, 5, 4, 3, 2]], [[10, 7]]))
    assert r.status.tolist() == [0]
    assert r.assignment.tolist() == [[1, 0, 0, -1, -1]]
    assert r.knap_load.tolist() == [[9, 6]] and r.knap_value.tolist() == [[9, 6]] and r.total_value.tolist() == [15]
    r = oracle.solve_batch(greedy_seq([[4, 4, 4, 4]], [[4, 4, 4, 4]], [[8, 8]]))
    assert r.assignment.tolist() == [[0, 0, 1, 1]] and r.knap_load.tolist() == [[8, 8]]
    r = oracle.solve_batch(greedy_seq([[5, 3, 3]], [[1, 9, 9]], [[6]]))
    assert r.assignment.tolist() == [[0, -1, -1]]
    assert r.knap_load.tolist() == [[5]] and r.knap_value.tolist() == [[1]] and r.total_value.tolist() == [1]


def test_worked_by_hand_one_time_per_link(oracle):
    """Two links, times on link 0: 2 3 4, on link 1: 9 6 8; caps (5, 14).
    Link 0 (cap 5) first, its order 4 3 2: takes item 2 (left 1), nothing else.
    Link 1 (cap 14), its order 9 8 6 over what is left (items 0, 1): 9 fits (left 5), 6 does not.
    Equal caps (6, 6): link 0 first again: 4 (left 2), 2 (left 0); link 1: item 1 (6)."""
    kj = W.hetero_joint(batch=2, n=3, c1=5, c2=14)
    kj.weights[:] = np.array([[2, 3, 4], [9, 6, 8]])
    kj.values[:] = np.array([10, 20, 30])
    kj.capacities[1] = (6, 6)
    r = oracle.solve_batch(W.as_greedy(kj))
    assert r.status.tolist() == [0, 0]
    assert r.assignment.tolist() == [[1, -1, 0], [0, 1, 0]]
    assert r.knap_load.tolist() == [[4, 9], [6, 6]]
    assert r.knap_value.tolist() == [[30, 10], [40, 20]]


def test_closed_forms(oracle):
    # equal times, one knapsack: the first floor(C / w) items in index order
    r = oracle.solve_batch(greedy_seq([[7] * 9], [[7] * 9], [[40]]))
    assert r.assignment.tolist() == [[0] * 5 + [-1] * 4] and r.knap_load.tolist() == [[35]]
    # everything fits the smallest knapsack: it takes all, the others stay empty
    r = oracle.solve_batch(greedy_seq([[3, 9, 1, 4]], [[3, 9, 1, 4]], [[50, 17, 30]]))
    assert r.assignment.tolist() == [[1, 1, 1, 1]] and r.knap_load.tolist() == [[0, 17, 0]]
    # nothing fits anywhere
    r = oracle.solve_batch(greedy_seq([[30, 40]], [[30, 40]], [[10, 20]]))
    assert r.assignment.tolist() == [[-1, -1]] and r.total_value.tolist() == [0]


def knapsack_order(caps, m):
    return sorted(range(m), key=lambda j: (caps[j], j))


@pytest.mark.parametrize("seed,ties", [(31, False), (32, True)])
def test_every_answer_is_feasible_and_leaves_nothing_takeable(oracle, seed, ties):
    """For every item, every knapsack that had its turn before the item's own (all of them
    if the item stayed out) must be too full for it: capacities only shrink, so an item
    that fits the final remainder fitted when its turn came."""
    kb = W.random_sequential(seed, batch=60, n_max=40, m_max=5, w_hi=60, v_hi=60, cap_hi=300, ties=ties)
    r = oracle.solve_batch(W.as_greedy(kb))
    assert (r.status == 0).all()
    for b in range(kb.batch):
        n, m = int(kb.n_items[b]), int(kb.n_knapsacks[b])
        w, asg, caps = kb.weights[b, :n], r.assignment[b, :n], kb.capacities[b]
        order = knapsack_order(caps, m)
        turn = {j: s for s, j in enumerate(order)}
        for j in range(m):
            assert r.knap_load[b, j] == w[asg == j].sum() <= caps[j]
            assert r.knap_value[b, j] == kb.values[b, :n][asg == j].sum()
        for i in range(n):
            last = turn[asg[i]] if asg[i] >= 0 else m
            for s in range(last):
                j = order[s]
                assert w[i] > caps[j] - r.knap_load[b, j], (b, i, j)
        assert r.total_value[b] == r.knap_value[b, :m].sum()


def test_input_order_does_not_matter_without_ties(oracle):
    """Distinct times and distinct capacities: the sorts decide everything, so shuffling
    the items and the knapsacks must give the same placement under the relabelling."""
    rng = np.random.default_rng(77)
    for _ in range(20):
        n, m = 30, 4
        w = rng.choice(np.arange(1, 200), size=n, replace=False)
        caps = rng.choice(np.arange(50, 400), size=m, replace=False)
        r0 = oracle.solve_batch(greedy_seq([w], [w], [caps]))
        pi, pk = rng.permutation(n), rng.permutation(m)
        r1 = oracle.solve_batch(greedy_seq([w[pi]], [w[pi]], [caps[pk]]))
        back = np.full(m + 1, -1)
        back[:m] = pk                      # new id s holds old knapsack pk[s]
        assert (back[r1.assignment[0]] == r0.assignment[0][pi]).all()


def test_exact_solvers_bound_the_heuristic(oracle):
    """One knapsack: greedy <= Problem 1's optimum.  Two links: greedy <= Problem 2's optimum."""
    one = W.random_sequential(41, batch=40, n_max=30, m_max=1, w_hi=50, v_hi=50, cap_hi=200, ties=True)
    one.n_knapsacks[:] = 1
    assert (oracle.solve_batch(W.as_greedy(one)).total_value <= oracle.solve_batch(one).total_value).all()
    kj = W.random_joint(42, 30, 12, 20, 40, 60, 60)
    g, e = oracle.solve_batch(W.as_greedy(kj)), oracle.solve_batch(kj)
    ok = e.status == 0
    assert (g.status == e.status).all() and (g.total_value[ok] <= e.total_value[ok]).all()


def test_status_codes(oracle):
    kb = W.as_greedy(W.random_sequential(51, batch=5, n_max=6, m_max=2, w_hi=9, v_hi=9, cap_hi=20, ragged=False))
    kb.weights[1, 2] = 0
    kb.capacities[2, 0] = -1
    kb.capacities[3, 1] = 21
    kb.values[4] = 2 ** 29
    assert oracle.solve_batch(kb, cap_limit=20).status.tolist() == [0, 1, 1, 2, 3]
    kj = W.as_greedy(W.random_joint(52, 3, 5, 5, 5, 10, 10, ragged=False))
    kj.n_knapsacks[1] = 1
    kj.weights[2, 1, 0] = 0
    assert oracle.solve_batch(kj).status.tolist() == [0, 1, 1]
