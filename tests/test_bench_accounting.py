"""bench.py's split of the oracle's cell-updates into those the solver evaluates and those
it does not (stages settled without a sweep, items after the capacity is reached), no GPU:
checked on small cases whose split can be written down by hand."""
import numpy as np

import bench
from paper_2503_16815_amd import workloads as W
from tests.test_oracle_pins import make_seq


def test_stage_where_everything_fits_is_settled(oracle):
    # window 1 (cap 10) cannot hold 6+5+4, window 2 (cap 20) holds what is left
    kb = make_seq([[6, 5, 4, 3, 2, 2, 2]], [[6, 5, 4, 3, 2, 2, 2]], [[10, 20]])
    r = oracle.solve_batch(kb)
    settled, full = bench.cells_not_swept(kb, r, True)
    left = [w for w, a in zip(kb.weights[0], r.assignment[0]) if a != 0]
    assert sum(left) <= 20
    # window 1: 6 + 4 reaches the capacity with the third item, the check after the fourth sees it
    assert settled == sum(20 - w + 1 for w in left) and full == 3 * (10 - 2 + 1)
    assert int(r.touched_cells[0]) == sum(10 - w + 1 for w in kb.weights[0]) + settled


def test_few_offered_items_count_as_settled_on_the_lds_path_only(oracle):
    kb = make_seq([[9, 8, 7]], [[9, 8, 7]], [[12]])          # three items, not all fit
    r = oracle.solve_batch(kb)
    assert bench.cells_not_swept(kb, r, True) == (int(r.touched_cells[0]), 0)
    assert bench.cells_not_swept(kb, r, False) == (0, 0)


def test_items_after_the_capacity_is_reached(oracle):
    """Twenty items of weight 1 and capacity 7 (a short list: checked after every second item):
    the sum 7 can be reached after the 7th item, the check after the 8th sees it, so items
    9..20 are never swept: 12 x (7 - 1 + 1) cells.  With a check after every item (the bit-set
    kernel) the sweep ends after the 7th."""
    kb = make_seq([[1] * 20], [[1] * 20], [[7]])
    r = oracle.solve_batch(kb)
    assert bench.cells_not_swept(kb, r, True) == (0, 12 * 7)
    assert bench.cells_not_swept(kb, r, True, check_every=1) == (0, 13 * 7)
    # weight 2, capacity 8: the odd sums are never reached, the capacity is after four items
    k2 = make_seq([[2] * 20], [[2] * 20], [[8]])
    assert bench.cells_not_swept(k2, oracle.solve_batch(k2), True) == (0, 16 * 7)
    # a list of more than 64 items is checked after every eighth
    k4 = make_seq([[2] * 70], [[2] * 70], [[8]])
    assert bench.cells_not_swept(k4, oracle.solve_batch(k4), True) == (0, 62 * 7)
    # capacity 9: the best is 8, the capacity itself is never reached
    k3 = make_seq([[2] * 20], [[2] * 20], [[9]])
    assert bench.cells_not_swept(k3, oracle.solve_batch(k3), True) == (0, 0)
    assert bench.cells_not_swept(kb, r, False) == (0, 0)      # rows in global memory: no such rule
    # values that differ from the weights: the rule does not apply
    kv = make_seq([[1] * 20], [[2] * 20], [[7]])
    assert bench.cells_not_swept(kv, oracle.solve_batch(kv), True) == (0, 0)


def test_counts_never_exceed_the_oracles(oracle):
    kb = W.resnet101_shaped(k=2, batch=6)
    r = oracle.solve_batch(kb)
    settled, full = bench.cells_not_swept(kb, r, True)
    assert 0 < settled and 0 <= full and settled + full < int(r.touched_cells.sum())
