"""Pins for the oracle of the capacity sweep (Section IV.C feedback: the same item list
solved again with other capacities), no GPU: every capacity by enumeration of all
subsets, a case worked by hand, and monotonicity in the capacity."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests import bruteforce as bf


@pytest.mark.parametrize("seed,ties", [(91, False), (92, True)])
def test_every_capacity_matches_enumeration(oracle, seed, ties):
    kb = W.random_capacity_sweep(seed, batch=40, n_max=12, m_max=7, w_hi=9, v_hi=15, cap_hi=45, ties=ties)
    r = oracle.solve_batch(kb)
    assert (r.status == 0).all()
    for b in range(kb.batch):
        n, m = int(kb.n_items[b]), int(kb.n_knapsacks[b])
        masks = np.zeros(kb.item_stride, np.int64)
        for j in range(m):
            val, mask = bf.best_subset(kb.weights[b, :n], kb.values[b, :n], kb.capacities[b, j])
            assert r.knap_value[b, j] == val, (b, j)
            sel = np.array([(mask >> t) & 1 for t in range(n)], dtype=bool)
            assert r.knap_load[b, j] == kb.weights[b, :n][sel].sum()
            masks[:n] |= sel.astype(np.int64) << j
        assert (r.knap_value[b, m:] == 0).all() and (r.knap_load[b, m:] == 0).all()
        assert r.assignment[b].tolist() == masks.tolist(), b
        top = int(np.argmax(kb.capacities[b, :m])) if m else -1
        assert r.total_value[b] == (r.knap_value[b, top] if m else 0)


def test_worked_by_hand(oracle):
    """w = v = (5, 4, 3), capacities (7, 3, 12, 8): 7 -> {4,3}; 3 -> {3}; 12 -> all; 8 -> {5,3}.
    Item masks: item 0 (5): capacities 2, 3 -> 0b1100; item 1 (4): 0, 2 -> 0b0101; item 2 (3): all -> 0b1111."""
    kb = W.random_capacity_sweep(1, batch=1, n_max=3, m_max=4, w_hi=9, v_hi=9, cap_hi=9, ragged=False)
    kb.weights[:] = (5, 4, 3)
    kb.values[:] = (5, 4, 3)
    kb.capacities[:] = (7, 3, 12, 8)
    r = oracle.solve_batch(kb)
    assert r.status.tolist() == [0]
    assert r.knap_value.tolist() == [[7, 3, 12, 8]] and r.knap_load.tolist() == [[7, 3, 12, 8]]
    assert r.assignment.tolist() == [[0b1100, 0b0101, 0b1111]]
    assert r.total_value.tolist() == [12]


def test_value_grows_with_capacity_at_paper_shape(oracle):
    kb = W.inflation_sweep_shaped(batch=4)
    r = oracle.solve_batch(kb)
    assert (r.status == 0).all()
    assert (np.diff(r.knap_value, axis=1) >= 0).all()
    assert (r.knap_load <= kb.capacities).all()
    assert (r.total_value == r.knap_value[:, -1]).all()
    for j in range(kb.knap_stride):
        sel = (r.assignment >> j) & 1
        assert ((kb.weights * sel).sum(axis=1) == r.knap_load[:, j]).all()


def test_status_codes(oracle):
    kb = W.random_capacity_sweep(93, batch=5, n_max=6, m_max=3, w_hi=9, v_hi=9, cap_hi=20, ragged=False)
    kb.weights[1, 0] = 0
    kb.capacities[2, 2] = -1
    kb.capacities[3, 1] = 21
    kb.values[4] = 2 ** 29
    r = oracle.solve_batch(kb, cap_limit=20)
    assert r.status.tolist() == [0, 1, 1, 2, 3]
    assert (r.assignment[1:] == 0).all()
    big = W.random_capacity_sweep(94, batch=1, n_max=4, m_max=32, w_hi=9, v_hi=9, cap_hi=20, ragged=False)
    assert oracle.solve_batch(big).status.tolist() == [1]      # at most 31 capacities
