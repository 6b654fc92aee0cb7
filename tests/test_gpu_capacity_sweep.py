"""GPU parity of the capacity sweep (Section IV.C feedback): the HIP path answers every
capacity from one DP sweep at the largest; the oracle solves each capacity from scratch.
Bit-exact on every output."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests.test_gpu_parity import assert_same, binding, run  # noqa: F401  (binding is a fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cap_hi,max_capacity", [
    (700, 1023), (3000, 4095), (8000, 8191), (10000, 10239), (13000, 13055), (19900, 19967), (20000, 26111), (38900, 38911),
])
def test_random_ragged_every_lds_variant(binding, oracle, cap_hi, max_capacity):
    """Ragged n and capacity counts (0 .. 31, more capacities than wavefronts per
    instance), capacities in random order from 0 up, items heavier than some or all of
    them; then a tie-heavy batch."""
    kb = W.random_capacity_sweep(9000 + cap_hi, batch=23, n_max=100, m_max=31, w_hi=max(20, cap_hi // 4),
                                 v_hi=1000, cap_hi=cap_hi)
    run(binding, oracle, kb, max_capacity=max_capacity)
    kt = W.random_capacity_sweep(9500 + cap_hi, batch=13, n_max=70, m_max=12, w_hi=max(9, cap_hi // 40), v_hi=9,
                                 cap_hi=cap_hi, ties=True)
    run(binding, oracle, kt, max_capacity=max_capacity)


def test_status_and_degenerate(binding, oracle):
    kb = W.random_capacity_sweep(9601, batch=8, n_max=9, m_max=4, w_hi=9, v_hi=9, cap_hi=20, ragged=False)
    kb.n_items[0] = 0
    kb.n_knapsacks[1] = 0
    kb.weights[2, 3] = 0
    kb.capacities[3, 2] = -1
    kb.capacities[4, 1] = 21
    kb.values[5] = 2 ** 29
    kb.weights[6] = 100
    kb.capacities[7] = 5            # the same capacity four times
    ref = run(binding, oracle, kb, max_capacity=20)
    assert ref.status.tolist() == [0, 0, 1, 1, 2, 3, 0, 0]
    big = W.random_capacity_sweep(9602, batch=2, n_max=5, m_max=32, w_hi=9, v_hi=9, cap_hi=20, ragged=False)
    big.n_knapsacks[1] = 31
    refb = run(binding, oracle, big, max_capacity=20)
    assert refb.status.tolist() == [1, 0]


def test_rows_in_global_memory(binding, oracle):
    """Capacities beyond the LDS-resident row: the same mode on the global-row path (one sweep
    at the largest capacity, one walk per capacity), small batch (tiled sweeps) and a batch
    large enough for the persistent sweep."""
    kb = W.random_capacity_sweep(9603, batch=7, n_max=40, m_max=9, w_hi=9000, v_hi=500, cap_hi=70000)
    run(binding, oracle, kb, max_capacity=70000)
    kt = W.random_capacity_sweep(9604, batch=160, n_max=30, m_max=5, w_hi=3000, v_hi=9, cap_hi=50000, ties=True)
    run(binding, oracle, kt, max_capacity=50000)
    bad = W.random_capacity_sweep(9605, batch=3, n_max=5, m_max=32, w_hi=9, v_hi=9, cap_hi=45000, ragged=False)
    bad.n_knapsacks[1] = 31
    bad.weights[2, 0] = 0
    ref = run(binding, oracle, bad, max_capacity=45000)
    assert ref.status.tolist() == [1, 0, 1]


def test_inflation_sweep_at_paper_shape(binding, oracle):
    """1024 ResNet-101-shaped instances x 11 capacities (the window and ten inflations),
    every output of every instance."""
    run(binding, oracle, W.inflation_sweep_shaped())
