"""GPU parity of the paper's greedy heuristic (Section III.C) against its oracle,
bit-exact on every output, on both layouts."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests.test_gpu_parity import assert_same, binding, run  # noqa: F401  (binding is a fixture)

pytestmark = pytest.mark.gpu


def test_random_ragged_and_tie_heavy(binding, oracle):
    """Ragged n (crossing the 64-entry chunks and the power-of-two padding of the sort)
    and m, then small weights with many equal times and equal capacities."""
    kb = W.random_sequential(8001, batch=61, n_max=300, m_max=8, w_hi=400, v_hi=1000, cap_hi=3000)
    run(binding, oracle, W.as_greedy(kb))
    kt = W.random_sequential(8002, batch=47, n_max=130, m_max=6, w_hi=6, v_hi=9, cap_hi=40, ties=True)
    kt.capacities[:, 1] = kt.capacities[:, 0]          # equal capacities: lower id goes first
    run(binding, oracle, W.as_greedy(kt))


def test_two_link_layout(binding, oracle):
    kj = W.random_joint(8003, 53, 70, 40, 500, 300, 300)
    run(binding, oracle, W.as_greedy(kj))
    ke = W.random_joint(8004, 21, 64, 5, 9, 40, 40)
    ke.capacities[:, 1] = ke.capacities[:, 0]
    run(binding, oracle, W.as_greedy(ke))


def test_largest_item_count(binding, oracle):
    """4096 items (the library's limit: twelve index bits in the sort key), weights up to
    2^31 - 1 among them."""
    kb = W.random_sequential(8005, batch=3, n_max=4096, m_max=3, w_hi=50, v_hi=50, cap_hi=20000, ragged=False)
    kb.weights[0, 17] = 2 ** 31 - 1
    kb.n_items[2] = 4095
    run(binding, oracle, W.as_greedy(kb))


def test_status_and_degenerate(binding, oracle):
    kb = W.as_greedy(W.random_sequential(8006, batch=8, n_max=9, m_max=3, w_hi=9, v_hi=9, cap_hi=20, ragged=False))
    kb.n_items[0] = 0
    kb.n_knapsacks[1] = 0
    kb.weights[2, 3] = 0
    kb.capacities[3, 1] = -1
    kb.capacities[4, 0] = 21
    kb.values[5] = 2 ** 29
    kb.weights[6] = 100
    ref = run(binding, oracle, kb, max_capacity=20)
    assert ref.status.tolist() == [0, 0, 1, 1, 2, 3, 0, 0]
    kj = W.as_greedy(W.random_joint(8007, 4, 6, 5, 5, 10, 10, ragged=False))
    kj.n_knapsacks[1] = 1
    kj.weights[2, 1, 0] = 0
    kj.capacities[3, 1] = 11
    refj = run(binding, oracle, kj, max_c1=10, max_c2=10)
    assert refj.status.tolist() == [0, 1, 1, 2]


def test_paper_shaped_batches_full_size(binding, oracle):
    """The four benchmark shapes at full size, every output of every instance."""
    for kb in (W.resnet101_sweep(), W.vgg19_sweep(), W.gpt2_shaped(), W.hetero_joint()):
        run(binding, oracle, W.as_greedy(kb))
