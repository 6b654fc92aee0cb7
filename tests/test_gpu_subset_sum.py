"""GPU parity of the bit-set kernels (handles created with DEFT_FLAG_SUBSET_SUM: every value
equals its weight, one bit per capacity cell, the selection read off the per-cell record of
the first item that reached each sum), through the C ABI, bit-exact against the oracle's
int64 DP and walk on every output: every compiled variant, the paper's shapes at full size."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests.test_gpu_parity import assert_same, binding, run  # noqa: F401  (binding is a fixture)
from tests.test_gpu_schedule import FIELDS, assert_same as assert_same_schedule

pytestmark = pytest.mark.gpu

FLAG = 2   # DEFT_FLAG_SUBSET_SUM

VARIANTS = [(700, 1023), (4000, 4095), (10000, 10239), (14000, 14335), (20000, 20479), (26000, 26623),
            (38000, 38911), (65000, 65535)]


@pytest.mark.parametrize("cap_hi,max_capacity", VARIANTS)
def test_random_ragged_every_variant(binding, oracle, cap_hi, max_capacity):
    """Ragged n and m, random fill order, capacities from 0 up; light items, items of a few
    hundred to a few thousand cells (word shifts with every bit offset) and items heavier than
    the guard zone below the set (clamped reads).  With each layout of first[]: a handle for
    at most 255 items gets 8-bit cells, for at most 511 8-bit cells and a snapshot of the set,
    beyond that 16-bit cells."""
    for seed, n_max, w_hi in ((1, 60, max(9, cap_hi // 40)), (2, 45, max(20, cap_hi // 6)), (3, 30, cap_hi)):
        kb = W.random_sequential(21000 + 7 * cap_hi + seed, batch=37, n_max=n_max, m_max=4, w_hi=w_hi, v_hi=9,
                                 cap_hi=cap_hi, ties=True)
        run(binding, oracle, kb, max_capacity=max_capacity, flags=FLAG)          # 8-bit cells of first[]
        if seed == 1:
            run(binding, oracle, kb, max_capacity=max_capacity, max_items=300, flags=FLAG)   # 8-bit cells + snapshot
        if seed == 2:
            run(binding, oracle, kb, max_capacity=max_capacity, max_items=600, flags=FLAG)   # 16-bit cells


@pytest.mark.parametrize("max_capacity,n_max,w_hi,batch", [
    (4095, 250, 60, 40), (20479, 255, 300, 24), (38911, 255, 600, 16),     # lists short enough for 8-bit cells
    (4095, 511, 30, 40), (10239, 500, 70, 28), (14335, 511, 80, 24), (20479, 511, 140, 24),   # 8-bit cells + snapshot
    (26623, 480, 200, 16), (38911, 511, 260, 16), (65535, 500, 450, 8),
    (4095, 600, 30, 40), (10239, 1450, 30, 28), (14335, 1890, 30, 24), (26623, 3000, 39, 16), (65535, 2000, 140, 8),
])
def test_rows_that_fill_early_every_variant(binding, oracle, max_capacity, n_max, w_hi, batch):
    """Capacities in the upper half of each variant's range, light items, several windows in
    random order: the sweeps end early and the leftovers feed the next window."""
    kb = W.filling_rows(22000 + max_capacity, batch=batch, n_max=n_max, m_max=3, w_hi=w_hi,
                        cap_lo=max_capacity * 55 // 100, cap_hi=max_capacity)
    run(binding, oracle, kb, max_capacity=max_capacity, flags=FLAG)


@pytest.mark.parametrize("cap_hi,max_capacity", VARIANTS)
def test_algorithm1_every_variant(binding, oracle, cap_hi, max_capacity):
    """DEFT_MODE_RECURSIVE on the bit-set kernels: every level's value read off the set before
    the item that ends it, the walk from the best level; each layout of first[]."""
    kr = W.random_recursive(23000 + cap_hi, batch=17, n_max=150, w_hi=max(9, cap_hi // 40), v_hi=9, cap_hi=cap_hi,
                            t_hi=max(1, cap_hi // 200), ties=True)
    run(binding, oracle, kr, max_capacity=max_capacity, flags=FLAG)
    run(binding, oracle, kr, max_capacity=max_capacity, max_items=600, flags=FLAG)
    kh = W.random_recursive(23500 + cap_hi, batch=17, n_max=70, w_hi=max(20, cap_hi // 2), v_hi=9, cap_hi=cap_hi,
                            t_hi=max(2, cap_hi // 60), ties=True)          # items heavier than most levels
    run(binding, oracle, kh, max_capacity=max_capacity, max_items=300, flags=FLAG)
    kl = W.random_recursive(23700 + cap_hi, batch=9, n_max=500, w_hi=max(3, cap_hi // 150), v_hi=9, cap_hi=cap_hi,
                            t_hi=max(1, cap_hi // 800), ties=True)         # lists beyond position 255: the snapshot
    run(binding, oracle, kl, max_capacity=max_capacity, flags=FLAG)
    # drop times of 0 and 1, some lists with none at all: levels that tie with the whole list once
    # the remaining time itself is reached (where the sweep ends), the deepest of them wins
    kz = W.random_recursive(23900 + cap_hi, batch=24, n_max=200, w_hi=max(9, cap_hi // 60), v_hi=9, cap_hi=cap_hi,
                            t_hi=1, ties=True)
    kz.drop_time[::3] = 0
    kz.drop_time[1::3, 40:] = 0
    run(binding, oracle, kz, max_capacity=max_capacity, flags=FLAG)


@pytest.mark.parametrize("cap_hi,max_capacity", VARIANTS)
def test_capacity_sweep_every_variant(binding, oracle, cap_hi, max_capacity):
    """DEFT_MODE_CAPACITY_SWEEP on the bit-set kernels: one sweep at the largest capacity, the
    value at every capacity read off the final set, the walks side by side (one lane each)."""
    kc = W.random_capacity_sweep(24000 + cap_hi, batch=13, n_max=70, m_max=31, w_hi=max(9, cap_hi // 30), v_hi=9,
                                 cap_hi=cap_hi, ties=True)
    run(binding, oracle, kc, max_capacity=max_capacity, flags=FLAG)
    run(binding, oracle, kc, max_capacity=max_capacity, max_items=600, flags=FLAG)
    kl = W.random_capacity_sweep(24500 + cap_hi, batch=9, n_max=480, m_max=11, w_hi=max(3, cap_hi // 150), v_hi=9,
                                 cap_hi=cap_hi, ties=True)              # lists beyond position 255: the snapshot
    run(binding, oracle, kl, max_capacity=max_capacity, flags=FLAG)


def test_instances_that_break_the_promise_and_other_faults(binding, oracle):
    kb = W.random_sequential(25001, batch=8, n_max=12, m_max=2, w_hi=9, v_hi=9, cap_hi=30, ragged=False, ties=True)
    ref = oracle.solve_batch(kb, cap_limit=30)
    kb.values[2, 5] += 1            # breaks the promise
    kb.weights[4, 0] = 0            # invalid anyway
    kb.values[4, 0] = 0
    kb.capacities[6, 1] = 31        # above the limit
    kb.fill_order[7] = [1, 1]       # not a permutation
    bad = oracle.solve_batch(kb, cap_limit=30)
    assert bad.status.tolist() == [0, 0, 0, 0, 1, 0, 2, 1]
    import torch
    out = binding.solve(kb, max_capacity=30, flags=FLAG)
    torch.cuda.synchronize()
    assert out.status.cpu().numpy().tolist() == [0, 0, 1, 0, 1, 0, 2, 1]
    for b in range(8):
        if b == 2:
            assert int(out.total_value[b]) == 0 and (out.assignment[b].cpu().numpy() == -1).all()
            assert (out.knap_value[b].cpu().numpy() == 0).all() and (out.knap_load[b].cpu().numpy() == 0).all()
        else:
            want = bad if b in (4, 6, 7) else ref
            assert int(out.total_value[b]) == int(want.total_value[b])
            assert np.array_equal(out.assignment[b].cpu().numpy(), want.assignment[b])
            assert np.array_equal(out.knap_value[b].cpu().numpy(), want.knap_value[b])
            assert np.array_equal(out.knap_load[b].cpu().numpy(), want.knap_load[b])


def test_create_limits_and_info(binding):
    with pytest.raises(binding.DeftError) as e:
        binding.DeftKnapsack(max_batch=4, max_items=8, max_knapsacks=2, max_capacity=65536, flags=FLAG)
    assert e.value.code == binding.DEFT_ERR_LIMIT
    with binding.DeftKnapsack(max_batch=4, max_items=8, max_knapsacks=2, max_capacity=13000, flags=FLAG) as h:
        info = h.info()
        assert info.seq_path == 4 and info.seq_threads == 64 and info.seq_cells_per_thread == 7 * 32


def test_paper_shapes_at_full_size(binding, oracle):
    """The value-equals-weight sequential workloads of bench.py at their full sizes."""
    run(binding, oracle, W.resnet101_sweep(), flags=FLAG)
    run(binding, oracle, W.vgg19_sweep(), flags=FLAG)
    for k in (1, 3):
        run(binding, oracle, W.resnet101_shaped(k=k), flags=FLAG)
    run(binding, oracle, W.backward_stage_shaped(), flags=FLAG)            # Algorithm 1 on the bit-set kernels
    run(binding, oracle, W.inflation_sweep_shaped(), flags=FLAG)           # the capacity sweep on them


def test_task_queues(binding, oracle):
    """Forward stages on the sequential bit-set kernels, backward stages on Algorithm 1's."""
    import torch
    sb = W.resnet101_schedules(batch=256)
    want = oracle.simulate_batch(sb, nthreads=16)
    cap = int(max(sb.backward_time.max(), sb.forward_time.max()))
    with binding.DeftKnapsack(max_batch=sb.batch, max_items=sb.n_buckets, max_knapsacks=2, max_capacity=cap,
                              flags=FLAG) as h:
        out = binding.simulate_schedule(h, binding.DeviceSchedules(sb, h.device))
        torch.cuda.synchronize()
        assert_same_schedule({k: getattr(out, k).cpu().numpy() for k in FIELDS}, want)
