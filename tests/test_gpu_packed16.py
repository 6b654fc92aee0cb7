"""GPU parity of the kernels with rows of 16-bit cells (handles created with
DEFT_FLAG_VALUES_ARE_WEIGHTS: every value equals its weight, capacities up to 26623),
through the C ABI, bit-exact against the oracle on every output: every compiled variant,
every mode that runs on them, the paper's shapes at full size."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests.test_gpu_parity import assert_same, binding, run  # noqa: F401  (binding is a fixture)
from tests.test_gpu_schedule import FIELDS, assert_same as assert_same_schedule

pytestmark = pytest.mark.gpu

FLAG = 1   # DEFT_FLAG_VALUES_ARE_WEIGHTS

VARIANTS = [
    (700, 1023),       # one wavefront per instance
    (3000, 4095),      # 256 x 16
    (8000, 8191),      # 256 x 32
    (9500, 9599),      # 320 x 30 (five wavefronts)
    (10000, 10239),    # 512 x 20
    (13000, 13311),    # 512 x 26
    (19900, 19967),    # 768 x 26
    (26000, 26623),    # 1024 x 26
]


@pytest.mark.parametrize("cap_hi,max_capacity", VARIANTS)
def test_random_ragged_every_variant(binding, oracle, cap_hi, max_capacity):
    """Ragged n and m, random fill order, capacities from 0 up: light items (below one lane
    row), items around the lane count (lanes on both sides of the shift) and items of several
    lane rows (the per-lane word offsets of the heavy path), odd and even pair counts."""
    for seed, n_max, w_hi in ((1, 60, max(9, cap_hi // 40)), (2, 45, max(20, cap_hi // 6)), (3, 30, cap_hi)):
        kb = W.random_sequential(11000 + 7 * cap_hi + seed, batch=37, n_max=n_max, m_max=4, w_hi=w_hi, v_hi=9,
                                 cap_hi=cap_hi, ties=True)
        run(binding, oracle, kb, max_capacity=max_capacity, flags=FLAG)


@pytest.mark.parametrize("max_capacity,n_max,w_hi,batch", [
    (1023, 160, 30, 64), (4095, 600, 30, 40), (8191, 1160, 30, 32), (9599, 1360, 30, 28), (10239, 1450, 30, 28), (13311, 1890, 30, 24),
    (19967, 2830, 30, 20), (26623, 3000, 39, 16),
])
def test_rows_that_fill_early_every_variant(binding, oracle, max_capacity, n_max, w_hi, batch):
    """Capacities in the upper half of each variant's range, light items, several windows in
    random order: the sweeps end early; the swept-cell count must match the replay."""
    import torch
    import bench
    kb = W.filling_rows(12000 + max_capacity, batch=batch, n_max=n_max, m_max=3, w_hi=w_hi,
                        cap_lo=max_capacity * 55 // 100, cap_hi=max_capacity)
    print(f"case {kb.name} batch={kb.batch} n<={n_max} max_capacity={max_capacity}", flush=True)
    ref = oracle.solve_batch(kb, nthreads=16, cap_limit=max_capacity)
    settled, full = bench.cells_not_swept(kb, ref, True)
    assert full > 0.2 * int(ref.touched_cells.sum())
    with binding.DeftKnapsack(max_batch=kb.batch, max_items=kb.item_stride, max_knapsacks=kb.knap_stride,
                              max_capacity=max_capacity, flags=FLAG) as h:
        assert h.info().seq_path in (1, 2)
        db = h.upload(kb)
        h.set_profiling(True)
        out = h.solve_batch(db)
        torch.cuda.synchronize()
        prof = h.get_profile()
        assert_same(kb, out, ref)
    assert int(prof.swept_cell_updates) == int(ref.touched_cells.sum()) - settled - full, kb.name


@pytest.mark.parametrize("cap_hi,max_capacity", VARIANTS)
def test_algorithm1_and_capacity_sweep_every_variant(binding, oracle, cap_hi, max_capacity):
    kr = W.random_recursive(13000 + cap_hi, batch=17, n_max=150, w_hi=max(9, cap_hi // 40), v_hi=9, cap_hi=cap_hi,
                            t_hi=max(1, cap_hi // 200), ties=True)
    run(binding, oracle, kr, max_capacity=max_capacity, flags=FLAG)
    kh = W.random_recursive(13500 + cap_hi, batch=17, n_max=70, w_hi=max(20, cap_hi // 2), v_hi=9, cap_hi=cap_hi,
                            t_hi=max(2, cap_hi // 60), ties=True)          # items heavier than most levels
    run(binding, oracle, kh, max_capacity=max_capacity, flags=FLAG)
    # sweeps that end at the reached remaining time; drop times of 0 and 1: tying levels
    kz = W.random_recursive(13700 + cap_hi, batch=24, n_max=400, w_hi=max(9, cap_hi // 60), v_hi=9,
                            cap_hi=cap_hi, t_hi=1, ties=True)
    kz.drop_time[::3] = 0
    kz.drop_time[1::3, 40:] = 0
    run(binding, oracle, kz, max_capacity=max_capacity, flags=FLAG)
    kc = W.random_capacity_sweep(14000 + cap_hi, batch=13, n_max=70, m_max=31, w_hi=max(9, cap_hi // 30), v_hi=9,
                                 cap_hi=cap_hi, ties=True)
    run(binding, oracle, kc, max_capacity=max_capacity, flags=FLAG)


def test_instances_that_break_the_promise_and_other_faults(binding, oracle):
    """A value that differs from its weight is INVALID_ARG on these handles (zeros, -1), like
    any other bad input; its neighbours are solved."""
    kb = W.random_sequential(15001, batch=8, n_max=12, m_max=2, w_hi=9, v_hi=9, cap_hi=30, ragged=False, ties=True)
    ref = oracle.solve_batch(kb, cap_limit=30)
    kb.values[2, 5] += 1            # breaks the promise
    kb.weights[4, 0] = 0            # invalid anyway
    kb.values[4, 0] = 0
    kb.capacities[6, 1] = 31        # above the limit
    bad = oracle.solve_batch(kb, cap_limit=30)
    assert bad.status.tolist() == [0, 0, 0, 0, 1, 0, 2, 0]
    import torch
    out = binding.solve(kb, max_capacity=30, flags=FLAG)
    torch.cuda.synchronize()
    status = out.status.cpu().numpy()
    assert status.tolist() == [0, 0, 1, 0, 1, 0, 2, 0]
    for b in range(8):
        if b == 2:
            assert int(out.total_value[b]) == 0 and (out.assignment[b].cpu().numpy() == -1).all()
            assert (out.knap_value[b].cpu().numpy() == 0).all() and (out.knap_load[b].cpu().numpy() == 0).all()
        else:
            want = bad if b in (4, 6) else ref
            assert int(out.total_value[b]) == int(want.total_value[b])
            assert np.array_equal(out.assignment[b].cpu().numpy(), want.assignment[b])
            assert np.array_equal(out.knap_value[b].cpu().numpy(), want.knap_value[b])
            assert np.array_equal(out.knap_load[b].cpu().numpy(), want.knap_load[b])


def test_create_limits(binding):
    with pytest.raises(binding.DeftError) as e:
        binding.DeftKnapsack(max_batch=4, max_items=8, max_knapsacks=2, max_capacity=26624, flags=FLAG)
    assert e.value.code == binding.DEFT_ERR_LIMIT
    with binding.DeftKnapsack(max_batch=4, max_items=8, max_knapsacks=2, max_capacity=26623, flags=FLAG) as h:
        assert h.info().seq_threads == 1024


def test_paper_shapes_at_full_size(binding, oracle):
    """The value-equals-weight workloads of bench.py at their full sizes and launch shapes."""
    run(binding, oracle, W.resnet101_sweep(), flags=FLAG)
    run(binding, oracle, W.vgg19_sweep(), flags=FLAG)
    for k in (1, 3):
        run(binding, oracle, W.resnet101_shaped(k=k), flags=FLAG)
    run(binding, oracle, W.backward_stage_shaped(), flags=FLAG)
    run(binding, oracle, W.inflation_sweep_shaped(), flags=FLAG)


def test_task_queues(binding, oracle):
    import torch
    sb = W.random_schedules(16001, batch=41, n=40, iterations=12, w_hi=900, t_hi=300, f_hi=5000, b_hi=12000)
    ref = oracle.simulate_batch(sb, cap_limit=13055, nthreads=16)
    big = W.resnet101_schedules(batch=256)
    ref_big = oracle.simulate_batch(big, nthreads=16)
    for s, want, cap in ((sb, ref, 13055), (big, ref_big, int(max(big.backward_time.max(), big.forward_time.max())))):
        print(f"case {s.name} batch={s.batch}", flush=True)
        with binding.DeftKnapsack(max_batch=s.batch, max_items=s.n_buckets, max_knapsacks=2, max_capacity=cap,
                                  flags=FLAG) as h:
            out = binding.simulate_schedule(h, binding.DeviceSchedules(s, h.device))
            torch.cuda.synchronize()
            assert_same_schedule({k: getattr(out, k).cpu().numpy() for k in FIELDS}, want)
