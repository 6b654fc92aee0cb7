"""GPU parity of the task-queue simulation (Section III.B, Cases 1-4): the device-side
driver (set-up kernel, Algorithm 1 solver, apply kernel per stage) against the oracle's
plain loop, bit-exact on every record."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests.test_gpu_parity import binding  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

FIELDS = ("stage_case", "stage_count", "stage_time", "update_k", "tail", "status")


def simulate(binding, sb, max_capacity, max_batch=None):
    import torch
    with binding.DeftKnapsack(max_batch=max_batch or sb.batch, max_items=sb.n_buckets, max_knapsacks=2,
                              max_capacity=max_capacity) as h:
        out = binding.simulate_schedule(h, binding.DeviceSchedules(sb, h.device))
        torch.cuda.synchronize()
        return {k: getattr(out, k).cpu().numpy() for k in FIELDS}


def assert_same(got, ref, rows=None):
    for k in FIELDS:
        g, e = got[k], getattr(ref, k)
        if rows is not None:
            g = g[rows]
        assert g.shape == e.shape, k
        if not np.array_equal(g, e):
            bad = np.argwhere(g != e)[0]
            raise AssertionError(f"{k} differs first at {bad.tolist()}: gpu={g[tuple(bad)]} oracle={e[tuple(bad)]}")


@pytest.mark.parametrize("seed,n,w_hi,f_hi,b_hi,max_capacity", [
    (301, 9, 9, 14, 30, 1023),          # one wavefront per candidate
    (302, 70, 60, 700, 2000, 4095),     # lists longer than one 64-entry chunk
    (303, 40, 900, 5000, 12000, 13055),
])
def test_random_candidates(binding, oracle, seed, n, w_hi, f_hi, b_hi, max_capacity):
    print(f"case seed={seed} n={n}", flush=True)
    sb = W.random_schedules(seed, batch=41, n=n, iterations=12, w_hi=w_hi, t_hi=max(2, b_hi // 40), f_hi=f_hi,
                            b_hi=b_hi)
    ref = oracle.simulate_batch(sb, cap_limit=max_capacity, nthreads=16)
    assert set(np.unique(ref.stage_case[:, :, 1])) >= {2, 3, 4}       # the batch really visits every case
    assert_same(simulate(binding, sb, max_capacity), ref)


def test_status_and_reuse_of_one_handle(binding, oracle):
    """Faulted candidates get their status and zeros; a second, smaller call on the same
    handle (same buffers) is not disturbed by the first."""
    import torch
    sb = W.random_schedules(304, batch=6, n=5, iterations=4, w_hi=9, t_hi=3, f_hi=10, b_hi=10)
    sb.comm_time[1, 2] = 0
    sb.drop_time[2, 0] = -1
    sb.backward_time[3] = 11
    sb.comm_time[4] = 2 ** 30
    sb.forward_time[5] = -1
    ref = oracle.simulate_batch(sb, cap_limit=10)
    assert ref.status.tolist() == [0, 1, 1, 2, 3, 1]
    small = W.random_schedules(305, batch=3, n=4, iterations=7, w_hi=5, t_hi=2, f_hi=10, b_hi=10)
    ref_small = oracle.simulate_batch(small, cap_limit=10)
    with binding.DeftKnapsack(max_batch=6, max_items=5, max_knapsacks=2, max_capacity=10) as h:
        for batch, want in ((sb, ref), (small, ref_small), (sb, ref)):
            out = binding.simulate_schedule(h, binding.DeviceSchedules(batch, h.device))
            torch.cuda.synchronize()
            assert_same({k: getattr(out, k).cpu().numpy() for k in FIELDS}, want)


def test_rows_in_global_memory(binding, oracle):
    """Windows beyond the LDS-resident row: the same simulation on the global-row path."""
    sb = W.random_schedules(306, batch=11, n=20, iterations=6, w_hi=9000, t_hi=2000, f_hi=30000, b_hi=70000)
    ref = oracle.simulate_batch(sb, cap_limit=70000, nthreads=11)
    assert set(np.unique(ref.stage_case[:, :, 1])) >= {2, 3, 4}
    assert_same(simulate(binding, sb, 70000), ref)


def test_host_side_errors(binding):
    sb = W.random_schedules(307, batch=2, n=5, iterations=3, w_hi=9, t_hi=3, f_hi=10, b_hi=10)
    with binding.DeftKnapsack(max_batch=1, max_items=5, max_knapsacks=2, max_capacity=10) as h:      # batch above the limit
        with pytest.raises(binding.DeftError) as e:
            binding.simulate_schedule(h, binding.DeviceSchedules(sb, h.device))
        assert e.value.code == binding.DEFT_ERR_LIMIT
    with binding.DeftKnapsack(max_batch=2, max_items=5, max_knapsacks=2, max_c1=10, max_c2=10) as h:  # no sequential mode
        with pytest.raises(binding.DeftError) as e:
            binding.simulate_schedule(h, binding.DeviceSchedules(sb, h.device))
        assert e.value.code == binding.DEFT_ERR_LIMIT


def test_resnet101_shape_full_batch(binding, oracle):
    """1024 candidates x 314 buckets x 8 iterations in one call, as timed: every record of
    every candidate against the oracle (n DPs per backward stage: some tens of seconds on the
    host cores); besides, every iteration applied once or still waiting and no stage above
    its window."""
    sb = W.resnet101_schedules()
    print(f"case {sb.name} batch={sb.batch}", flush=True)
    got = simulate(binding, sb, int(max(sb.backward_time.max(), sb.forward_time.max())))
    assert (got["status"] == 0).all()
    assert (got["update_k"].sum(axis=1) + got["tail"].sum(axis=1) == sb.iterations).all()
    assert (got["stage_time"][:, :, 0] <= sb.forward_time[:, None]).all()
    assert (got["stage_time"][:, :, 1] <= sb.backward_time[:, None]).all()
    print("oracle replay of all candidates ...", flush=True)
    assert_same(got, oracle.simulate_batch(sb, nthreads=16))
