"""GPU parity of Algorithm 1 (RecursiveKnapsack, Section III.B): the HIP path, which
reads every level off one DP sweep, against the oracle, which runs the recursion with
one DP per level.  Bit-exact on every output."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests.test_gpu_parity import assert_same, binding, run  # noqa: F401  (binding is a fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cap_hi,max_capacity", [
    (700, 1023), (3000, 4095), (8000, 8191), (10000, 10239), (13000, 13055), (19900, 19967), (20000, 26111), (38900, 38911),
])
def test_random_ragged_every_lds_variant(binding, oracle, cap_hi, max_capacity):
    """Ragged n up to 150 (three 64-entry list chunks), weights up to well above the
    remaining time (items that fit no level), drop times large enough that the deep
    levels run out of time, for each compiled variant; then a tie-heavy batch (v == w,
    small weights, many equal levels)."""
    kb = W.random_recursive(5000 + cap_hi, batch=29, n_max=150, w_hi=max(20, cap_hi // 3), v_hi=1000,
                            cap_hi=cap_hi, t_hi=max(2, cap_hi // 60))
    run(binding, oracle, kb, max_capacity=max_capacity)
    kt = W.random_recursive(6000 + cap_hi, batch=17, n_max=70, w_hi=max(9, cap_hi // 40), v_hi=9,
                            cap_hi=cap_hi, t_hi=max(1, cap_hi // 200), ties=True)
    run(binding, oracle, kt, max_capacity=max_capacity)
    # value = weight, lists long and light enough to reach the remaining time itself (where the
    # sweep ends), drop times of 0 and 1 and lists with none after some point: the levels that
    # tie with the whole list, of which the deepest must be reported
    kz = W.random_recursive(6500 + cap_hi, batch=24, n_max=400, w_hi=max(9, cap_hi // 60), v_hi=9,
                            cap_hi=cap_hi, t_hi=1, ties=True)
    kz.drop_time[::3] = 0
    kz.drop_time[1::3, 40:] = 0
    run(binding, oracle, kz, max_capacity=max_capacity)


def test_levels_that_must_not_win(binding, oracle):
    """Zero drop times (every level has the full time: the deepest level that reaches the
    optimum must be reported), drop times above the remaining time (only level 0 counts),
    and a list whose last items fit nowhere."""
    base = W.random_recursive(7001, batch=24, n_max=80, w_hi=300, v_hi=50, cap_hi=3000, t_hi=0)
    run(binding, oracle, base)
    big = W.random_recursive(7002, batch=24, n_max=80, w_hi=300, v_hi=50, cap_hi=3000, t_hi=5)
    big.drop_time[:] = 4000
    run(binding, oracle, big)
    tail = W.random_recursive(7003, batch=24, n_max=80, w_hi=300, v_hi=50, cap_hi=3000, t_hi=30, ragged=False)
    tail.weights[:, 60:] = 5000
    run(binding, oracle, tail)


def test_status_and_degenerate(binding, oracle):
    kb = W.random_recursive(7101, batch=8, n_max=12, w_hi=9, v_hi=9, cap_hi=30, t_hi=3, ragged=False)
    kb.n_items[0] = 0
    kb.capacities[1, 0] = 0
    kb.drop_time[2, 5] = -1          # invalid
    kb.n_knapsacks[3] = 2            # invalid: one window only
    kb.capacities[4, 0] = 31         # above the create-time limit
    kb.values[5] = 2 ** 28           # value sum overflows
    kb.weights[6] = 100              # nothing fits any level
    ref = run(binding, oracle, kb, max_capacity=30)
    assert ref.status.tolist() == [0, 0, 1, 1, 2, 3, 0, 0]


def test_rows_in_global_memory(binding, oracle):
    """Remaining times beyond the LDS-resident row: the same mode on the global-row path (one
    launch per item, the level read off the row each launch starts from)."""
    kb = W.random_recursive(7201, batch=9, n_max=40, w_hi=9000, v_hi=500, cap_hi=70000, t_hi=900)
    run(binding, oracle, kb, max_capacity=70000)
    kt = W.random_recursive(7202, batch=140, n_max=30, w_hi=3000, v_hi=9, cap_hi=50000, t_hi=300, ties=True)
    run(binding, oracle, kt, max_capacity=50000)
    bad = W.random_recursive(7203, batch=4, n_max=6, w_hi=9, v_hi=9, cap_hi=45000, t_hi=3, ragged=False)
    bad.drop_time[1, 2] = -1
    bad.n_knapsacks[2] = 2
    bad.n_items[3] = 0
    ref = run(binding, oracle, bad, max_capacity=45000)
    assert ref.status.tolist() == [0, 1, 1, 0]


def test_host_side_errors(binding):
    """A missing drop_time array is INVALID_ARG; nothing is enqueued."""
    kb = W.random_recursive(7204, batch=4, n_max=12, w_hi=9, v_hi=9, cap_hi=30, t_hi=3)
    with binding.DeftKnapsack(max_batch=4, max_items=12, max_knapsacks=2, max_capacity=30) as h:
        db = h.upload(kb)
        db.drop_time = None
        with pytest.raises(binding.DeftError) as e:
            h.solve_batch(db)
        assert e.value.code == binding.DEFT_ERR_INVALID_ARG


def test_backward_stage_at_paper_shape(binding, oracle):
    """1024 ResNet-101-shaped backward stages (314 buckets) in one call, as timed: every
    output of every instance against the oracle's recursion (n DPs per instance, a few
    seconds on the host cores), and what holds for every answer besides: feasible for its
    own level, made of that level's items only, totals consistent."""
    import torch
    kb = W.backward_stage_shaped()
    ref = run(binding, oracle, kb)
    assert (ref.status == 0).all()
    out = binding.solve(kb)
    torch.cuda.synchronize()
    kv, kl, asg = out.knap_value.cpu().numpy(), out.knap_load.cpu().numpy(), out.assignment.cpu().numpy()
    n = kb.item_stride
    sel = asg == 0
    assert ((asg == 0) | (asg == -1)).all()
    d = kv[:, 1]
    pos = np.arange(n)[None, :]
    assert not (sel & (pos >= (n - d)[:, None])).any()
    remain = kb.capacities[:, 0].astype(np.int64) - (kb.drop_time * (pos >= (n - d)[:, None])).sum(axis=1)
    has = kv[:, 0] > 0
    assert (kl[has, 1] == remain[has]).all() and (kl[~has, 1] == 0).all()
    assert ((kb.weights * sel).sum(axis=1) == kl[:, 0]).all() and (kl[:, 0] <= np.maximum(remain, 0)).all()
    assert ((kb.values * sel).sum(axis=1) == kv[:, 0]).all()
    assert (out.total_value.cpu().numpy() == kv[:, 0]).all()
