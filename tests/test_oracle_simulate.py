"""Pins for the oracle of the task-queue simulation (Section III.B, Cases 1-4), no GPU.
The paper gives the cases in prose and a figure that is not part of its text, so no
printed numbers exist to compare with; the checks are the sequence of cases and updates
that the paper narrates for that figure (tests/golden/fig4_walkthrough.txt), sequences
worked by hand from the cases, closed forms, conservation of iterations, and a replay of every stage with the
enumeration solvers of tests/bruteforce.py (which checks the lists, capacities and index
maps the oracle hands to its own solvers, not the reading of the cases)."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests import bruteforce as bf


def one(comm, drop, fwd, bwd, iterations):
    n = len(comm)
    return W.ScheduleBatch(name="t", batch=1, n_buckets=n, iterations=iterations,
                           comm_time=np.array([comm], np.int32), drop_time=np.array([drop], np.int32),
                           forward_time=np.array([fwd], np.int32), backward_time=np.array([bwd], np.int32))


def test_sequence_worked_by_hand(oracle):
    """Buckets (4, 3, 2), no drop times, forward window 0, backward window 6.
    it 0: queue empty -> Case 4: Algorithm 1 over (4,3,2) with 6 -> {4,2}; bucket 3 waits (k=1).
    it 1: 3 fits 6 -> Case 3: it goes first (time 3, its iteration is complete); Algorithm 1 with the
          other 3: the whole list and the list without its last bucket both reach 3, the shorter
          list wins -> {3}; (4,2) wait.  Update k=1.
    it 2: (4,2) fit exactly -> Case 3: both go, nothing left for the new buckets, all three wait.  Update k=1.
    it 3: 9 > 6 -> Case 2: knapsack -> {4,2}; the new buckets wait in the future queue.  No update.
    it 4: 3 fits -> Case 3: it goes (complete, k=1); future queue holds two iterations; Algorithm 1
          with 3 -> {3}; (4,2) wait with k=2.  Update k=1.
    it 5: (4,2) go (complete, k=2); nothing left; the new buckets wait.  Update k=2."""
    r = oracle.simulate_batch(one([4, 3, 2], [0, 0, 0], 0, 6, 6))
    assert r.status.tolist() == [0]
    assert r.stage_case[0, :, 1].tolist() == [4, 3, 3, 2, 3, 3]
    assert r.stage_case[0, :, 0].tolist() == [0, 1, 1, 1, 1, 1]
    assert r.stage_count[0, :, 1].tolist() == [2, 2, 2, 2, 2, 2] and (r.stage_count[0, :, 0] == 0).all()
    assert r.stage_time[0, :, 1].tolist() == [6, 6, 6, 6, 6, 6]
    assert r.update_k[0].tolist() == [0, 1, 1, 0, 1, 2]
    assert r.tail[0].tolist() == [1, 0]


def _fig4_fixture():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "fig4_walkthrough.txt")
    data, told = {}, {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            if key == "narrated":
                told[rest[0]] = [None if x == "-" else int(x) for x in rest[1:]]
            else:
                data[key] = [int(x) for x in rest]
    return data, told


def test_walk_through_of_fig4(oracle):
    """The paper's own walk through its Fig. 4 (Section III.B, after Case 4), on an
    eight-bucket instance: every case, leftover count and update the text states must come
    out of the oracle's reading of the two queues.  The first two iterations worked by hand
    (times 1 8 6 4 8 4 5 4, drop times 1 1 3 0 2 0 0 0, windows 10 / 21):
    it 1 backward: queue empty -> Case 4.  Remaining time per list length 8..4: 21 21 21 21 19.
      Lengths 8..5 all reach 21 and length 4 reaches 19, so the shortest list that reaches 21
      wins: 1+8+4+8 of the first five -> four buckets sent, (6, 4, 5, 4) at positions 2 5 6 7 wait.
    it 2 forward (10): Case 1 over (6, 4, 5, 4): 6+4 (smallest mask among the sums of 10) -> two
      sent, (5, 4) wait: the two buckets left from the first iteration.
    it 2 backward: 9 fits 21 -> Case 3: both go first (the first iteration is complete), 12
      left.  Remaining time per length 8..1: 12 12 12 12 10 10 7 6; values 12 12 12 12 10 9 1 1;
      length 5 is the shortest that reaches 12: 8+4 -> two sent; count 2 + 2 = 4, time 9 + 12.
      Update with k = 1 at the end of iteration 2."""
    data, told = _fig4_fixture()
    n = data["buckets"][0]
    iters = len(told["backward_case"])
    r = oracle.simulate_batch(one(data["comm_time"], data["drop_time"], data["forward_window"][0],
                                  data["backward_window"][0], iters))
    assert r.status.tolist() == [0] and len(data["comm_time"]) == n == 8
    case, cnt, upd = r.stage_case[0], r.stage_count[0], r.update_k[0]
    assert case[0].tolist() == [0, 4]            # nothing to send before the first backward stage
    for t in range(iters):
        if told["backward_case"][t] is not None:
            assert case[t, 1] == told["backward_case"][t], t
        if told["forward_case"][t] is not None:
            assert case[t, 0] == told["forward_case"][t], t
        if told["update_k"][t] is not None:
            assert upd[t] == told["update_k"][t], t
        if told["left_before_backward"][t] is not None:
            # the queue was filled by the previous backward stage (Case 4: all n new buckets
            # minus what Algorithm 1 sent) and served by this iteration's forward stage
            assert case[t - 1, 1] == 4 and n - cnt[t - 1, 1] - cnt[t, 0] == told["left_before_backward"][t], t
        if told["left_after_backward"][t] is not None:
            # the next backward stage finds the queue empty (Case 4), so what was left is
            # exactly what the forward stage in between sent
            assert case[t + 1, 1] == 4 and case[t + 1, 0] == 1 and cnt[t + 1, 0] == told["left_after_backward"][t], t
        if told["merged_iterations_in_backward_list"][t] is not None:
            # the merged list's iterations are applied together, in the update that follows
            k = told["merged_iterations_in_backward_list"][t]
            later = upd[t:]
            assert case[t - 1, 1] == 2 and k in later.tolist(), t
    # the hand-worked first two iterations, and the rest as the reading gives it
    assert cnt[:2].tolist() == [[0, 4], [2, 4]] and r.stage_time[0, :2].tolist() == [[0, 21], [10, 21]]
    assert case.tolist() == [[0, 4], [1, 3], [1, 3], [1, 2], [1, 4], [1, 3]]
    assert upd.tolist() == [0, 1, 1, 0, 1, 2] and r.tail[0].tolist() == [1, 0]


def test_forward_stage_clears_the_queue(oracle):
    """One bucket of time 5, forward window 5, backward window 4 (too short for it): it is
    generated in every backward stage, waits, goes in the next forward stage (Case 1), and
    its iteration is applied at the end of that iteration (queue found empty: Case 4)."""
    r = oracle.simulate_batch(one([5], [0], 5, 4, 5))
    assert r.stage_case[0].tolist() == [[0, 4], [1, 4], [1, 4], [1, 4], [1, 4]]
    assert r.stage_count[0].tolist() == [[0, 0], [1, 0], [1, 0], [1, 0], [1, 0]]
    assert r.update_k[0].tolist() == [0, 1, 1, 1, 1]
    assert r.tail[0].tolist() == [1, 0]


def test_closed_forms(oracle):
    comm = [7, 3, 9, 4, 6]
    # a backward window that holds everything: every iteration synchronises all and updates (plain data parallelism)
    r = oracle.simulate_batch(one(comm, [0] * 5, 10, sum(comm), 4))
    assert r.stage_case[0].tolist() == [[0, 4]] * 4 and r.stage_count[0].tolist() == [[0, 5]] * 4
    assert r.update_k[0].tolist() == [1, 1, 1, 1] and r.tail[0].tolist() == [0, 0]
    # no time at all: nothing is ever synchronised, gradients pile up in the future queue
    r = oracle.simulate_batch(one(comm, [0] * 5, 0, 0, 4))
    assert r.stage_case[0].tolist() == [[0, 4], [1, 2], [1, 2], [1, 2]]
    assert (r.stage_count == 0).all() and (r.update_k == 0).all() and r.tail[0].tolist() == [1, 3]
    assert r.sweep_cells.tolist() == [0]


def replay(sb, b, r):
    """The cases replayed with the enumeration solvers; returns what the oracle should report."""
    n, comm, drop = sb.n_buckets, sb.comm_time[b], sb.drop_time[b]
    cur = np.zeros(n, bool)
    cur_k = fut_k = done_k = 0
    cases, counts, times, upd = [], [], [], []
    for t in range(sb.iterations):
        for stage, window in ((0, int(sb.forward_time[b])), (1, int(sb.backward_time[b]))):
            ids = np.flatnonzero(cur)
            if len(ids) and (stage == 0 or comm[ids].sum() > window):
                val, mask = bf.best_subset(comm[ids], comm[ids], window)
                got = [ids[a] for a in range(len(ids)) if (mask >> a) & 1]
                cur[got] = False
                cases.append(1 if stage == 0 else 2); counts.append(len(got)); times.append(int(comm[got].sum()))
                fut_k += stage
                if not cur.any():
                    done_k += cur_k; cur_k = 0
            elif stage == 1:
                first_count, first_time = len(ids), int(comm[ids].sum())
                if len(ids):
                    done_k += cur_k
                val, load, lvl, rem, asg = bf.recursive_prefixes(comm, comm, drop, window - first_time)
                take = np.array(asg) == 0
                cases.append(3 if len(ids) else 4); counts.append(first_count + int(take.sum()))
                times.append(first_time + int(comm[take].sum()))
                cur = ~take
                cur_k, fut_k = fut_k + 1, 0
                if not cur.any():
                    done_k += cur_k; cur_k = 0
            else:
                cases.append(0); counts.append(0); times.append(0)
        upd.append(done_k); done_k = 0
    return cases, counts, times, upd, [cur_k, fut_k]


@pytest.mark.parametrize("seed", [201, 202, 203])
def test_replay_with_enumeration_and_conservation(oracle, seed):
    sb = W.random_schedules(seed, batch=30, n=9, iterations=10, w_hi=9, t_hi=3, f_hi=14, b_hi=30)
    r = oracle.simulate_batch(sb)
    assert (r.status == 0).all()
    assert (r.update_k.sum(axis=1) + r.tail.sum(axis=1) == sb.iterations).all()   # every iteration is applied once or still waits
    for b in range(sb.batch):
        cases, counts, times, upd, tail = replay(sb, b, r)
        assert r.stage_case[b].ravel().tolist() == cases, b
        assert r.stage_count[b].ravel().tolist() == counts, b
        assert r.stage_time[b].ravel().tolist() == times, b
        assert r.update_k[b].tolist() == upd and r.tail[b].tolist() == tail, b


def test_paper_shape_properties(oracle):
    """ResNet-101 shape: a stage never uses more than its window; every iteration is applied
    once or still waits; with b + f buckets per iteration on average the updates per
    iteration approach (b + f) / n."""
    sb = W.resnet101_schedules(batch=3, iterations=6)
    r = oracle.simulate_batch(sb, nthreads=3)
    assert (r.status == 0).all()
    assert (r.stage_time[:, :, 0] <= sb.forward_time[:, None]).all()
    assert (r.stage_time[:, :, 1] <= sb.backward_time[:, None]).all()
    assert (r.update_k.sum(axis=1) + r.tail.sum(axis=1) == sb.iterations).all()


def test_status_codes(oracle):
    sb = W.random_schedules(204, batch=5, n=4, iterations=3, w_hi=9, t_hi=3, f_hi=10, b_hi=10)
    sb.comm_time[1, 2] = 0
    sb.drop_time[2, 0] = -1
    sb.backward_time[3] = 11
    sb.comm_time[4] = 2 ** 30
    r = oracle.simulate_batch(sb, cap_limit=10)
    assert r.status.tolist() == [0, 1, 1, 2, 3]
    assert (r.stage_case[1:] == 0).all() and (r.update_k[1:] == 0).all()
