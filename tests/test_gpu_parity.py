"""GPU parity: the HIP path (through the C ABI) against the CPU oracle,
bit-exact on every output, on the same seeded inputs."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_16815_amd import binding as b
    b.load_library()
    return b


def assert_same(kb, out, ref):
    import torch
    torch.cuda.synchronize()
    got = dict(status=out.status.cpu().numpy(), total_value=out.total_value.cpu().numpy(),
               knap_value=out.knap_value.cpu().numpy(), knap_load=out.knap_load.cpu().numpy(),
               assignment=out.assignment.cpu().numpy())
    exp = dict(status=ref.status, total_value=ref.total_value, knap_value=ref.knap_value,
               knap_load=ref.knap_load, assignment=ref.assignment)
    for key in ("status", "total_value", "knap_value", "knap_load", "assignment"):
        g, e = got[key], exp[key]
        assert g.shape == e.shape, key
        if not np.array_equal(g, e):
            bad = np.argwhere(g != e)[0]
            raise AssertionError(f"{kb.name}: {key} differs first at {bad.tolist()}: "
                                 f"gpu={g[tuple(bad)]} oracle={e[tuple(bad)]} "
                                 f"({(g != e).sum()} of {g.size} entries differ)")


def run(binding, oracle, kb, **limits):
    print(f"case {kb.name} batch={kb.batch} n={kb.item_stride} m={kb.knap_stride} limits={limits}", flush=True)
    seq = kb.mode not in (W.MODE_JOINT2, W.MODE_GREEDY2)
    ref = oracle.solve_batch(kb, nthreads=16, cap_limit=limits.get("max_capacity", -1) if seq else -1,
                             c1_limit=limits.get("max_c1", -1), c2_limit=limits.get("max_c2", -1))
    out = binding.solve(kb, **limits)
    assert_same(kb, out, ref)
    return ref


def test_tiny_single_and_bruteforce_batch(binding, oracle):
    run(binding, oracle, W.tiny_single())
    run(binding, oracle, W.tiny_bruteforce())


@pytest.mark.parametrize("cap_hi,max_capacity", [
    (700, 1023),       # wavefront-per-instance variant
    (3000, 4095),      # 256 x 16
    (8000, 8191),      # 256 x 32
    (10000, 10239),    # 512 x 20
    (13000, 13055),    # 512 x 26
    (19900, 19967),    # 768 x 26
    (20000, 26111),    # 1024 x 26
    (38900, 38911),    # 1024 x 38
])
def test_random_ragged_every_lds_variant(binding, oracle, cap_hi, max_capacity):
    """Ragged n and m, random fill order, capacities from 0 up to several tiles
    with a ragged tail, for each compiled (threads, cells) variant."""
    kb = W.random_sequential(1000 + cap_hi, batch=37, n_max=45, m_max=4, w_hi=max(20, cap_hi // 6),
                             v_hi=1000, cap_hi=cap_hi)
    run(binding, oracle, kb, max_capacity=max_capacity)
    kt = W.random_sequential(2000 + cap_hi, batch=19, n_max=60, m_max=3, w_hi=max(9, cap_hi // 40),
                             v_hi=9, cap_hi=cap_hi, ties=True)
    run(binding, oracle, kt, max_capacity=max_capacity)


def test_global_row_path_large_capacity(binding, oracle):
    """Rows too long for LDS go through the global-memory path: several 2048-cell
    wave chunks, a ragged tail, ragged n/m, random fill order."""
    kb = W.random_sequential(3001, batch=9, n_max=40, m_max=3, w_hi=9000, v_hi=5000, cap_hi=70000)
    run(binding, oracle, kb, max_capacity=70000)
    kt = W.random_sequential(3002, batch=5, n_max=50, m_max=2, w_hi=3000, v_hi=9, cap_hi=50000, ties=True)
    run(binding, oracle, kt, max_capacity=50000)


def test_global_row_path_persistent_sweep(binding, oracle):
    """Batches of at least half the compute units take the one-workgroup-per-instance
    sweep (row streamed through an LDS ring): light items, items heavier than the
    ring can hold (shifted operand from global memory), ragged n/m, tie-heavy data."""
    kb = W.random_sequential(3101, batch=140, n_max=14, m_max=3, w_hi=60000, v_hi=5000, cap_hi=90000)
    run(binding, oracle, kb, max_capacity=90000)
    kl = W.random_sequential(3102, batch=130, n_max=24, m_max=2, w_hi=3000, v_hi=50, cap_hi=60000)
    run(binding, oracle, kl, max_capacity=60000)
    kt = W.random_sequential(3103, batch=129, n_max=30, m_max=2, w_hi=2500, v_hi=9, cap_hi=45000, ties=True)
    run(binding, oracle, kt, max_capacity=45000)


def test_joint_two_link(binding, oracle):
    run(binding, oracle, W.random_joint(4001, batch=21, n_max=30, w_hi=40, v_hi=1000, c1_hi=150, c2_hi=200))
    run(binding, oracle, W.hetero_joint(batch=6, n=40, c1=200, c2=129))
    kb = W.random_joint(4002, batch=8, n_max=20, w_hi=6, v_hi=6, c1_hi=40, c2_hi=70, ragged=False)
    kb.weights[:, 1] = kb.weights[:, 0]
    kb.values[:] = kb.weights[:, 0]          # w0 == w1 == v: the paper's Problem 2, tie-heavy
    run(binding, oracle, kb)


def test_paper_shaped_batches_reduced(binding, oracle):
    run(binding, oracle, W.resnet101_shaped(k=4, batch=48))
    run(binding, oracle, W.vgg19_shaped(k=4, batch=192))
    run(binding, oracle, W.gpt2_shaped(batch=3))
    run(binding, oracle, W.hetero_joint(batch=4))


def _faulty_sequential():
    kb = W.random_sequential(61, batch=9, n_max=6, m_max=2, w_hi=9, v_hi=9, cap_hi=20, ragged=False,
                             permute_order=False)
    kb.weights[1, 2] = 0
    kb.values[2, 0] = -1
    kb.capacities[3, 1] = -5
    kb.fill_order[4] = [1, 1]
    kb.values[5, :] = 2 ** 30
    kb.capacities[6, 0] = 1000
    kb.n_items[7] = 7
    kb.n_knapsacks[8] = -1
    return kb


def test_per_instance_status_lds_and_global_paths(binding, oracle):
    kb = _faulty_sequential()
    ref = run(binding, oracle, kb, max_capacity=100)
    assert ref.status.tolist() == [0, 1, 1, 1, 1, 3, 2, 1, 1]
    run(binding, oracle, kb, max_capacity=50000)           # same data through the global-row path
    kj = W.random_joint(62, 5, 5, 5, 5, 10, 10, ragged=False)
    kj.n_knapsacks[1] = 1
    kj.capacities[2, 1] = 11
    kj.weights[3, 1, 4] = 0
    kj.values[4, :] = 2 ** 30
    refj = run(binding, oracle, kj, max_c1=10, max_c2=10)
    assert refj.status.tolist() == [0, 1, 2, 1, 3]


def test_empty_and_degenerate(binding, oracle):
    kb = W.random_sequential(71, batch=6, n_max=5, m_max=2, w_hi=9, v_hi=9, cap_hi=20, ragged=False)
    kb.n_items[0] = 0
    kb.n_knapsacks[1] = 0
    kb.capacities[2] = 0
    kb.weights[3] = 100              # nothing fits
    kb.values[4] = 0                 # zero values: nothing is ever taken
    run(binding, oracle, kb)
    run(binding, oracle, kb, max_capacity=45000)


def test_repeat_runs_are_bit_identical(binding, oracle):
    """The in-place LDS sweep has a read-before-write hazard across wavefronts
    that the barriers must close: repeated solves must agree exactly."""
    import torch
    kb = W.resnet101_shaped(k=2, batch=64)
    with binding.DeftKnapsack(max_batch=64, max_items=314, max_knapsacks=4,
                              max_capacity=int(kb.capacities.max())) as h:
        db = h.upload(kb)
        first = None
        for _ in range(5):
            out = h.solve_batch(db)
            torch.cuda.synchronize()
            cur = (out.total_value.clone(), out.assignment.clone(), out.knap_load.clone())
            if first is None:
                first = cur
            else:
                assert all(torch.equal(a, b) for a, b in zip(first, cur))


def test_one_handle_reused_across_layouts(binding, oracle):
    """Calls with different knapsack strides and item counts reuse one handle's
    scratch at shifting offsets; every repeat must still match the oracle (nothing
    written by an earlier launch may be served again from a cache)."""
    import torch
    calls = [W.vgg19_shaped(k=k, batch=512) for k in (1, 2, 3, 4)]
    calls.append(W.random_sequential(991, batch=300, n_max=30, m_max=5, w_hi=900, v_hi=50, cap_hi=9000))
    refs = [oracle.solve_batch(kb, nthreads=16) for kb in calls]
    with binding.DeftKnapsack(max_batch=512, max_items=38, max_knapsacks=8, max_capacity=9300) as h:
        dbs = [h.upload(kb) for kb in calls]
        for rep in range(4):
            outs = [h.solve_batch(db) for db in dbs]
            torch.cuda.synchronize()
            for kb, out, ref in zip(calls, outs, refs):
                assert_same(kb, out, ref)


def test_full_size_sweeps(binding, oracle):
    """The two LDS-path workloads at the sizes and in the launch shape bench.py times:
    every output of every instance against the oracle."""
    run(binding, oracle, W.resnet101_sweep())
    run(binding, oracle, W.vgg19_sweep())


def test_full_size_gpt2_and_two_link(binding, oracle):
    """The GPT-2-shaped batch (rows in global memory, persistent sweep) and the two-link
    batch at full size: every output of every instance against the oracle."""
    run(binding, oracle, W.gpt2_shaped())
    run(binding, oracle, W.hetero_joint())


@pytest.mark.parametrize("seed,n_max,w_hi,cap_hi,ties", [
    (4001, 12, 9, 30, True),       # few items: enumeration, everything-fits and empty stages
    (4002, 12, 40, 60, False),
    (4003, 90, 6, 300, True),      # many small equal-value items: rows fill up long before the list ends
    (4004, 90, 6, 300, False),     # the same with values that differ from the weights (no early end)
    (4005, 200, 30, 4000, True),   # 256-lane variant, several 64-entry list chunks, rows that fill up
])
def test_stage_shortcuts_randomized(binding, oracle, seed, n_max, w_hi, cap_hi, ties):
    """Large random batches aimed at the stages that are settled without a sweep (nothing
    offered, everything fits, at most six items) and at sweeps that end when the row is
    full, mixed with ordinary stages in one instance; ragged n and m, random fill order."""
    kb = W.random_sequential(seed, batch=1500, n_max=n_max, m_max=6, w_hi=w_hi, v_hi=50, cap_hi=cap_hi, ties=ties)
    run(binding, oracle, kb)


@pytest.mark.parametrize("max_capacity,n_max,w_hi,batch", [
    (1023, 160, 30, 64),        # wavefront-per-instance variant
    (4095, 600, 30, 40),        # 256 x 16
    (8191, 1160, 30, 32),       # 256 x 32
    (10239, 1450, 30, 28),      # 512 x 20
    (13311, 1890, 30, 24),      # 512 x 26
    (19967, 2830, 30, 20),      # 768 x 26: write-back groups on both sides of the second add-TID base
    (26623, 3000, 39, 16),      # 1024 x 26
    (38911, 3000, 57, 12),      # 1024 x 38
])
def test_rows_that_fill_early_every_lds_variant(binding, oracle, max_capacity, n_max, w_hi, batch):
    """Value = weight, light items, capacities in the upper half of each variant's range and two
    or three windows in random order: every swept stage reaches "every sum up to C is reachable"
    well before its list ends, so the sweep's early end, the write-back of a row that uses the
    variant's highest slots, the partial keep-row flags and the walk that starts at the last
    swept item all run together; the library's swept-cell count must equal the replay of the
    early end from the oracle's results (which also shows that rows did fill)."""
    import torch
    import bench
    kb = W.filling_rows(8000 + max_capacity, batch=batch, n_max=n_max, m_max=3, w_hi=w_hi,
                        cap_lo=max_capacity * 55 // 100, cap_hi=max_capacity)
    print(f"case {kb.name} batch={kb.batch} n<={n_max} max_capacity={max_capacity}", flush=True)
    ref = oracle.solve_batch(kb, nthreads=16, cap_limit=max_capacity)
    settled, full = bench.cells_not_swept(kb, ref, True)
    assert full > 0.2 * int(ref.touched_cells.sum()), "the case is meant to end sweeps early"
    with binding.DeftKnapsack(max_batch=kb.batch, max_items=kb.item_stride, max_knapsacks=kb.knap_stride,
                              max_capacity=max_capacity) as h:
        assert h.info().seq_path in (1, 2)
        db = h.upload(kb)
        h.set_profiling(True)
        out = h.solve_batch(db)
        torch.cuda.synchronize()
        prof = h.get_profile()
        assert_same(kb, out, ref)
    assert int(prof.swept_cell_updates) == int(ref.touched_cells.sum()) - settled - full, kb.name


def test_swept_cell_counter_matches_the_replay_from_the_oracle(binding, oracle):
    """The library's count of the cell-updates its sweeps evaluated (measurement only) against
    the same number derived from the oracle's results and the two rules (stages settled without
    a sweep, items after a full row), on shapes where both rules fire."""
    import torch
    import bench
    for kb in (W.resnet101_shaped(k=3, batch=96), W.vgg19_shaped(k=4, batch=200),
               W.random_sequential(4101, batch=300, n_max=90, m_max=5, w_hi=6, v_hi=9, cap_hi=300, ties=True)):
        ref = oracle.solve_batch(kb, nthreads=16)
        settled, full = bench.cells_not_swept(kb, ref, True)
        with binding.DeftKnapsack(max_batch=kb.batch, max_items=kb.item_stride, max_knapsacks=kb.knap_stride,
                                  max_capacity=max(1, int(kb.capacities.max()))) as h:
            assert h.info().seq_path in (1, 2)
            db = h.upload(kb)
            h.set_profiling(True)
            out = h.solve_batch(db)
            torch.cuda.synchronize()
            prof = h.get_profile()
            assert_same(kb, out, ref)
        assert int(prof.swept_cell_updates) == int(ref.touched_cells.sum()) - settled - full, kb.name
