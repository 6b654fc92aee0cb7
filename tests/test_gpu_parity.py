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
    seq = kb.mode == W.MODE_SEQUENTIAL
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
    (13000, 13055),    # 256 x 51
    (20000, 26111),    # 512 x 51
    (33000, 38000),    # 1024 x 40
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
