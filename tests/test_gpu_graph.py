"""A solve call only enqueues kernels (no allocation, no memset, no host read), so it can be
recorded into a HIP graph and replayed.  Each replay, with fresh inputs copied into the same
device buffers and the program's own eager work in between, must match the oracle."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W
from tests.test_gpu_parity import assert_same, binding  # noqa: F401  (binding is a fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("max_capacity", [3000, 60000])   # rows in LDS / rows in global memory
def test_solve_batch_replayed_from_a_graph(binding, oracle, max_capacity):
    import torch
    cap_hi = max_capacity - 100
    batches = [W.random_sequential(5000 + s, batch=40, n_max=50, m_max=4, w_hi=max(20, cap_hi // 8), v_hi=500,
                                   cap_hi=cap_hi, ragged=False) for s in range(3)]
    refs = [oracle.solve_batch(kb, nthreads=8) for kb in batches]
    with binding.DeftKnapsack(max_batch=40, max_items=50, max_knapsacks=4, max_capacity=max_capacity) as h:
        db = h.upload(batches[0])
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            h.solve_batch(db)                      # warm-up outside the capture
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            h.solve_batch(db, torch.cuda.current_stream())
        for rep in range(2):
            for kb, ref in zip(batches, refs):
                for name in ("n_items", "n_knapsacks", "weights", "values", "capacities", "fill_order"):
                    getattr(db, name).copy_(torch.from_numpy(np.ascontiguousarray(getattr(kb, name), np.int32)))
                for t in (db.out.total_value, db.out.assignment, db.out.knap_value, db.out.knap_load, db.out.status):
                    t.fill_(-7)                    # eager work between the replays
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert_same(kb, db.out, ref)


def test_two_handles_on_two_streams_at_once(binding, oracle):
    """Handles share nothing: solves enqueued alternately on two streams, each with its own
    handle (one with rows in LDS, one with rows in global memory), overlap on the GPU and both
    match the oracle."""
    import torch
    ka = W.resnet101_shaped(k=2, batch=600)
    kg = W.random_sequential(5100, batch=130, n_max=40, m_max=3, w_hi=9000, v_hi=500, cap_hi=70000)
    ra, rg = oracle.solve_batch(ka, nthreads=16), oracle.solve_batch(kg, nthreads=16)
    sa, sg = torch.cuda.Stream(), torch.cuda.Stream()
    with binding.DeftKnapsack(max_batch=600, max_items=314, max_knapsacks=4,
                              max_capacity=int(ka.capacities.max())) as ha, \
            binding.DeftKnapsack(max_batch=130, max_items=40, max_knapsacks=3, max_capacity=70000) as hg:
        da, dg = ha.upload(ka), hg.upload(kg)
        torch.cuda.synchronize()
        for _ in range(3):
            oa = ha.solve_batch(da, sa)
            og = hg.solve_batch(dg, sg)
        sa.synchronize()
        sg.synchronize()
        assert_same(ka, oa, ra)
        assert_same(kg, og, rg)
