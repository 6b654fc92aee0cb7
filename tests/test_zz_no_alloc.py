"""The entry point that allocates nothing (deft_knapsack_solve_batch_static: no handle, the
library's built-in scratch array) against the handle-based deft_knapsack_solve_batch, through
the C ABI, bit-exact on every output: two calls in a row, the second smaller than the first
(whatever the first left in the shared array must not show), then a third on another kernel."""
import numpy as np
import pytest

from paper_2503_16815_amd import workloads as W

pytestmark = pytest.mark.gpu

KEYS = ("status", "total_value", "knap_value", "knap_load", "assignment")


def _host(out):
    return {k: getattr(out, k).cpu().numpy().copy() for k in KEYS}


def test_static_entry_matches_the_handle_entry(oracle):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_16815_amd import binding
    binding.load_library()
    dev = torch.device("cuda", 0)
    calls = [
        (W.resnet101_shaped(k=2, batch=64), 13055),                       # 42 MB of the 64 MiB array, 512-lane kernel
        (W.resnet101_shaped(k=1, batch=9, seed=77), 13055),               # smaller, same kernel, other data
        (W.random_sequential(9101, batch=50, n_max=40, m_max=4, w_hi=150, v_hi=900, cap_hi=1000), 1023),
        (W.filling_rows(9102, batch=5, n_max=700, m_max=3, w_hi=30, cap_lo=2500, cap_hi=4095), 4095),
    ]
    # the handle entry point's answers first (each handle freed before the static calls run)
    want = []
    for kb, cap in calls:
        with binding.DeftKnapsack(max_batch=kb.batch, max_items=kb.item_stride, max_knapsacks=kb.knap_stride,
                                  max_capacity=cap) as h:
            out = h.solve_batch(h.upload(kb))
            torch.cuda.synchronize()
            want.append(_host(out))
    dbs = [binding.DeviceBatch(kb, dev) for kb, _ in calls]
    for db in dbs:                                    # poison the outputs: every slot must be written
        for k in KEYS:
            getattr(db.out, k).fill_(-7)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info(dev)[0]
    for i, ((kb, cap), db) in enumerate(zip(calls, dbs)):
        print(f"static call {i}: {kb.name} batch={kb.batch} n={kb.item_stride} max_capacity={cap}", flush=True)
        out = binding.solve_batch_static(db, cap)     # back to back on one stream, no sync in between
    torch.cuda.synchronize()
    print(f"device memory free before/after the static calls: {free0} / {torch.cuda.mem_get_info(dev)[0]}", flush=True)
    for i, ((kb, cap), db) in enumerate(zip(calls, dbs)):
        got = _host(db.out)
        for k in KEYS:
            assert np.array_equal(got[k], want[i][k]), (i, kb.name, k)
        ref = oracle.solve_batch(kb, nthreads=16, cap_limit=cap)
        for k in KEYS:
            assert np.array_equal(got[k], getattr(ref, k)), (i, kb.name, k, "oracle")


def test_static_entry_refuses_what_does_not_fit():
    import torch
    from paper_2503_16815_amd import binding
    dev = torch.device("cuda", 0)
    big = binding.DeviceBatch(W.resnet101_shaped(k=1, batch=1024), dev)          # 660 MB of keep table
    with pytest.raises(binding.DeftError) as e:
        binding.solve_batch_static(big, 13055)
    assert e.value.code == binding.DEFT_ERR_LIMIT
    small = binding.DeviceBatch(W.tiny_single(), dev)
    with pytest.raises(binding.DeftError) as e:
        binding.solve_batch_static(small, 50000)                                   # rows in global memory: no
    assert e.value.code == binding.DEFT_ERR_LIMIT
    with pytest.raises(binding.DeftError) as e:
        binding.solve_batch_static(small, 0)
    assert e.value.code == binding.DEFT_ERR_INVALID_ARG
    joint = binding.DeviceBatch(W.hetero_joint(batch=2, n=8, c1=20, c2=20), dev)
    with pytest.raises(binding.DeftError) as e:
        binding.solve_batch_static(joint, 1000)
    assert e.value.code == binding.DEFT_ERR_INVALID_ARG
    out = binding.solve_batch_static(small, 1000)                                  # and still serves what fits
    torch.cuda.synchronize()
    assert int(out.status[0]) == 0 and int(out.total_value[0]) > 0
