"""Optimality-gap report: the paper's greedy heuristic (Sec. III.C) against the exact
solvers of this library, on the same synthetic profiles, all through the HIP path.

    python -m paper_2503_16815_amd.greedy_gap

Per workload: mean and worst ratio greedy / exact of the scheduled value, the share of
instances where the heuristic reaches the exact value, and the time of each solve.
"Exact" is the sequential fill (each window solved exactly, Sec. III.B) for the
one-link shapes and the joint two-link optimum (Sec. III.C, Problem 2) for the two-link
shape; the latter is the true optimum of the problem the heuristic approximates.
"""
from __future__ import annotations

import json
import sys
import time

import numpy as np


def main() -> int:
    import torch
    from . import binding, workloads as W

    if not torch.cuda.is_available():
        print("greedy_gap: no GPU visible", file=sys.stderr)
        return 1
    hj = W.hetero_joint()
    hj_time = hj.slice(0, hj.batch)
    hj_time.name = "hetero_joint, value = time on link 0"
    hj_time.values = np.ascontiguousarray(hj.weights[:, 0, :])
    cases = [W.resnet101_sweep(), W.vgg19_sweep(), W.gpt2_shaped(), hj, hj_time]
    rows = []
    for kb in cases:
        two = kb.mode == W.MODE_JOINT2
        limits = dict(max_batch=kb.batch, max_items=kb.item_stride, max_knapsacks=kb.knap_stride)
        if two:
            limits.update(max_c1=int(kb.capacities[:, 0].max()), max_c2=int(kb.capacities[:, 1].max()))
        else:
            limits.update(max_capacity=int(kb.capacities.max()))
        with binding.DeftKnapsack(**limits) as h:
            res = {}
            for name, batch in (("exact", kb), ("greedy", W.as_greedy(kb))):
                db = h.upload(batch)
                h.solve_batch(db)                      # warm-up
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                out = h.solve_batch(db)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3
                assert (out.status == 0).all()
                res[name] = (out.total_value.cpu().numpy().astype(np.float64), ms)
        exact, greedy = res["exact"][0], res["greedy"][0]
        ok = exact > 0
        ratio = greedy[ok] / exact[ok]
        rows.append(dict(workload=kb.name, instances=int(kb.batch), items=int(kb.item_stride),
                         mean_ratio=float(ratio.mean()), worst_ratio=float(ratio.min()),
                         best_ratio=float(ratio.max()), share_equal=float((greedy[ok] == exact[ok]).mean()),
                         share_greedy_above=float((greedy[ok] > exact[ok]).mean()),
                         exact_ms=res["exact"][1], greedy_ms=res["greedy"][1]))
        print(json.dumps(rows[-1]), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
