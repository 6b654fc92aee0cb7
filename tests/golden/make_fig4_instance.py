"""Finds an eight-bucket instance on which the oracle's task-queue simulation goes through
the sequence of cases and updates that the paper narrates for its Fig. 4 (Sec. III.B), and
prints it in the format of fig4_walkthrough.txt.  Calls only the oracle.  Seeded: the
first hit of the search is the committed instance.

    python tests/golden/make_fig4_instance.py
"""
import os
import sys
from types import SimpleNamespace

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import oracle  # noqa: E402


def main() -> int:
    r = np.random.default_rng(5)
    B, n, iters = 200000, 8, 6
    comm = r.integers(1, 10, size=(B, n)).astype(np.int32)
    drop = r.integers(0, 4, size=(B, n)).astype(np.int32)
    fwd = r.integers(2, 12, size=B).astype(np.int32)
    bwd = r.integers(6, 24, size=B).astype(np.int32)
    sb = SimpleNamespace(batch=B, n_buckets=n, iterations=iters, comm_time=comm, drop_time=drop,
                         forward_time=fwd, backward_time=bwd)
    res = oracle.simulate_batch(sb, nthreads=os.cpu_count() or 1)
    c, cnt, u = res.stage_case, res.stage_count, res.update_k
    ok = (c[:, 0, 1] == 4) & (c[:, 1, 0] == 1) & (c[:, 1, 1] == 3) & (c[:, 3, 1] == 2) & (c[:, 4, 1] == 4)
    ok &= (u[:, 0] == 0) & (u[:, 1] == 1) & (u[:, 5] == 2)
    ok &= n - cnt[:, 0, 1] - cnt[:, 1, 0] == 2      # two buckets of iteration 1 left before iteration 2's backward stage
    ok &= (c[:, 4, 0] == 1) & (cnt[:, 4, 0] == 2)   # the two left after iteration 4's backward stage go in iteration 5's forward stage
    hits = np.flatnonzero(ok)
    if len(hits) == 0:
        print("no instance found", file=sys.stderr)
        return 1
    b = int(hits[0])
    print("buckets", n)
    print("comm_time", *comm[b].tolist())
    print("drop_time", *drop[b].tolist())
    print("forward_window", int(fwd[b]))
    print("backward_window", int(bwd[b]))
    return 0


if __name__ == "__main__":
    sys.exit(main())
