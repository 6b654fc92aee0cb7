"""Seeded synthetic knapsack batches shaped on the paper's three DNN profiles.

This module only draws inputs; it holds none of the solver's arithmetic and is
the one piece shared by the CPU oracle's tests and the HIP path's tests/bench.
It depends on numpy alone.

The paper's real per-bucket profiles are not available, so every batch is a
stand-in built from the aggregate times it prints:

* Table I gives forward / backward / communication time per iteration
  (ResNet-101 59/118/242 ms, VGG-19 37/93/258 ms, GPT-2 169/381/546.4 ms):
  the backward and forward windows are the knapsack capacities, the
  communication time is the total item weight (Section III.B, Problem 1).
* Table II gives six VGG-19 bucket times with one bucket far above every
  window: the VGG-shaped generator reproduces that heavy tail.
* Section III.A (coverage ratio N:M) and III.B: when communication exceeds
  the windows of one iteration, leftovers are served by the windows of later
  iterations, so the (backward, forward) pair is repeated k times -> m = 2k
  knapsacks filled in time order.
* Section III.C, Problem 2: two links of different speed; one item costs a
  different time on each link.

Times are discretised by the caller: 10 us units for the ResNet/VGG shapes,
1 us units for the GPT-2 shape.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

MODE_SEQUENTIAL = 0
MODE_JOINT2 = 1
MODE_RECURSIVE = 2
MODE_GREEDY = 3       # the paper's greedy heuristic on the sequential layout
MODE_GREEDY2 = 4      # the same on the two-link layout (one time per link)
MODE_CAPACITY_SWEEP = 5   # one item list, several capacities of one knapsack (Section IV.C feedback)

SEED_TINY = 1001
SEED_RESNET = 1002
SEED_VGG = 1003
SEED_GPT2 = 1004
SEED_HETERO = 1005


@dataclass
class KnapsackBatch:
    """Host-side (numpy, int32, C-contiguous) image of one solver call.

    weights: [batch, item_stride] (sequential) or [batch, 2, item_stride] (joint)
    values: [batch, item_stride]
    capacities, fill_order: [batch, knap_stride]; fill_order may be None
    """

    name: str
    mode: int
    batch: int
    item_stride: int
    knap_stride: int
    n_items: np.ndarray
    n_knapsacks: np.ndarray
    weights: np.ndarray
    values: np.ndarray
    capacities: np.ndarray
    fill_order: Optional[np.ndarray] = None
    meta: dict = field(default_factory=dict)
    drop_time: Optional[np.ndarray] = None   # [batch, item_stride], recursive mode only

    def slice(self, lo: int, hi: int) -> "KnapsackBatch":
        fo = None if self.fill_order is None else np.ascontiguousarray(self.fill_order[lo:hi])
        return KnapsackBatch(
            name=f"{self.name}[{lo}:{hi}]", mode=self.mode, batch=hi - lo,
            item_stride=self.item_stride, knap_stride=self.knap_stride,
            n_items=np.ascontiguousarray(self.n_items[lo:hi]),
            n_knapsacks=np.ascontiguousarray(self.n_knapsacks[lo:hi]),
            weights=np.ascontiguousarray(self.weights[lo:hi]),
            values=np.ascontiguousarray(self.values[lo:hi]),
            capacities=np.ascontiguousarray(self.capacities[lo:hi]),
            fill_order=fo, meta=dict(self.meta),
            drop_time=None if self.drop_time is None else np.ascontiguousarray(self.drop_time[lo:hi]))

    def max_capacity(self) -> int:
        return int(self.capacities.max()) if self.capacities.size else 0


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _rescale_to_sum(x: np.ndarray, total: float) -> np.ndarray:
    """Round x * total / sum(x) per row to integers >= 1 (time discretisation)."""
    s = x.sum(axis=-1, keepdims=True)
    return np.maximum(1, np.rint(x * (total / s))).astype(np.int64)


def _sequential(name, weights, values, capacities, fill_order=None, meta=None) -> KnapsackBatch:
    weights = _i32(weights)
    b, n = weights.shape
    capacities = _i32(capacities)
    m = capacities.shape[1]
    return KnapsackBatch(
        name=name, mode=MODE_SEQUENTIAL, batch=b, item_stride=n, knap_stride=m,
        n_items=_i32(np.full(b, n)), n_knapsacks=_i32(np.full(b, m)),
        weights=weights, values=_i32(values), capacities=capacities,
        fill_order=None if fill_order is None else _i32(fill_order), meta=meta or {})


def tiny_single(seed: int = SEED_TINY) -> KnapsackBatch:
    """One instance: n=32, w~U{1..200}, v~U{1..1000}, capacities (1000, 500)."""
    r = _rng(seed)
    w = r.integers(1, 201, size=(1, 32))
    v = r.integers(1, 1001, size=(1, 32))
    return _sequential("tiny_single", w, v, [[1000, 500]], meta={"seed": seed})


def tiny_bruteforce(seed: int = SEED_TINY, batch: int = 64, n: int = 16) -> KnapsackBatch:
    """64 instances small enough (n=16) to enumerate; capacities (500, 250)."""
    r = _rng(seed + 7919)
    w = r.integers(1, 201, size=(batch, n))
    v = r.integers(1, 1001, size=(batch, n))
    cap = np.tile(np.array([[500, 250]]), (batch, 1))
    return _sequential("tiny_bruteforce", w, v, cap, meta={"seed": seed})


def resnet101_shaped(k: int = 1, batch: int = 1024, n: int = 314,
                     seed: int = SEED_RESNET) -> KnapsackBatch:
    """ResNet-101 shape (Table I, 10 us units): total comm 24200, backward
    window 11800 and forward window 5900 each jittered +-10 % per instance,
    the pair repeated k times (m = 2k); value = weight (Problem 1)."""
    r = _rng(seed)
    x = r.lognormal(mean=0.0, sigma=1.2, size=(batch, n))
    w = _rescale_to_sum(x, 24200.0)
    u = r.uniform(0.9, 1.1, size=(batch, 2))
    pair = np.rint(np.array([11800.0, 5900.0])[None, :] * u).astype(np.int64)
    cap = np.tile(pair, (1, k))
    return _sequential(f"resnet101_k{k}", w, w.copy(), cap, meta={"seed": seed, "k": k})


def vgg19_shaped(k: int = 1, batch: int = 4096, n: int = 38,
                 seed: int = SEED_VGG) -> KnapsackBatch:
    """VGG-19 shape (Tables I and II, 10 us units): total comm 25800 with three
    heavy items holding about 85 % of it; windows 9300 / 3700; value = weight."""
    r = _rng(seed)
    heavy_share = r.uniform(0.9, 1.1, size=(batch, 3))
    heavy_share = heavy_share / heavy_share.sum(axis=1, keepdims=True)
    heavy = np.maximum(1, np.rint(heavy_share * (0.85 * 25800.0))).astype(np.int64)
    light = _rescale_to_sum(r.lognormal(0.0, 1.0, size=(batch, n - 3)), 0.15 * 25800.0)
    w = np.empty((batch, n), dtype=np.int64)
    for b in range(batch):
        pos = r.permutation(n)
        w[b, pos[:3]] = heavy[b]
        w[b, pos[3:]] = light[b]
    cap = np.tile(np.array([[9300, 3700]]), (batch, k))
    return _sequential(f"vgg19_k{k}", w, w.copy(), cap, meta={"seed": seed, "k": k})


def concat(batches, name: str) -> KnapsackBatch:
    """One call holding the instances of several sequential batches with the same
    item count; shorter capacity rows are padded with unused (zero) knapsacks."""
    ks = max(kb.knap_stride for kb in batches)

    def pad(a: np.ndarray) -> np.ndarray:
        out = np.zeros((a.shape[0], ks), dtype=np.int32)
        out[:, :a.shape[1]] = a
        return out

    assert all(kb.mode == MODE_SEQUENTIAL and kb.fill_order is None and
               kb.item_stride == batches[0].item_stride for kb in batches)
    return KnapsackBatch(
        name=name, mode=MODE_SEQUENTIAL, batch=sum(kb.batch for kb in batches),
        item_stride=batches[0].item_stride, knap_stride=ks,
        n_items=_i32(np.concatenate([kb.n_items for kb in batches])),
        n_knapsacks=_i32(np.concatenate([kb.n_knapsacks for kb in batches])),
        weights=_i32(np.concatenate([kb.weights for kb in batches])),
        values=_i32(np.concatenate([kb.values for kb in batches])),
        capacities=_i32(np.concatenate([pad(kb.capacities) for kb in batches])),
        meta={"parts": [kb.name for kb in batches]})


def resnet101_sweep(batch: int = 1024, ks=(4, 3, 2, 1)) -> KnapsackBatch:
    """The ResNet-101-shaped candidate set as one call: `batch` perturbed profiles,
    each with the window pair repeated k times for every k in `ks` (Section III.A:
    the delayed-update frequency decides how many windows serve one iteration's
    communication).  Longest instances (largest k) come first."""
    return concat([resnet101_shaped(k=k, batch=batch) for k in ks], "resnet101_sweep")


def vgg19_sweep(batch: int = 4096, ks=(4, 3, 2, 1)) -> KnapsackBatch:
    """The VGG-19-shaped candidate set as one call (see resnet101_sweep)."""
    return concat([vgg19_shaped(k=k, batch=batch) for k in ks], "vgg19_sweep")


def gpt2_shaped(batch: int = 256, n: int = 148, seed: int = SEED_GPT2) -> KnapsackBatch:
    """GPT-2 shape (Table I, 1 us units): total comm 546400, windows 381000 /
    169000; value = weight x U[1,4] priority."""
    r = _rng(seed)
    w = _rescale_to_sum(r.lognormal(0.0, 0.8, size=(batch, n)), 546400.0)
    v = np.rint(w * r.uniform(1.0, 4.0, size=(batch, n))).astype(np.int64)
    cap = np.tile(np.array([[381000, 169000]]), (batch, 1))
    return _sequential("gpt2", w, v, cap, meta={"seed": seed})


def hetero_joint(batch: int = 256, n: int = 64, c1: int = 512, c2: int = 512,
                 seed: int = SEED_HETERO) -> KnapsackBatch:
    """Two-link shape (Problem 2 with per-link times): w1~U{1..64} on the fast
    link, w2 = w1 x U{3..6} on the slow link, v~U{1..1000}, C1 = C2 = 512."""
    r = _rng(seed)
    w1 = r.integers(1, 65, size=(batch, n))
    w2 = w1 * r.integers(3, 7, size=(batch, n))
    v = r.integers(1, 1001, size=(batch, n))
    w = np.stack([w1, w2], axis=1)
    return KnapsackBatch(
        name="hetero_joint", mode=MODE_JOINT2, batch=batch, item_stride=n, knap_stride=2,
        n_items=_i32(np.full(batch, n)), n_knapsacks=_i32(np.full(batch, 2)),
        weights=_i32(w), values=_i32(v),
        capacities=_i32(np.tile(np.array([[c1, c2]]), (batch, 1))), meta={"seed": seed})


def random_sequential(seed: int, batch: int, n_max: int, m_max: int, w_hi: int, v_hi: int,
                      cap_hi: int, ragged: bool = True, ties: bool = False,
                      permute_order: bool = True) -> KnapsackBatch:
    """General ragged batch for parity and edge-case tests: per-instance n in
    [0, n_max], m in [0, m_max], capacities in [0, cap_hi], optional random fill
    order, optional value = weight (tie-heavy)."""
    r = _rng(seed)
    n_items = r.integers(0, n_max + 1, size=batch) if ragged else np.full(batch, n_max)
    n_knap = r.integers(0, m_max + 1, size=batch) if ragged else np.full(batch, m_max)
    w = r.integers(1, w_hi + 1, size=(batch, n_max))
    v = w.copy() if ties else r.integers(0, v_hi + 1, size=(batch, n_max))
    cap = r.integers(0, cap_hi + 1, size=(batch, max(m_max, 1)))
    order = np.tile(np.arange(max(m_max, 1)), (batch, 1))
    if permute_order:
        for b in range(batch):
            m = int(n_knap[b])
            order[b, :m] = r.permutation(m)
    kb = _sequential(f"random_seq_{seed}", w, v, cap, order, meta={"seed": seed})
    kb.n_items = _i32(n_items)
    kb.n_knapsacks = _i32(n_knap)
    return kb


def filling_rows(seed: int, batch: int, n_max: int, m_max: int, w_hi: int, cap_lo: int,
                 cap_hi: int) -> KnapsackBatch:
    """Value = weight with many light items and capacities in [cap_lo, cap_hi]: every sum up
    to the capacity becomes reachable long before the item list ends, stage after stage
    (the leftover of one window still overfills the next).  n in [n_max / 2, n_max], m in
    [2, m_max], random fill order."""
    r = _rng(seed)
    n_items = r.integers(n_max // 2, n_max + 1, size=batch)
    n_knap = r.integers(2, m_max + 1, size=batch)
    w = r.integers(1, w_hi + 1, size=(batch, n_max))
    cap = r.integers(cap_lo, cap_hi + 1, size=(batch, m_max))
    order = np.tile(np.arange(m_max), (batch, 1))
    for b in range(batch):
        m = int(n_knap[b])
        order[b, :m] = r.permutation(m)
    kb = _sequential(f"filling_rows_{seed}", w, w.copy(), cap, order, meta={"seed": seed})
    kb.n_items = _i32(n_items)
    kb.n_knapsacks = _i32(n_knap)
    return kb


def random_joint(seed: int, batch: int, n_max: int, w_hi: int, v_hi: int, c1_hi: int,
                 c2_hi: int, ragged: bool = True) -> KnapsackBatch:
    r = _rng(seed)
    n_items = r.integers(0, n_max + 1, size=batch) if ragged else np.full(batch, n_max)
    w = r.integers(1, w_hi + 1, size=(batch, 2, n_max))
    v = r.integers(0, v_hi + 1, size=(batch, n_max))
    cap = np.stack([r.integers(0, c1_hi + 1, size=batch), r.integers(0, c2_hi + 1, size=batch)], axis=1)
    return KnapsackBatch(
        name=f"random_joint_{seed}", mode=MODE_JOINT2, batch=batch, item_stride=n_max, knap_stride=2,
        n_items=_i32(n_items), n_knapsacks=_i32(np.full(batch, 2)), weights=_i32(w), values=_i32(v),
        capacities=_i32(cap), meta={"seed": seed})


def random_recursive(seed: int, batch: int, n_max: int, w_hi: int, v_hi: int, cap_hi: int, t_hi: int,
                     ragged: bool = True, ties: bool = False) -> KnapsackBatch:
    """Batches for Algorithm 1 (Section III.B): items in generation order, one remaining
    time per instance, and per item the time that leaving it out of the list takes off
    the remaining time (drawn in [0, t_hi]).  knap_stride is 2: slot 1 of the outputs
    reports the level whose answer was returned."""
    r = _rng(seed)
    n_items = r.integers(0, n_max + 1, size=batch) if ragged else np.full(batch, n_max)
    w = r.integers(1, w_hi + 1, size=(batch, n_max))
    v = w.copy() if ties else r.integers(0, v_hi + 1, size=(batch, n_max))
    cap = np.zeros((batch, 2), dtype=np.int64)
    cap[:, 0] = r.integers(0, cap_hi + 1, size=batch)
    drop = r.integers(0, t_hi + 1, size=(batch, n_max))
    return KnapsackBatch(
        name=f"random_recursive_{seed}", mode=MODE_RECURSIVE, batch=batch, item_stride=n_max, knap_stride=2,
        n_items=_i32(n_items), n_knapsacks=_i32(np.full(batch, 1)), weights=_i32(w), values=_i32(v),
        capacities=_i32(cap), meta={"seed": seed}, drop_time=_i32(drop))


def backward_stage_shaped(batch: int = 1024, n: int = 314, seed: int = SEED_RESNET + 50) -> KnapsackBatch:
    """ResNet-101-shaped backward stage for Algorithm 1 (Cases 3 and 4): the buckets of
    the running iteration appear one after the other while the backward pass computes, so
    scheduling only the first N - d of them may start d bucket computations later: items
    = bucket communication times (as resnet101_shaped), remaining time = the backward
    window, and leaving out bucket i costs its share of the backward computation time
    (proportional to its size, summing to the window)."""
    r = _rng(seed)
    x = r.lognormal(mean=0.0, sigma=1.2, size=(batch, n))
    w = _rescale_to_sum(x, 24200.0)
    cap = np.zeros((batch, 2), dtype=np.int64)
    cap[:, 0] = np.rint(11800.0 * r.uniform(0.9, 1.1, size=batch)).astype(np.int64)
    drop = np.maximum(0, np.rint(x / x.sum(axis=1, keepdims=True) * cap[:, :1])).astype(np.int64)
    return KnapsackBatch(
        name="backward_stage", mode=MODE_RECURSIVE, batch=batch, item_stride=n, knap_stride=2,
        n_items=_i32(np.full(batch, n)), n_knapsacks=_i32(np.full(batch, 1)), weights=_i32(w), values=_i32(w.copy()),
        capacities=_i32(cap), meta={"seed": seed}, drop_time=_i32(drop))


def as_greedy(kb: KnapsackBatch) -> KnapsackBatch:
    """The same instances, to be solved by the greedy heuristic of Section III.C
    (sequential layout -> MODE_GREEDY, two-link layout -> MODE_GREEDY2)."""
    assert kb.mode in (MODE_SEQUENTIAL, MODE_JOINT2)
    g = kb.slice(0, kb.batch)
    g.name = kb.name + "_greedy"
    g.mode = MODE_GREEDY if kb.mode == MODE_SEQUENTIAL else MODE_GREEDY2
    g.fill_order = None
    return g


def random_capacity_sweep(seed: int, batch: int, n_max: int, m_max: int, w_hi: int, v_hi: int, cap_hi: int,
                          ragged: bool = True, ties: bool = False) -> KnapsackBatch:
    """Capacity sweeps (Section IV.C feedback: the Solver called again with a larger
    capacity): per instance one item list and up to m_max capacities in random order."""
    r = _rng(seed)
    n_items = r.integers(0, n_max + 1, size=batch) if ragged else np.full(batch, n_max)
    m = r.integers(0, m_max + 1, size=batch) if ragged else np.full(batch, m_max)
    w = r.integers(1, w_hi + 1, size=(batch, n_max))
    v = w.copy() if ties else r.integers(0, v_hi + 1, size=(batch, n_max))
    cap = r.integers(0, cap_hi + 1, size=(batch, m_max))
    return KnapsackBatch(
        name=f"random_capacity_sweep_{seed}", mode=MODE_CAPACITY_SWEEP, batch=batch, item_stride=n_max,
        knap_stride=m_max, n_items=_i32(n_items), n_knapsacks=_i32(m), weights=_i32(w), values=_i32(v),
        capacities=_i32(cap), meta={"seed": seed})


def inflation_sweep_shaped(batch: int = 1024, n: int = 314, probes: int = 11, seed: int = SEED_RESNET + 60) -> KnapsackBatch:
    """ResNet-101-shaped feedback sweep: the backward window (11800 +-10 %, 10 us units) and
    ten inflated capacities, +5 % of the window each (the paper retries up to ten times and
    does not say by how much the capacity grows), over the 314 bucket times of
    resnet101_shaped."""
    r = _rng(seed)
    x = r.lognormal(mean=0.0, sigma=1.2, size=(batch, n))
    w = _rescale_to_sum(x, 24200.0)
    base = 11800.0 * r.uniform(0.9, 1.1, size=(batch, 1))
    cap = np.rint(base * (1.0 + 0.05 * np.arange(probes)[None, :])).astype(np.int64)
    return KnapsackBatch(
        name="inflation_sweep", mode=MODE_CAPACITY_SWEEP, batch=batch, item_stride=n, knap_stride=probes,
        n_items=_i32(np.full(batch, n)), n_knapsacks=_i32(np.full(batch, probes)), weights=_i32(w),
        values=_i32(w.copy()), capacities=_i32(cap), meta={"seed": seed})


@dataclass
class ScheduleBatch:
    """Candidate schedules for the task-queue simulation (Section III.B, Cases 1-4): per
    candidate the n bucket communication times in Algorithm 1's list order, the time each
    takes off the remaining time when left off the list, and the forward and backward
    windows; simulated for `iterations` iterations."""
    name: str
    batch: int
    n_buckets: int
    iterations: int
    comm_time: np.ndarray      # int32 [batch, n_buckets]
    drop_time: np.ndarray      # int32 [batch, n_buckets]
    forward_time: np.ndarray   # int32 [batch]
    backward_time: np.ndarray  # int32 [batch]


def random_schedules(seed: int, batch: int, n: int, iterations: int, w_hi: int, t_hi: int, f_hi: int,
                     b_hi: int) -> ScheduleBatch:
    r = _rng(seed)
    return ScheduleBatch(
        name=f"random_schedules_{seed}", batch=batch, n_buckets=n, iterations=iterations,
        comm_time=_i32(r.integers(1, w_hi + 1, size=(batch, n))),
        drop_time=_i32(r.integers(0, t_hi + 1, size=(batch, n))),
        forward_time=_i32(r.integers(0, f_hi + 1, size=batch)),
        backward_time=_i32(r.integers(0, b_hi + 1, size=batch)))


def resnet101_schedules(batch: int = 1024, n: int = 314, iterations: int = 8,
                        seed: int = SEED_RESNET + 70) -> ScheduleBatch:
    """ResNet-101-shaped candidates: bucket times as resnet101_shaped (sum 24200 in 10 us
    units), backward window 11800 and forward window 5900, each +-10 % per candidate (Table
    I); leaving a bucket off Algorithm 1's list costs its share of the backward window."""
    r = _rng(seed)
    x = r.lognormal(mean=0.0, sigma=1.2, size=(batch, n))
    w = _rescale_to_sum(x, 24200.0)
    bwd = np.rint(11800.0 * r.uniform(0.9, 1.1, size=batch)).astype(np.int64)
    fwd = np.rint(5900.0 * r.uniform(0.9, 1.1, size=batch)).astype(np.int64)
    drop = np.rint(x / x.sum(axis=1, keepdims=True) * bwd[:, None]).astype(np.int64)
    return ScheduleBatch(name="resnet101_schedules", batch=batch, n_buckets=n, iterations=iterations,
                         comm_time=_i32(w), drop_time=_i32(drop), forward_time=_i32(fwd), backward_time=_i32(bwd))
