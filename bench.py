#!/usr/bin/env python3
"""Throughput of the batched knapsack solver on one MI355X.

A step is one pass of the whole hot path (validation, every stage's DP sweep,
keep-table stream, traceback, outputs) over one synthetic batch resident in
HBM.  Prints ONE JSON line: DP cell-updates/s (the cell-updates the kernels
evaluate; the job's count as the CPU oracle performs it is beside it),
instances/s, the LDS roofline of the sweep kernel from HIP events on the launch
stream, and the CPU oracle timed on this machine's host cores.  The default run
(ResNet-101 shape) also measures, in the same process, every other
configuration (`per_config`) and the device's LDS / HBM rates (`peaks`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X figures used for the rooflines
N_CU = 256
CLOCK_HZ = 2.4e9
LDS_BYTES_PER_CLK_PER_CU = 128
PEAK_LDS_GBS = N_CU * LDS_BYTES_PER_CLK_PER_CU * CLOCK_HZ / 1e9      # 78643 GB/s
PEAK_INT_LANE_OPS = N_CU * 64 * CLOCK_HZ                              # 39.3e12 int32 lane-ops/s
PEAK_HBM_GBS = 8000.0


def cells_not_swept(kb, ref, lds_path: bool, enumerate_small: bool = True, check_every: int = 8):
    """Touched cells (as the oracle counts them) that the solver never evaluates, for a
    sequential-mode batch; returns (settled, full):
    settled - stages settled without a DP sweep: the offered items (not placed by an earlier
        stage, w <= C) all fit together, or (LDS-row path only) number at most six;
    full    - (LDS-row path, instances whose values all equal their weights) the items of a swept
        stage that come after the capacity itself is reached: after every eighth offered item
        (every second one when at most 64 are offered) the solver checks whether the sum C can be reached and ends the stage's sweep if so (the
        value is final and the walk back from C takes none of the later items).  Replayed here
        with the subset-sum bit recurrence on Python integers; `check_every` = 1 for the bit-set
        kernel, which looks after every item.
    The oracle's assignment says which stage placed what."""
    if kb.mode != 0:
        return 0, 0
    n = np.arange(kb.item_stride)[None, :] < kb.n_items[:, None]
    m = kb.n_knapsacks
    order = kb.fill_order if kb.fill_order is not None else np.tile(np.arange(kb.knap_stride), (kb.batch, 1))
    placed = np.zeros((kb.batch, kb.item_stride), bool)
    w = kb.weights.astype(np.int64)
    veqw = ((kb.weights == kb.values) | ~n).all(axis=1)
    settled = full = 0
    rows = np.arange(kb.batch)
    for s in range(kb.knap_stride):
        live = (s < m) & (ref.status == 0)
        j = order[:, s]
        cap = kb.capacities[rows, j].astype(np.int64)[:, None]
        offered = n & ~placed & (w <= cap) & live[:, None]
        fits = (w * offered).sum(axis=1) <= cap[:, 0]
        if lds_path and enumerate_small:
            fits |= offered.sum(axis=1) <= 6
        settled += int((np.maximum(cap - w + 1, 0) * offered)[fits].sum())
        if lds_path:
            for b in np.flatnonzero(~fits & veqw & live):
                C = int(cap[b, 0])
                goal = (1 << (C + 1)) - 1
                bits = 1
                ws = w[b][offered[b]].tolist()
                every = check_every if check_every == 1 or len(ws) > 64 else 2
                for q, wq in enumerate(ws):
                    bits |= bits << wq
                    bits &= goal
                    if q % every == every - 1 and (bits >> C) & 1:
                        full += sum(C - x + 1 for x in ws[q + 1:])
                        break
        placed |= (ref.assignment == j[:, None]) & live[:, None]
    return settled, full


def make_workload(name: str, batch_scale: float, per_k_calls: bool):
    from paper_2503_16815_amd import workloads as W
    sc = lambda b: max(1, int(round(b * batch_scale)))
    if name == "resnet101":
        if per_k_calls:
            calls = [W.resnet101_shaped(k=k, batch=sc(1024)) for k in (1, 2, 3, 4)]
            how = f"4 calls (k=1..4, m=2k), each batch {sc(1024)}"
        else:
            calls = [W.resnet101_sweep(batch=sc(1024))]
            how = f"one call of {4 * sc(1024)} candidate schedules = {sc(1024)} perturbed profiles x k=1..4 (m=2k)"
        desc = f"ResNet-101-shaped: {how}, n=314, windows 11800/5900 +-10%, v=w"
        algo = dict(bound="lds", bytes_per_cell=8.0, ops_per_cell=3.0)
    elif name == "vgg19":
        if per_k_calls:
            calls = [W.vgg19_shaped(k=k, batch=sc(4096)) for k in (1, 2, 3, 4)]
            how = f"4 calls (k=1..4, m=2k), each batch {sc(4096)}"
        else:
            calls = [W.vgg19_sweep(batch=sc(4096))]
            how = f"one call of {4 * sc(4096)} candidate schedules = {sc(4096)} profiles x k=1..4 (m=2k)"
        desc = f"VGG-19-shaped: {how}, n=38, windows 9300/3700, v=w"
        algo = dict(bound="lds", bytes_per_cell=8.0, ops_per_cell=3.0)
    elif name == "gpt2":
        calls = [W.gpt2_shaped(batch=sc(256))]
        desc = f"GPT-2-shaped: batch {sc(256)}, n=148, windows 381000/169000 (1 us units), v=w*U[1,4]"
        algo = dict(bound="hbm", bytes_per_cell=8.125, ops_per_cell=4.0)
    elif name == "hetero":
        calls = [W.hetero_joint(batch=sc(256))]
        desc = f"two-link joint DP: batch {sc(256)}, n=64, C1=C2=512"
        algo = dict(bound="hbm", bytes_per_cell=8.25, ops_per_cell=6.0)
    elif name == "backward":
        calls = [W.backward_stage_shaped(batch=sc(1024))]
        desc = (f"Algorithm 1 on ResNet-101-shaped backward stages: batch {sc(1024)}, n=314, remaining time "
                f"11800 +-10%, v=w, every level read off one sweep")
        algo = dict(bound="lds", bytes_per_cell=8.0, ops_per_cell=3.0)
    elif name == "inflation":
        calls = [W.inflation_sweep_shaped(batch=sc(1024))]
        desc = (f"capacity sweep on ResNet-101-shaped backward windows: batch {sc(1024)}, n=314, the window "
                f"(11800 +-10%) and ten inflations of +5% each, v=w, all read off one sweep at the largest")
        algo = dict(bound="lds", bytes_per_cell=8.0, ops_per_cell=3.0)
    elif name == "tiny":
        calls = [W.tiny_bruteforce(batch=sc(64))]
        desc = f"Tiny: batch {sc(64)}, n=16, capacities 500/250"
        algo = dict(bound="lds", bytes_per_cell=8.0, ops_per_cell=4.0)
    else:
        raise SystemExit(f"unknown workload {name}")
    return calls, desc, algo


def calibration_copy(dev) -> None:
    """One plain 1 GiB fill and one 1 GiB device-to-device copy: rows of known HBM traffic in a
    counter profile of this command, to scale FETCH_SIZE / WRITE_SIZE by."""
    import torch
    src = torch.empty(1 << 28, dtype=torch.int32, device=dev)
    src.fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize(dev)
    dst.copy_(src)            # the calibration row: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize(dev)
    del src, dst


def run_schedule(args):
    """The task-queue simulation (Sec. III.B, Cases 1-4) on the ResNet-101 shape: a step is one
    call simulating every candidate for 8 iterations (16 stages, each one solver launch).
    Returns (line, parity)."""
    import torch
    from oracle import oracle
    from paper_2503_16815_amd import binding, workloads as W

    sb = W.resnet101_schedules(batch=max(1, int(round(1024 * args.batch_scale))))
    cap = int(max(sb.backward_time.max(), sb.forward_time.max()))
    oracle.build()
    threads = min(os.cpu_count() or 1, 16)
    # the oracle's recursion costs n DPs per backward stage: it replays a sample of the candidates
    rows = np.arange(sb.batch) if args.batch_scale < 0.2 else np.linspace(0, sb.batch - 1, 96).astype(int)
    part = W.ScheduleBatch(name="sample", batch=len(rows), n_buckets=sb.n_buckets, iterations=sb.iterations,
                           comm_time=sb.comm_time[rows], drop_time=sb.drop_time[rows],
                           forward_time=sb.forward_time[rows], backward_time=sb.backward_time[rows])
    t0 = time.perf_counter()
    ref = oracle.simulate_batch(part, nthreads=threads)
    t_cpu = time.perf_counter() - t0
    dev = torch.device("cuda", 0)
    stream = torch.cuda.Stream(device=dev)
    packed16 = bool(getattr(args, "packed16", False))
    with binding.DeftKnapsack(device=0, max_batch=sb.batch, max_items=sb.n_buckets, max_knapsacks=2,
                              max_capacity=cap, flags=2 if getattr(args, "subset_sum", False) else 1 if packed16 else 0) as h:
        info = h.info()
        ds = binding.DeviceSchedules(sb, dev)
        torch.cuda.synchronize(dev)
        if getattr(args, "calibrate_copy", False):
            calibration_copy(dev)
        for _ in range(args.warmup):
            binding.simulate_schedule(h, ds, stream)
        stream.synchronize()
        h.set_profiling(True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            out = binding.simulate_schedule(h, ds, stream)
        stream.synchronize()
        t1 = time.perf_counter()
        prof = h.get_profile()
        got = {k: getattr(out, k).cpu().numpy() for k in ("stage_case", "stage_count", "stage_time", "update_k",
                                                          "tail", "status")}
    parity = all(np.array_equal(got[k][rows], getattr(ref, k)) for k in got)
    # cell-updates of the sweeps the solver runs: per stage, sum over the listed buckets of
    # max(0, window left - time + 1); the lists follow from the records, the oracle counts
    # them for its sample and the per-candidate mean is applied to the batch
    cells_step = float(ref.sweep_cells.mean()) * sb.batch
    ms_step = (t1 - t0) * 1e3 / args.steps
    sweep_s = float(prof.sweep_ms) * 1e-3
    launches = int(prof.sweep_launches)
    swept_step = int(prof.swept_cell_updates) // args.steps   # counted by the library: what the sweeps evaluated
    bitset = bool(getattr(args, "subset_sum", False))
    bytes_per_cell, ops_per_cell = (4.0, 1.75) if packed16 else (8.0, 3.0)
    if bitset:
        # every stage on the bit-set kernels, which count nothing: the one-sweep cells the oracle's
        # sample gives (what the int32 kernels would be offered), at the bit-set kernels' own 12 LDS
        # bytes and four vector instructions per 32 cells - for the record, the kernels are bound by latency
        swept_step = int(cells_step)
        bytes_per_cell, ops_per_cell = 0.375, 0.125
    achieved = swept_step * args.steps * bytes_per_cell / sweep_s / 1e9 if sweep_s > 0 else 0.0
    ops = swept_step * args.steps * ops_per_cell / sweep_s if sweep_s > 0 else 0.0
    upd = got["update_k"]
    line = dict(
        metric="knapsack DP cell-updates/sec", value=swept_step / (ms_step * 1e-3), unit="cell-updates/s", n_gpus=1,
        steps=args.steps, warmup=args.warmup, ms_per_step=ms_step, higher_is_better=True, scaling="weak",
        vs_baseline=None, dtype="int32", data="synthetic",
        config=dict(workload=f"task-queue simulation (Cases 1-4), ResNet-101-shaped: {sb.batch} candidates x "
                             f"{sb.n_buckets} buckets x {sb.iterations} iterations, windows 5900 / 11800 +-10%"
                             + (" [rows of 16-bit cells]" if packed16 else "")
                             + (" [bit-set rows; cell-updates as the oracle's sample counts them for one sweep per stage]"
                                if bitset else ""),
                    value_counts=("one-sweep cell-updates per stage as estimated from the oracle's sample (the bit-set "
                                  "kernels count none)" if bitset else
                                  "cell-updates the sweeps evaluate (counted by the library)"),
                    candidates_per_step=sb.batch, iterations=sb.iterations,
                    one_sweep_cell_updates_per_step_estimated_from_sample=cells_step,
                    cell_updates_swept_per_step=swept_step, seq_path=int(info.seq_path),
                    threads_per_instance=int(info.seq_threads), cells_per_thread=int(info.seq_cells_per_thread),
                    updates_per_iteration_mean=float((upd > 0).mean()),
                    buckets_per_iteration_mean=float(got["stage_count"].sum(axis=(1, 2)).mean() / sb.iterations)),
        candidate_iterations_per_s=sb.batch * sb.iterations / (ms_step * 1e-3), parity_vs_oracle=bool(parity),
        parity_checked=f"{len(rows)} of {sb.batch} candidates (every candidate: tests/test_gpu_schedule.py)",
        profile=dict(total_ms_per_step=float(prof.total_ms) / args.steps,
                     sweep_ms_per_step=float(prof.sweep_ms) / args.steps),
        roofline=dict(bound="lds", achieved=achieved, peak=PEAK_LDS_GBS, unit="GB/s", frac=achieved / PEAK_LDS_GBS,
                      traffic=None, kernel="seq_bits_kernel" if bitset else "seq_lds_kernel",
                      bytes_per_cell=bytes_per_cell, launches=launches,
                      avg_launch_ms=float(prof.sweep_ms) / max(launches, 1),
                      swept_cell_updates_per_s=swept_step * args.steps / sweep_s if sweep_s > 0 else 0.0,
                      alu=dict(ops_per_cell=ops_per_cell, peak_lane_ops_per_s=PEAK_INT_LANE_OPS,
                               frac=ops / PEAK_INT_LANE_OPS)),
        cpu_baseline=None if args.no_cpu else dict(
            value=float(ref.sweep_cells.sum()) / t_cpu, unit="cell-updates/s", cores=int(ref.threads), kind="oracle",
            sample=f"{len(rows)} of the {sb.batch} candidates, all {sb.iterations} iterations, {t_cpu:.2f} s wall "
                   f"(the oracle solves Algorithm 1 level by level; the figure counts the same one-sweep cells as "
                   f"the GPU line)",
            candidate_iterations_per_s=len(rows) * sb.iterations / t_cpu))
    return line, bool(parity)


def subset(kb, rows):
    """The instances `rows` of a batch (oracle sampling)."""
    from paper_2503_16815_amd import workloads as W
    pick = lambda a: None if a is None else np.ascontiguousarray(a[rows])
    return W.KnapsackBatch(name=f"{kb.name}[sample]", mode=kb.mode, batch=len(rows), item_stride=kb.item_stride,
                           knap_stride=kb.knap_stride, n_items=pick(kb.n_items), n_knapsacks=pick(kb.n_knapsacks),
                           weights=pick(kb.weights), values=pick(kb.values), capacities=pick(kb.capacities),
                           fill_order=pick(kb.fill_order), meta=dict(kb.meta), drop_time=pick(kb.drop_time))


def run_solver(args):
    """One workload through deft_knapsack_solve_batch.  Returns (line, parity)."""
    import torch
    from paper_2503_16815_amd import binding

    calls, desc, algo = make_workload(args.workload, args.batch_scale, args.per_k_calls or bool(args.only_k))
    if args.only_k:
        calls = [kb for kb in calls if kb.meta.get("k") == args.only_k]
        desc += f" [only k={args.only_k}]"
    if args.max_stages:
        for kb in calls:
            kb.n_knapsacks[:] = np.minimum(kb.n_knapsacks, args.max_stages)
        desc += f" [n_knapsacks clamped to {args.max_stages}]"
    plain_run = args.batch_scale == 1.0 and not (args.per_k_calls or args.only_k or args.max_stages or
                                                 getattr(args, "packed16", False) or getattr(args, "subset_sum", False))
    seq = calls[0].mode != 1
    cap = max(int(kb.capacities.max()) for kb in calls)
    limits = dict(max_batch=max(kb.batch for kb in calls), max_items=max(kb.item_stride for kb in calls),
                  max_knapsacks=max(kb.knap_stride for kb in calls))
    packed16 = bool(getattr(args, "packed16", False))
    if packed16:
        limits["flags"] = 1
        desc += " [rows of 16-bit cells]"
        # two 16-bit cells per LDS word and per packed instruction: 2 B read + 2 B written per cell
        # (LDS bound 128 B / 4 B = 32 cells per clock and CU); subtract and max per pair of cells,
        # permute + shift + bit-field insert per two pairs = 1.75 vector instructions per cell (ALU
        # bound 64 / 1.75 = 36.6; lanes below the item's shift add a byte permute per pair): LDS is
        # the nearer bound and the one the fraction is taken against
        algo = dict(bound="lds", bytes_per_cell=4.0, ops_per_cell=1.75)
    subset_sum = bool(getattr(args, "subset_sum", False))
    if subset_sum:
        limits["flags"] = 2
        desc += " [bit-set rows]"
        # one bit per cell: two 4-byte words read and one written per 32 cells, four vector instructions
        # per 32 cells; a latency-bound kernel (one wavefront per instance), stated against the LDS peak
        # at its own bytes for the record
        algo = dict(bound="lds", bytes_per_cell=0.375, ops_per_cell=0.125)
    if seq:
        limits["max_capacity"] = cap
    else:
        limits["max_c1"] = max(int(kb.capacities[:, 0].max()) for kb in calls)
        limits["max_c2"] = max(int(kb.capacities[:, 1].max()) for kb in calls)

    # ---- CPU oracle: cell counts for the metric, reference outputs, cpu_baseline
    from oracle import oracle
    oracle.build()
    threads = min(os.cpu_count() or 1, 16)
    cpu = None
    refs = []
    t_cpu = 0.0
    for kb in calls:
        t0 = time.perf_counter()
        refs.append(oracle.solve_batch(kb, nthreads=threads))
        t_cpu += time.perf_counter() - t0
    touched = [int(r.touched_cells.sum()) for r in refs]
    table = [int(r.table_cells.sum()) for r in refs]
    # The job's cell-updates are the oracle's count (touched cells of every stage).  The solver
    # does not evaluate all of them: stages it settles without a sweep and, where every value
    # equals its weight, the items after the capacity itself is reached.  `value` and the roofline are priced
    # on the cell-updates it does evaluate (swept_step); both counts are reported.
    not_swept = {path: [cells_not_swept(kb, r, path) for kb, r in zip(calls, refs)] for path in (False, True)}
    not_swept["bits"] = [cells_not_swept(kb, r, True, enumerate_small=False, check_every=1) for kb, r in zip(calls, refs)]
    settled = sum(x[0] for x in not_swept[True])     # corrected below once the handle says which path runs
    after_full = sum(x[1] for x in not_swept[True])
    cells_step = sum(touched)
    swept_step = cells_step - settled - after_full
    recursion_cells = None
    if calls[0].mode in (2, 5):
        # Algorithm 1 / capacity sweep: the oracle runs one DP per level / per capacity and counts
        # them all; the solver does one sweep over the whole list at the full remaining time / the
        # largest capacity, and that is what the metric counts
        recursion_cells = cells_step
        cells_step = 0
        for kb in calls:
            live = np.arange(kb.item_stride)[None, :] < kb.n_items[:, None]
            top = kb.capacities[:, :1] if kb.mode == 2 else kb.capacities.max(axis=1, keepdims=True)
            room = top.astype(np.int64) - kb.weights + 1
            cells_step += int((np.maximum(room, 0) * live).sum())
        swept_step = cells_step
    inst_step = sum(kb.batch for kb in calls)
    if not args.no_cpu:
        cpu_cells = recursion_cells if recursion_cells is not None else sum(touched)   # the oracle sweeps every stage
        cpu = dict(value=cpu_cells / t_cpu, unit="cell-updates/s", cores=int(refs[0].threads), kind="oracle",
                   sample=f"the full step ({inst_step} instances, {cpu_cells} cell-updates performed), "
                          f"instances split statically over {int(refs[0].threads)} threads, {t_cpu:.2f} s wall",
                   instances_per_s=inst_step / t_cpu)
        if getattr(args, "single_thread", True):
            # one thread, on a bounded sample of the same step (a stride through the instances)
            per_inst = cpu_cells / max(inst_step, 1) / max(cpu["value"] / max(int(refs[0].threads), 1), 1.0)
            want = max(1, min(inst_step, int(4.0 / max(per_inst, 1e-9))))      # about four seconds of one core
            t1_cells, t1_time, t1_inst = 0, 0.0, 0
            for kb in calls:
                rows = np.unique(np.linspace(0, kb.batch - 1, max(1, want * kb.batch // inst_step)).astype(int))
                part = subset(kb, rows)
                t0 = time.perf_counter()
                r1 = oracle.solve_batch(part, nthreads=1)
                t1_time += time.perf_counter() - t0
                t1_cells += int(r1.touched_cells.sum())
                t1_inst += len(rows)
            cpu["single_thread"] = dict(value=t1_cells / t1_time, unit="cell-updates/s", cores=1,
                                        sample=f"{t1_inst} of the {inst_step} instances (evenly strided), "
                                               f"{t1_cells} cell-updates, {t1_time:.2f} s wall",
                                        instances_per_s=t1_inst / t1_time)

    # ---- GPU
    dev = torch.device("cuda", 0)
    stream = torch.cuda.Stream(device=dev)
    with binding.DeftKnapsack(device=0, **limits) as h:
        info = h.info()
        if seq and calls[0].mode == 0:
            rules = "bits" if info.seq_path == 4 else info.seq_path in (1, 2)
            settled = sum(x[0] for x in not_swept[rules])
            after_full = sum(x[1] for x in not_swept[rules])
            swept_step = cells_step - settled - after_full
        dbs = [h.upload(kb) for kb in calls]
        torch.cuda.synchronize(dev)

        def step():
            for db in dbs:
                h.solve_batch(db, stream)

        if args.calibrate_copy:
            calibration_copy(dev)
        for _ in range(args.warmup):
            step()
        stream.synchronize()
        torch.cuda.synchronize(dev)
        h.set_profiling(True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        stream.synchronize()
        torch.cuda.synchronize(dev)
        t1 = time.perf_counter()
        prof = h.get_profile()
        h.set_profiling(False)

        parity = True
        for db, ref in zip(dbs, refs):
            o = db.out
            parity &= bool(np.array_equal(o.status.cpu().numpy(), ref.status))
            parity &= bool(np.array_equal(o.total_value.cpu().numpy(), ref.total_value))
            parity &= bool(np.array_equal(o.knap_value.cpu().numpy(), ref.knap_value))
            parity &= bool(np.array_equal(o.knap_load.cpu().numpy(), ref.knap_load))
            parity &= bool(np.array_equal(o.assignment.cpu().numpy(), ref.assignment))

    ms_step = (t1 - t0) * 1e3 / args.steps
    # rows in LDS: the library counts the cell-updates its sweeps evaluated (C - w + 1 per swept
    # item); value and roofline are priced on that count.  For the sequential mode the same number
    # follows from the oracle's results and the two rules (swept_step above): both are reported.
    replayed_swept = swept_step
    counted_swept = int(prof.swept_cell_updates) // args.steps if seq and info.seq_path in (1, 2) else None
    if counted_swept is not None:
        swept_step = counted_swept
    value = swept_step / (ms_step * 1e-3)
    launches = int(prof.sweep_launches)
    sweep_s = float(prof.sweep_ms) * 1e-3
    algo_bytes_total = swept_step * args.steps * algo["bytes_per_cell"]
    if seq and info.seq_path == 3 and int(prof.streamed_row_cells) > 0:
        # rows in global memory: a pass over a row (4 B read + 4 B written per cell) may serve two
        # items; the library counts the row cells it read and wrote, the keep stream is 1/8 B per
        # cell-update
        algo_bytes_total = int(prof.streamed_row_cells) * 4.0 + swept_step * args.steps / 8.0
        algo = dict(algo, bytes_per_cell=algo_bytes_total / (swept_step * args.steps))
    achieved_gbs = algo_bytes_total / sweep_s / 1e9 if sweep_s > 0 else 0.0
    peak = PEAK_HBM_GBS if algo["bound"] == "hbm" else PEAK_LDS_GBS
    # HBM bytes per launch of the dominant kernel: NOT measured in this run, read from the
    # committed rocprofv3 counter passes of this same command (FETCH_SIZE and WRITE_SIZE scaled
    # by a copy of known size); only for the unmodified workload.
    traffic = traffic_source = None
    kernel = ("seq_bits_kernel" if (seq and info.seq_path == 4 and calls[0].mode in (0, 2, 5)) else
              "seq_lds_kernel" if (seq and info.seq_path in (1, 2, 4)) else ("sg_sweep_all" if seq else "jt_sweep_all"))
    tf = os.path.join(ROOT, "profiles", f"{kernel}_{args.workload}_traffic.txt")
    if plain_run and os.path.exists(tf):
        try:
            with open(tf) as f:
                traffic = float(json.load(f)["hbm_bytes_per_launch"])
            traffic_source = (f"profiles/{os.path.basename(tf)}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes of this "
                              f"command, committed; not measured in this run")
        except (ValueError, KeyError):
            traffic = None
    roofline = dict(
        bound=algo["bound"], achieved=achieved_gbs, peak=peak, unit="GB/s", frac=achieved_gbs / peak,
        traffic=traffic, traffic_source=traffic_source,
        kernel=kernel,
        bytes_per_cell=algo["bytes_per_cell"], launches=launches,
        avg_launch_ms=float(prof.sweep_ms) / max(launches, 1),
        algorithmic_bytes_per_launch=algo_bytes_total / max(launches, 1),
        swept_cell_updates_per_s=swept_step * args.steps / sweep_s if sweep_s > 0 else 0.0,
        alu=dict(ops_per_cell=algo["ops_per_cell"], peak_lane_ops_per_s=PEAK_INT_LANE_OPS,
                 frac=(swept_step * args.steps * algo["ops_per_cell"] / sweep_s) / PEAK_INT_LANE_OPS
                 if sweep_s > 0 else 0.0))
    if not seq:
        # the table streams from HBM (the bound above); the LDS side of the same kernel, for the
        # record: two shifted reads and one write per cell
        roofline["lds"] = dict(bytes_per_cell=12.0, peak=PEAK_LDS_GBS,
                               frac=(swept_step * args.steps * 12.0 / sweep_s / 1e9) / PEAK_LDS_GBS if sweep_s > 0 else 0.0)
    line = dict(
        metric="knapsack DP cell-updates/sec", value=value, unit="cell-updates/s", n_gpus=1,
        steps=args.steps, warmup=args.warmup, ms_per_step=ms_step, higher_is_better=True, scaling="weak",
        vs_baseline=None, dtype="int32", data="synthetic",
        config=dict(workload=desc,
                    value_counts="cell-updates the kernels evaluate (cell_updates_swept_per_step); the job as the "
                                 "oracle performs it holds cell_updates_per_step, see effective_cell_updates_per_s",
                    instances_per_step=inst_step, cell_updates_per_step=cells_step,
                    cell_updates_swept_per_step=swept_step,
                    cell_updates_swept_per_step_replayed_from_oracle=replayed_swept if calls[0].mode == 0 else None,
                    table_cells_per_step=sum(table), seq_path=int(info.seq_path),
                    threads_per_instance=int(info.seq_threads), cells_per_thread=int(info.seq_cells_per_thread),
                    lds_bytes_per_workgroup=int(info.seq_lds_bytes),
                    workgroups_per_cu=int(info.seq_workgroups_per_cu), scratch_bytes=int(info.scratch_bytes),
                    oracle_cell_updates_of_stages_settled_without_sweep=settled,
                    oracle_cell_updates_after_the_capacity_is_reached=after_full,
                    oracle_recursion_cell_updates_per_step=recursion_cells),
        effective_cell_updates_per_s=cells_step / (ms_step * 1e-3),
        instances_per_s=inst_step / (ms_step * 1e-3), parity_vs_oracle=parity,
        profile=dict(total_ms_per_step=float(prof.total_ms) / args.steps,
                     sweep_ms_per_step=float(prof.sweep_ms) / args.steps),
        roofline=roofline, cpu_baseline=cpu)
    return line, parity


def compact(line: dict) -> dict:
    """The per-configuration record of the default run."""
    r = line["roofline"]
    out = dict(workload=line["config"]["workload"], steps=line["steps"], ms_per_step=line["ms_per_step"],
               cell_updates_evaluated_per_step=line["config"]["cell_updates_swept_per_step"],
               value=line["value"], unit=line["unit"],
               kernel=r["kernel"], kernel_launches_per_step=r["launches"] / max(line["steps"], 1),
               kernel_ms_per_step=line["profile"]["sweep_ms_per_step"],
               roofline=dict(bound=r["bound"], bytes_per_cell=r["bytes_per_cell"], achieved=r["achieved"], peak=r["peak"],
                             unit=r["unit"], frac=r["frac"], alu_frac=r["alu"]["frac"],
                             alu_ops_per_cell=r["alu"]["ops_per_cell"]),
               parity_vs_oracle=line["parity_vs_oracle"])
    if "lds" in r:
        out["roofline"][f"lds_frac_at_{r['lds']['bytes_per_cell']:g}_bytes_per_cell"] = r["lds"]["frac"]
    for key in ("instances_per_s", "candidate_iterations_per_s", "effective_cell_updates_per_s", "parity_checked"):
        if key in line:
            out[key] = line[key]
    if line.get("cpu_baseline"):
        out["cpu_baseline"] = {k: line["cpu_baseline"][k] for k in ("value", "unit", "cores", "sample")}
    return out


def measured_peaks() -> dict:
    """Nominal peaks used for the rooflines beside what the library's calibration kernels reach
    on this device (LDS: the sweep's access mix; HBM: a 1 GiB copy)."""
    from paper_2503_16815_amd import binding
    p = binding.measure_peaks(0)
    return dict(
        nominal=dict(lds_gbs=PEAK_LDS_GBS, hbm_gbs=PEAK_HBM_GBS, int32_lane_ops_per_s=PEAK_INT_LANE_OPS,
                     basis=f"{N_CU} CUs x {LDS_BYTES_PER_CLK_PER_CU} B/clk/CU x {CLOCK_HZ / 1e9} GHz; HBM3E 8 TB/s; "
                           f"{N_CU} CUs x 64 lanes x {CLOCK_HZ / 1e9} GHz"),
        measured=dict(lds_read_gbs=float(p.lds_read_gbs), lds_read_write_gbs=float(p.lds_read_write_gbs),
                      hbm_copy_gbs=float(p.hbm_copy_gbs), hbm_read_gbs=float(p.hbm_read_gbs),
                      hbm_write_gbs=float(p.hbm_write_gbs),
                      lds_read_write_bytes_per_clk_per_cu_at_nominal_clock=float(p.lds_read_write_gbs) * 1e9 / CLOCK_HZ / N_CU,
                      compute_units=int(p.compute_units), clock_mhz_reported=int(p.clock_mhz_reported),
                      how="deft_knapsack_measure_peaks: 4-byte conflict-free LDS reads; one shifted 4-byte read + one "
                          "lane-addressed 4-byte write per cell; 1 GiB streaming copy, read and fill kernels (16-byte accesses, four "
                          "in flight per lane); best of three launches"))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet101",
                    choices=["resnet101", "vgg19", "gpt2", "hetero", "backward", "inflation", "schedule", "tiny"])
    ap.add_argument("--batch-scale", type=float, default=1.0, help="scale the batch (debug only)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg (profiling runs)")
    ap.add_argument("--per-k-calls", action="store_true",
                    help="ResNet/VGG shapes: one call per k (4 calls of 1024 / 4096 instances) instead of one call "
                         "holding the whole sweep over k")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel, so that a counter profile of this "
                         "command holds a row of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--no-per-config", "--no-per-k", dest="no_per_config", action="store_true",
                    help="default workload only: skip the other configurations and the peak calibration "
                         "(profiling runs: keeps the kernel statistics to the headline launches)")
    ap.add_argument("--packed16", action="store_true",
                    help="value-equals-weight workloads: create the handle with DEFT_FLAG_VALUES_ARE_WEIGHTS "
                         "(rows of 16-bit cells)")
    ap.add_argument("--subset-sum", action="store_true",
                    help="value-equals-weight workloads: create the handle with DEFT_FLAG_SUBSET_SUM (bit-set "
                         "rows, one wavefront per instance)")
    ap.add_argument("--max-stages", type=int, default=0, help="clamp n_knapsacks (debug only)")
    ap.add_argument("--only-k", type=int, default=0, help="keep only the call with this k (debug only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (instances are independent; sharding is by "
              "instance index and is not part of this build); use --gpus 1", file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    run = run_schedule if args.workload == "schedule" else run_solver
    line, parity = run(args)
    headline = (args.workload == "resnet101" and args.batch_scale == 1.0 and
                not (args.per_k_calls or args.only_k or args.max_stages or args.no_per_config))
    if headline:
        # every other configuration, measured in this same process, same code path
        per_config = {}
        for name, extra in (("tiny", {}), ("resnet101_one_call_per_k", dict(workload="resnet101", per_k_calls=True)),
                            ("vgg19", {}), ("gpt2", {}), ("hetero", {}), ("backward", {}), ("inflation", {}),
                            ("schedule", {}),
                            # the value-equals-weight workloads again on handles created with
                            # DEFT_FLAG_VALUES_ARE_WEIGHTS (rows of 16-bit cells), priced on their own roofline
                            # (4 LDS bytes per cell instead of 8)
                            ("resnet101_rows16", dict(workload="resnet101", packed16=True)),
                            ("resnet101_one_call_per_k_rows16", dict(workload="resnet101", per_k_calls=True, packed16=True)),
                            ("vgg19_rows16", dict(workload="vgg19", packed16=True)),
                            ("backward_rows16", dict(workload="backward", packed16=True)),
                            ("inflation_rows16", dict(workload="inflation", packed16=True)),
                            ("schedule_rows16", dict(workload="schedule", packed16=True)),
                            # the value-equals-weight workloads on handles created with DEFT_FLAG_SUBSET_SUM
                            # (bit-set rows, one wavefront per instance)
                            ("resnet101_bitset", dict(workload="resnet101", subset_sum=True)),
                            ("resnet101_one_call_per_k_bitset", dict(workload="resnet101", per_k_calls=True, subset_sum=True)),
                            ("vgg19_bitset", dict(workload="vgg19", subset_sum=True)),
                            ("backward_bitset", dict(workload="backward", subset_sum=True)),
                            ("inflation_bitset", dict(workload="inflation", subset_sum=True)),
                            ("schedule_bitset", dict(workload="schedule", subset_sum=True))):
            sub = argparse.Namespace(**vars(args))
            sub.workload, sub.no_cpu = name, args.no_cpu or "rows16" in name or "bitset" in name
            sub.steps, sub.warmup, sub.single_thread = max(3, min(args.steps, 20)), 3, False
            for k, v in extra.items():
                setattr(sub, k, v)
            one, ok = (run_schedule if sub.workload == "schedule" else run_solver)(sub)
            per_config[name] = compact(one)
            if name == "tiny":
                per_config[name]["note"] = ("64 instances of 16 items on 256 compute units: the launch is latency "
                                            "(about 20 us), not throughput; the fraction says nothing here")
            parity = parity and ok
        line["per_config"] = per_config
        line["parity_vs_oracle_every_config"] = bool(parity)
        line["peaks"] = measured_peaks()
    print(json.dumps(line))
    return 0 if parity else 3


if __name__ == "__main__":
    sys.exit(main())
