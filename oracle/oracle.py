"""ctypes front end of the CPU oracle in deft_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg, never by the HIP product path.  It takes plain
numpy arrays (any object with the fields of a solver call: mode, batch,
item_stride, knap_stride, n_items, n_knapsacks, weights, values, capacities,
fill_order, and drop_time for the recursive mode) and imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "deft_oracle.c")
_LIB = os.path.join(_HERE, "libdeft_oracle.so")

ST_OK, ST_INVALID, ST_LIMIT, ST_OVERFLOW, ST_OOM = 0, 1, 2, 3, 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no tuning flags) into oracle/libdeft_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-pthread", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p32 = ctypes.POINTER(ctypes.c_int32)
        p64 = ctypes.POINTER(ctypes.c_int64)
        i32 = ctypes.c_int32
        lib.deft_oracle_solve_batch.restype = ctypes.c_int
        lib.deft_oracle_solve_batch.argtypes = [i32, i32, i32, i32, p32, p32, p32, p32, p32, p32, p32,
                                                i32, i32, i32, p64, p32, p32, p32, p32, p64, p64, i32]
        lib.deft_oracle_simulate_batch.restype = ctypes.c_int
        lib.deft_oracle_simulate_batch.argtypes = [i32, i32, i32, p32, p32, p32, p32, i32, p32, p32, p32, p32, p32,
                                                   p32, p64, i32]
        _lib = lib
    return _lib


@dataclass
class OracleResult:
    total_value: np.ndarray   # int64 [batch]
    knap_value: np.ndarray    # int32 [batch, knap_stride]
    knap_load: np.ndarray     # int32 [batch, knap_stride]
    assignment: np.ndarray    # int32 [batch, item_stride]
    status: np.ndarray        # int32 [batch]
    touched_cells: np.ndarray  # int64 [batch]  sum over stages/items of max(0, C - w + 1)
    table_cells: np.ndarray    # int64 [batch]  sum over stages of n_active * (C + 1)
    threads: int


def _p32(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _p64(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def solve_batch(kb, cap_limit: int = -1, c1_limit: int = -1, c2_limit: int = -1,
                nthreads: int = 1) -> OracleResult:
    lib = _load()
    B, IS, KS = int(kb.batch), int(kb.item_stride), int(kb.knap_stride)
    c = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    n_items, n_knap = c(kb.n_items), c(kb.n_knapsacks)
    w, v, cap = c(kb.weights), c(kb.values), c(kb.capacities)
    fo = None if kb.fill_order is None else c(kb.fill_order)
    dt = None if getattr(kb, "drop_time", None) is None else c(kb.drop_time)
    assert kb.mode != 2 or (dt is not None and dt.shape == (B, IS))
    assert n_items.shape == (B,) and n_knap.shape == (B,)
    assert v.shape == (B, IS) and cap.shape == (B, KS)
    assert w.shape == ((B, 2, IS) if kb.mode in (1, 4) else (B, IS))
    total = np.zeros(B, np.int64)
    kv = np.zeros((B, KS), np.int32)
    kl = np.zeros((B, KS), np.int32)
    asg = np.full((B, IS), -1, np.int32)
    st = np.zeros(B, np.int32)
    touched = np.zeros(B, np.int64)
    table = np.zeros(B, np.int64)
    used = lib.deft_oracle_solve_batch(
        kb.mode, B, IS, KS, _p32(n_items), _p32(n_knap), _p32(w), _p32(v), _p32(cap),
        None if fo is None else _p32(fo), None if dt is None else _p32(dt), cap_limit, c1_limit, c2_limit,
        _p64(total), _p32(kv), _p32(kl), _p32(asg), _p32(st), _p64(touched), _p64(table), nthreads)
    if used < 0:
        raise ValueError("oracle: bad batch arguments")
    return OracleResult(total, kv, kl, asg, st, touched, table, used)


@dataclass
class SimulationResult:
    stage_case: np.ndarray    # int32 [batch, iterations, 2]  0 = nothing to do, else Case 1..4
    stage_count: np.ndarray   # int32 [batch, iterations, 2]  buckets synchronised in the stage
    stage_time: np.ndarray    # int32 [batch, iterations, 2]  their communication time
    update_k: np.ndarray      # int32 [batch, iterations]     iterations of gradients applied at the end of t
    tail: np.ndarray          # int32 [batch, 2]              cur_k, fut_k after the last iteration
    status: np.ndarray        # int32 [batch]
    sweep_cells: np.ndarray   # int64 [batch]  sum over solved stages of sum_i max(0, capacity - comm_i + 1)
    threads: int


def simulate_batch(sb, cap_limit: int = -1, nthreads: int = 1) -> SimulationResult:
    """sb: any object with batch, n_buckets, iterations, comm_time [batch, n], drop_time [batch, n],
    forward_time [batch], backward_time [batch]."""
    lib = _load()
    B, n, I = int(sb.batch), int(sb.n_buckets), int(sb.iterations)
    c = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    comm, drop, fwd, bwd = c(sb.comm_time), c(sb.drop_time), c(sb.forward_time), c(sb.backward_time)
    assert comm.shape == (B, n) and drop.shape == (B, n) and fwd.shape == (B,) and bwd.shape == (B,)
    case = np.zeros((B, I, 2), np.int32)
    count = np.zeros((B, I, 2), np.int32)
    tim = np.zeros((B, I, 2), np.int32)
    upd = np.zeros((B, I), np.int32)
    tail = np.zeros((B, 2), np.int32)
    st = np.zeros(B, np.int32)
    cells = np.zeros(B, np.int64)
    used = lib.deft_oracle_simulate_batch(B, n, I, _p32(comm), _p32(drop), _p32(fwd), _p32(bwd), cap_limit,
                                          _p32(case), _p32(count), _p32(tim), _p32(upd), _p32(tail), _p32(st),
                                          _p64(cells), nthreads)
    if used < 0:
        raise ValueError("oracle: bad simulation arguments")
    return SimulationResult(case, count, tim, upd, tail, st, cells, used)
