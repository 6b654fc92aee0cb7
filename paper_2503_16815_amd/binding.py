"""Thin Python binding of include/deft_knapsack.h (argument marshalling only).

Every step of the solve runs in the HIP library; PyTorch supplies device memory
and streams.  There is no CPU fallback: if the library is missing or the device
is not a gfx950, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DEFT_KNAPSACK_LIB") or os.path.join(_HERE, "libdeft_knapsack.so")

DEFT_OK, DEFT_ERR_INVALID_ARG, DEFT_ERR_LIMIT, DEFT_ERR_OVERFLOW, DEFT_ERR_OOM, DEFT_ERR_DEVICE = range(6)
(DEFT_MODE_SEQUENTIAL, DEFT_MODE_JOINT2, DEFT_MODE_RECURSIVE, DEFT_MODE_GREEDY, DEFT_MODE_GREEDY2,
 DEFT_MODE_CAPACITY_SWEEP) = range(6)

EXPORTS = ("deft_knapsack_create", "deft_knapsack_solve_batch", "deft_knapsack_destroy",
           "deft_knapsack_get_info", "deft_knapsack_set_profiling", "deft_knapsack_get_profile",
           "deft_knapsack_status_string", "deft_knapsack_simulate_schedule",
           "deft_knapsack_solve_batch_static", "deft_knapsack_measure_peaks")
STATIC_SCRATCH_BYTES = 64 * 1024 * 1024
FLAG_VALUES_ARE_WEIGHTS = 1
FLAG_SUBSET_SUM = 2


class deft_knapsack_config_t(ctypes.Structure):
    _fields_ = [("device", ctypes.c_int32), ("max_batch", ctypes.c_int32), ("max_items", ctypes.c_int32),
                ("max_knapsacks", ctypes.c_int32), ("max_capacity", ctypes.c_int32),
                ("max_c1", ctypes.c_int32), ("max_c2", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class deft_knapsack_batch_t(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("batch", ctypes.c_int32), ("item_stride", ctypes.c_int32),
                ("knap_stride", ctypes.c_int32),
                ("n_items", ctypes.c_void_p), ("n_knapsacks", ctypes.c_void_p), ("weights", ctypes.c_void_p),
                ("values", ctypes.c_void_p), ("capacities", ctypes.c_void_p), ("fill_order", ctypes.c_void_p),
                ("total_value", ctypes.c_void_p), ("knap_value", ctypes.c_void_p),
                ("knap_load", ctypes.c_void_p), ("assignment", ctypes.c_void_p), ("status", ctypes.c_void_p),
                ("stream", ctypes.c_void_p), ("drop_time", ctypes.c_void_p)]


class deft_schedule_batch_t(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_buckets", ctypes.c_int32), ("iterations", ctypes.c_int32),
                ("comm_time", ctypes.c_void_p), ("drop_time", ctypes.c_void_p), ("forward_time", ctypes.c_void_p),
                ("backward_time", ctypes.c_void_p), ("stage_case", ctypes.c_void_p),
                ("stage_count", ctypes.c_void_p), ("stage_time", ctypes.c_void_p), ("update_k", ctypes.c_void_p),
                ("tail", ctypes.c_void_p), ("status", ctypes.c_void_p), ("stream", ctypes.c_void_p)]


class deft_knapsack_info_t(ctypes.Structure):
    _fields_ = [("scratch_bytes", ctypes.c_int64), ("seq_path", ctypes.c_int32), ("seq_threads", ctypes.c_int32),
                ("seq_cells_per_thread", ctypes.c_int32), ("seq_lds_bytes", ctypes.c_int32),
                ("seq_workgroups_per_cu", ctypes.c_int32), ("joint_path", ctypes.c_int32),
                ("compute_units", ctypes.c_int32)]


class deft_knapsack_profile_t(ctypes.Structure):
    _fields_ = [("total_ms", ctypes.c_float), ("sweep_ms", ctypes.c_float), ("sweep_launches", ctypes.c_int32),
                ("other_ms", ctypes.c_float), ("streamed_row_cells", ctypes.c_int64),
                ("swept_cell_updates", ctypes.c_int64)]


class deft_knapsack_peaks_t(ctypes.Structure):
    _fields_ = [("lds_read_gbs", ctypes.c_float), ("lds_read_write_gbs", ctypes.c_float),
                ("hbm_copy_gbs", ctypes.c_float), ("hbm_read_gbs", ctypes.c_float),
                ("hbm_write_gbs", ctypes.c_float),
                ("compute_units", ctypes.c_int32), ("clock_mhz_reported", ctypes.c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree library and declare the C signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2503_16815_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp = ctypes.c_void_p
    lib.deft_knapsack_create.restype = ctypes.c_int
    lib.deft_knapsack_create.argtypes = [ctypes.POINTER(deft_knapsack_config_t), ctypes.POINTER(vp)]
    lib.deft_knapsack_solve_batch.restype = ctypes.c_int
    lib.deft_knapsack_solve_batch.argtypes = [vp, ctypes.POINTER(deft_knapsack_batch_t)]
    lib.deft_knapsack_destroy.restype = None
    lib.deft_knapsack_destroy.argtypes = [vp]
    lib.deft_knapsack_get_info.restype = ctypes.c_int
    lib.deft_knapsack_get_info.argtypes = [vp, ctypes.POINTER(deft_knapsack_info_t)]
    lib.deft_knapsack_set_profiling.restype = ctypes.c_int
    lib.deft_knapsack_set_profiling.argtypes = [vp, ctypes.c_int32]
    lib.deft_knapsack_get_profile.restype = ctypes.c_int
    lib.deft_knapsack_get_profile.argtypes = [vp, ctypes.POINTER(deft_knapsack_profile_t)]
    lib.deft_knapsack_simulate_schedule.restype = ctypes.c_int
    lib.deft_knapsack_simulate_schedule.argtypes = [vp, ctypes.POINTER(deft_schedule_batch_t)]
    lib.deft_knapsack_solve_batch_static.restype = ctypes.c_int
    lib.deft_knapsack_solve_batch_static.argtypes = [ctypes.c_int32, ctypes.c_int32,
                                                     ctypes.POINTER(deft_knapsack_batch_t)]
    lib.deft_knapsack_measure_peaks.restype = ctypes.c_int
    lib.deft_knapsack_measure_peaks.argtypes = [ctypes.c_int32, ctypes.POINTER(deft_knapsack_peaks_t)]
    lib.deft_knapsack_status_string.restype = ctypes.c_char_p
    lib.deft_knapsack_status_string.argtypes = [ctypes.c_int32]
    _lib = lib
    return lib


class DeftError(RuntimeError):
    def __init__(self, where: str, code: int):
        self.code = code
        name = load_library().deft_knapsack_status_string(code).decode()
        super().__init__(f"{where}: {name} ({code})")


@dataclass
class SolveOutputs:
    total_value: torch.Tensor  # int64 [batch]
    knap_value: torch.Tensor   # int32 [batch, knap_stride]
    knap_load: torch.Tensor    # int32 [batch, knap_stride]
    assignment: torch.Tensor   # int32 [batch, item_stride]
    status: torch.Tensor       # int32 [batch]


def _dev_i32(x, device) -> torch.Tensor:
    if isinstance(x, torch.Tensor):
        t = x
    else:
        t = torch.from_numpy(x)
    t = t.to(device=device, dtype=torch.int32).contiguous()
    return t


class DeviceBatch:
    """Inputs of one call resident on the device, outputs pre-allocated."""

    def __init__(self, kb, device: torch.device):
        self.mode, self.batch = int(kb.mode), int(kb.batch)
        self.item_stride, self.knap_stride = int(kb.item_stride), int(kb.knap_stride)
        self.n_items = _dev_i32(kb.n_items, device)
        self.n_knapsacks = _dev_i32(kb.n_knapsacks, device)
        self.weights = _dev_i32(kb.weights, device)
        self.values = _dev_i32(kb.values, device)
        self.capacities = _dev_i32(kb.capacities, device)
        self.fill_order = None if kb.fill_order is None else _dev_i32(kb.fill_order, device)
        drop = getattr(kb, "drop_time", None)
        self.drop_time = None if drop is None else _dev_i32(drop, device)
        B, IS, KS = self.batch, self.item_stride, self.knap_stride
        self.out = SolveOutputs(
            total_value=torch.empty(B, dtype=torch.int64, device=device),
            knap_value=torch.empty((B, KS), dtype=torch.int32, device=device),
            knap_load=torch.empty((B, KS), dtype=torch.int32, device=device),
            assignment=torch.empty((B, IS), dtype=torch.int32, device=device),
            status=torch.empty(B, dtype=torch.int32, device=device))

    def c_struct(self, stream_handle: int) -> deft_knapsack_batch_t:
        o = self.out
        p = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
        return deft_knapsack_batch_t(
            self.mode, self.batch, self.item_stride, self.knap_stride,
            p(self.n_items), p(self.n_knapsacks), p(self.weights), p(self.values), p(self.capacities),
            p(self.fill_order), p(o.total_value), p(o.knap_value), p(o.knap_load), p(o.assignment),
            p(o.status), ctypes.c_void_p(stream_handle), p(self.drop_time))


class DeftKnapsack:
    """Owner of one deft_knapsack_t handle."""

    def __init__(self, max_batch: int, max_items: int, max_knapsacks: int, max_capacity: int = 0,
                 max_c1: int = 0, max_c2: int = 0, device: int = 0, flags: int = 0):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.device = torch.device("cuda", device)
        cfg = deft_knapsack_config_t(device, max_batch, max_items, max_knapsacks, max_capacity, max_c1,
                                     max_c2, flags)
        rc = self._lib.deft_knapsack_create(ctypes.byref(cfg), ctypes.byref(self._h))
        if rc != DEFT_OK:
            self._h = ctypes.c_void_p()
            raise DeftError("deft_knapsack_create", rc)

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.deft_knapsack_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = close

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def info(self) -> deft_knapsack_info_t:
        info = deft_knapsack_info_t()
        rc = self._lib.deft_knapsack_get_info(self._h, ctypes.byref(info))
        if rc != DEFT_OK:
            raise DeftError("deft_knapsack_get_info", rc)
        return info

    def set_profiling(self, enable: bool) -> None:
        rc = self._lib.deft_knapsack_set_profiling(self._h, int(enable))
        if rc != DEFT_OK:
            raise DeftError("deft_knapsack_set_profiling", rc)

    def get_profile(self) -> deft_knapsack_profile_t:
        prof = deft_knapsack_profile_t()
        rc = self._lib.deft_knapsack_get_profile(self._h, ctypes.byref(prof))
        if rc != DEFT_OK:
            raise DeftError("deft_knapsack_get_profile", rc)
        return prof

    def upload(self, kb) -> DeviceBatch:
        return DeviceBatch(kb, self.device)

    def solve_batch(self, db: DeviceBatch, stream: Optional[torch.cuda.Stream] = None) -> SolveOutputs:
        """Enqueue one solve on `stream` (default: torch's current stream)."""
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        cs = db.c_struct(stream.cuda_stream)
        rc = self._lib.deft_knapsack_solve_batch(self._h, ctypes.byref(cs))
        if rc != DEFT_OK:
            raise DeftError("deft_knapsack_solve_batch", rc)
        return db.out


@dataclass
class ScheduleOutputs:
    stage_case: torch.Tensor   # int32 [batch, iterations, 2]
    stage_count: torch.Tensor  # int32 [batch, iterations, 2]
    stage_time: torch.Tensor   # int32 [batch, iterations, 2]
    update_k: torch.Tensor     # int32 [batch, iterations]
    tail: torch.Tensor         # int32 [batch, 2]
    status: torch.Tensor       # int32 [batch]


class DeviceSchedules:
    """Inputs of one simulation call resident on the device, outputs pre-allocated."""

    def __init__(self, sb, device: torch.device):
        self.batch, self.n_buckets, self.iterations = int(sb.batch), int(sb.n_buckets), int(sb.iterations)
        self.comm_time = _dev_i32(sb.comm_time, device)
        self.drop_time = _dev_i32(sb.drop_time, device)
        self.forward_time = _dev_i32(sb.forward_time, device)
        self.backward_time = _dev_i32(sb.backward_time, device)
        B, I = self.batch, self.iterations
        e = lambda *shape: torch.empty(shape, dtype=torch.int32, device=device)
        self.out = ScheduleOutputs(e(B, I, 2), e(B, I, 2), e(B, I, 2), e(B, I), e(B, 2), e(B))

    def c_struct(self, stream_handle: int) -> deft_schedule_batch_t:
        o = self.out
        p = lambda t: ctypes.c_void_p(t.data_ptr())
        return deft_schedule_batch_t(
            self.batch, self.n_buckets, self.iterations, p(self.comm_time), p(self.drop_time),
            p(self.forward_time), p(self.backward_time), p(o.stage_case), p(o.stage_count), p(o.stage_time),
            p(o.update_k), p(o.tail), p(o.status), ctypes.c_void_p(stream_handle))


def simulate_schedule(h: "DeftKnapsack", ds: DeviceSchedules,
                      stream: Optional[torch.cuda.Stream] = None) -> ScheduleOutputs:
    """Enqueue one task-queue simulation on `stream` (default: torch's current stream)."""
    if stream is None:
        stream = torch.cuda.current_stream(h.device)
    cs = ds.c_struct(stream.cuda_stream)
    rc = h._lib.deft_knapsack_simulate_schedule(h._h, ctypes.byref(cs))
    if rc != DEFT_OK:
        raise DeftError("deft_knapsack_simulate_schedule", rc)
    return ds.out


def measure_peaks(device: int = 0) -> deft_knapsack_peaks_t:
    """LDS and HBM rates measured by the library's calibration kernels."""
    peaks = deft_knapsack_peaks_t()
    rc = load_library().deft_knapsack_measure_peaks(device, ctypes.byref(peaks))
    if rc != DEFT_OK:
        raise DeftError("deft_knapsack_measure_peaks", rc)
    return peaks


def solve_batch_static(db: DeviceBatch, max_capacity: int, device: int = 0,
                       stream: Optional[torch.cuda.Stream] = None) -> SolveOutputs:
    """Enqueue one sequential-mode solve through the entry point that allocates nothing
    (no handle; the library's built-in scratch array)."""
    if stream is None:
        stream = torch.cuda.current_stream(torch.device("cuda", device))
    cs = db.c_struct(stream.cuda_stream)
    rc = load_library().deft_knapsack_solve_batch_static(device, max_capacity, ctypes.byref(cs))
    if rc != DEFT_OK:
        raise DeftError("deft_knapsack_solve_batch_static", rc)
    return db.out


def solve(kb, device: int = 0, **limits) -> SolveOutputs:
    """Convenience: create a handle sized for `kb`, solve, synchronise, destroy."""
    seq = kb.mode not in (DEFT_MODE_JOINT2, DEFT_MODE_GREEDY2)
    cap = int(kb.capacities.max()) if kb.capacities.size else 1
    args = dict(max_batch=max(1, kb.batch), max_items=kb.item_stride, max_knapsacks=kb.knap_stride,
                max_capacity=max(1, cap) if seq else 0,
                max_c1=0 if seq else max(1, int(kb.capacities[:, 0].max())),
                max_c2=0 if seq else max(1, int(kb.capacities[:, 1].max())), device=device)
    args.update(limits)
    with DeftKnapsack(**args) as h:
        out = h.solve_batch(h.upload(kb))
        torch.cuda.synchronize(h.device)
        return out
