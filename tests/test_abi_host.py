"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before touching a
device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "deft_knapsack.h")
LIB = os.path.join(ROOT, "paper_2503_16815_amd", "libdeft_knapsack.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2503_16815_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(deft_knapsack_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"deft_knapsack_create", "deft_knapsack_solve_batch", "deft_knapsack_destroy"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None, name


def test_binding_struct_layouts_match_header():
    """The ctypes mirrors must have the field order and sizes the header states."""
    from paper_2503_16815_amd import binding as b   # imports torch, needs no GPU
    assert ctypes.sizeof(b.deft_knapsack_config_t) == 8 * 4
    assert [f[0] for f in b.deft_knapsack_config_t._fields_] == [
        "device", "max_batch", "max_items", "max_knapsacks", "max_capacity", "max_c1", "max_c2", "flags"]
    assert ctypes.sizeof(b.deft_knapsack_batch_t) == 4 * 4 + 13 * 8
    hdr = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    body = re.search(r"typedef struct \{([^}]*)\} deft_knapsack_batch_t;", hdr).group(1)
    fields = re.findall(r"\**\s*([a-z_0-9]+)\s*;", body)
    assert fields == [f[0] for f in b.deft_knapsack_batch_t._fields_]
    body = re.search(r"typedef struct \{([^}]*)\} deft_schedule_batch_t;", hdr).group(1)
    fields = re.findall(r"\**\s*([a-z_0-9]+)\s*;", body)
    assert fields == [f[0] for f in b.deft_schedule_batch_t._fields_]
    assert ctypes.sizeof(b.deft_schedule_batch_t) == 4 * 4 + 11 * 8
    for name in ("deft_knapsack_info_t", "deft_knapsack_profile_t", "deft_knapsack_config_t", "deft_knapsack_peaks_t"):
        body = re.search(r"typedef struct \{([^}]*)\} " + name + ";", hdr).group(1)
        fields = re.findall(r"\**\s*([a-z_0-9]+)\s*;", body)
        assert fields == [f[0] for f in getattr(b, name)._fields_], name
    assert set(b.EXPORTS) == set(declared_functions())


def test_status_strings(lib):
    lib.deft_knapsack_status_string.restype = ctypes.c_char_p
    names = [lib.deft_knapsack_status_string(i).decode() for i in range(6)]
    assert names == ["DEFT_OK", "DEFT_ERR_INVALID_ARG", "DEFT_ERR_LIMIT", "DEFT_ERR_OVERFLOW",
                     "DEFT_ERR_OOM", "DEFT_ERR_DEVICE"]
    assert lib.deft_knapsack_status_string(99).decode() == "DEFT_ERR_UNKNOWN"


def test_create_rejects_bad_configs_without_a_device(lib):
    from paper_2503_16815_amd.binding import deft_knapsack_config_t as Cfg
    h = ctypes.c_void_p()
    create = lib.deft_knapsack_create
    create.restype = ctypes.c_int
    create.argtypes = [ctypes.POINTER(Cfg), ctypes.POINTER(ctypes.c_void_p)]
    ok = dict(device=0, max_batch=4, max_items=8, max_knapsacks=2, max_capacity=100, max_c1=0, max_c2=0, flags=0)

    def rc(**kw):
        cfg = Cfg(**{**ok, **kw})
        r = create(ctypes.byref(cfg), ctypes.byref(h))
        assert not h.value
        return r

    assert create(None, ctypes.byref(h)) == 1
    assert create(ctypes.byref(Cfg(**ok)), None) == 1
    assert rc(flags=4) == 1                              # an unknown flag bit
    assert rc(flags=2, max_capacity=65536) == 2          # bit-set rows end at 65535 cells
    assert rc(flags=1, max_capacity=26624) == 2          # 16-bit rows end at 26623 cells
    assert rc(flags=1, max_capacity=0, max_c1=10, max_c2=10) == 2   # the flag needs the sequential layout
    assert rc(max_batch=0) == 1
    assert rc(max_items=0) == 1
    assert rc(max_knapsacks=0) == 1
    assert rc(max_capacity=-1) == 1
    assert rc(device=-1) == 1
    assert rc(max_capacity=0) == 1                       # neither mode enabled
    assert rc(max_capacity=0, max_c1=10, max_c2=10, max_knapsacks=1) == 1   # joint needs 2 knapsacks
    assert rc(max_items=1 << 20) == 2
    assert rc(max_knapsacks=65) == 2
    assert rc(max_capacity=(1 << 24) + 1) == 2
    assert rc(max_capacity=0, max_c1=5000, max_c2=10) == 2
    assert rc(max_batch=(1 << 20) + 1) == 2


def test_solve_and_misc_reject_null_handles(lib):
    lib.deft_knapsack_solve_batch.restype = ctypes.c_int
    lib.deft_knapsack_solve_batch.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.deft_knapsack_solve_batch(None, None) == 1
    lib.deft_knapsack_get_info.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.deft_knapsack_get_info(None, None) == 1
    lib.deft_knapsack_set_profiling.argtypes = [ctypes.c_void_p, ctypes.c_int32]
    assert lib.deft_knapsack_set_profiling(None, 1) == 1
    lib.deft_knapsack_get_profile.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.deft_knapsack_get_profile(None, None) == 1
    lib.deft_knapsack_destroy.argtypes = [ctypes.c_void_p]
    lib.deft_knapsack_destroy(None)                      # NULL-safe
    lib.deft_knapsack_solve_batch_static.restype = ctypes.c_int
    lib.deft_knapsack_solve_batch_static.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    assert lib.deft_knapsack_solve_batch_static(0, 100, None) == 1
    lib.deft_knapsack_measure_peaks.restype = ctypes.c_int
    lib.deft_knapsack_measure_peaks.argtypes = [ctypes.c_int32, ctypes.c_void_p]
    assert lib.deft_knapsack_measure_peaks(0, None) == 1


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
