"""Builds libdeft_knapsack.so (hipcc, gfx950 only) in-tree next to this file."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdeft_knapsack.so")
PKG = "paper_2503_16815_amd"
SOURCES = ["seq_lds.hip", "seq_lds_rec.hip", "seq_lds_p16.hip", "seq_lds_p16_rec.hip", "seq_bits.hip", "seq_bits_rec.hip", "joint2.hip", "seq_global.hip", "greedy.hip", "schedule_sim.hip", "api.hip", "profile.hip", "static_scratch.hip", "calibrate.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-command-line-argument", "-Wno-inline-asm"]


def _messages(res) -> str:
    return "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                     if "packed-fp32-ops" not in l and l.strip())


def build(verbose: bool = False) -> str:
    """Compiles every source to an object (all at once: the files are independent
    and the two sets of LDS kernels dominate) and links the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = tempfile.mkdtemp(prefix="deft_build_")
    try:
        jobs = []
        for src in SOURCES:
            obj = os.path.join(tmp, src + ".o")
            cmd = [hipcc, *FLAGS, "-c", "-o", obj, os.path.join(CSRC, src)]
            if verbose:
                print(" ".join(cmd), flush=True)
            jobs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
        objs = []
        for src, obj, proc in jobs:
            out, err = proc.communicate()
            res = subprocess.CompletedProcess(proc.args, proc.returncode, out, err)
            if res.returncode != 0:
                for _, _, other in jobs:
                    if other.poll() is None:
                        other.kill()
                raise RuntimeError(f"hipcc failed on {src}:\n" + _messages(res))
            if verbose and _messages(res):
                print(_messages(res), flush=True)
            objs.append(obj)
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", LIB, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        res = subprocess.run(link, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + _messages(res))
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
