"""Host-side check of the generated gfx950 code for one hardware rule the compiler does
not apply to inline asm: between a scalar write of M0 and an add-TID LDS access
(ds_read_addtid_b32 / ds_write_addtid_b32) there must be at least one other instruction.
seq_lds_kernel.h relies on the compiler to place and merge the M0 writes ("{m0}" operands) and
on m0_settle() to supply the wait state; this test compiles the file to assembly and
verifies that every run of add-TID accesses is so protected, in the four files that
instantiate the kernels.  No GPU needed."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRCS = [os.path.join(ROOT, "paper_2503_16815_amd", "csrc", f) for f in ("seq_lds.hip", "seq_lds_rec.hip", "seq_lds_p16.hip", "seq_lds_p16_rec.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

M0_WRITE = re.compile(r"^\s*s_\w+\s+m0\s*,")          # any scalar instruction whose destination is m0
ADDTID = re.compile(r"^\s*ds_(read|write)_addtid_b32\b")
INSTR = re.compile(r"^\s*[a-z_][a-z0-9_]*\b")          # an instruction line (not a label, comment, directive)


def instructions(asm_text):
    for line in asm_text.splitlines():
        code = line.split(";", 1)[0].rstrip()
        if not code.strip() or code.lstrip().startswith(".") or code.rstrip().endswith(":"):
            continue
        if INSTR.match(code):
            yield code.strip()


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_m0_write_is_never_directly_followed_by_an_addtid_access():
    with tempfile.TemporaryDirectory() as tmp:
        jobs = []
        for src in SRCS:   # all compilations at once
            out = os.path.join(tmp, os.path.basename(src) + ".s")
            cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-Xclang", "-target-feature",
                   "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
                   "--cuda-device-only", "-S", "-o", out, src]
            jobs.append((out, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
        texts = []
        for out, proc in jobs:
            _, err = proc.communicate()
            assert proc.returncode == 0, err[-2000:]
            texts.append(open(out).read())
    for text in texts:
        prev = None
        n_addtid = n_m0 = 0
        for ins in instructions(text):
            if ADDTID.match(ins):
                n_addtid += 1
                assert prev is None or not M0_WRITE.match(prev), \
                    f"add-TID access right after an M0 write: {prev!r} -> {ins!r}"
            if M0_WRITE.match(ins):
                n_m0 += 1
            prev = ins
        assert n_addtid > 100 and n_m0 > 0, (n_addtid, n_m0)   # the file really uses them
