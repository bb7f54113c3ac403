"""The diagonal-block elimination places its LDS column loads by hand (inline `ds_read_b128` whose results are
only valid after a later `s_waitcnt lgkmcnt(0)` written by hand as well). The compiler does not know that the
destination registers are still in flight between the two statements; this test compiles the file to assembly and
checks, in every kernel that contains the elimination, that no instruction names such a register before the
wait."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2506_22668_amd", "csrc", "gram_chol.hip")
KERNELS = ("chol_diag_kernel", "chol_step_kernel", "chol_update_kernelILb1")


def test_no_use_of_an_in_flight_lds_destination_before_its_wait():
    # exactly the flags of the shipped library (one list, in build.py), so that the code inspected here is the
    # code that runs; a machine without the compiler fails this test rather than passing it unseen
    from paper_2506_22668_amd.build import COMPILE_FLAGS, HIPCC
    assert os.path.exists(HIPCC) or shutil.which(HIPCC), "hipcc is needed to inspect the generated code"
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gram_chol.s")
        cmd = [HIPCC] + COMPILE_FLAGS + ["-S", "--cuda-device-only", SRC, "-o", out]
        subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        lines = open(out).read().split("\n")
    name, pending, reads, seen = "", {}, 0, set()
    for ln in lines:
        m = re.match(r"^(_Z\w+):", ln)
        if m:
            name, pending = m.group(1), {}
        if not any(k in name for k in KERNELS):
            continue
        t = ln.strip()
        if not t or t.startswith(";"):
            continue
        m = re.match(r"ds_read_b128 v\[(\d+):(\d+)\]", t)
        if m:
            reads += 1
            seen.add(name)
            for r in range(int(m.group(1)), int(m.group(2)) + 1):
                pending[r] = t
            continue
        if t.startswith("s_waitcnt") and "lgkmcnt(0)" in t:
            pending = {}
            continue
        if pending:
            regs = set()
            for a, b in re.findall(r"v\[(\d+):(\d+)\]", t):
                regs.update(range(int(a), int(b) + 1))
            regs.update(int(a) for a in re.findall(r"\bv(\d+)\b", t))
            hit = sorted(r for r in regs if r in pending)
            assert not hit, f"{name}: `{t}` names v{hit[0]} while `{pending[hit[0]]}` is in flight"
    # the elimination is there (16 column loads per kernel and column pair) in all three kernels
    assert len(seen) == 3 and reads >= 3 * 60
