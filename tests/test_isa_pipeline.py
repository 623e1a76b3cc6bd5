"""CPU-only check of the hand-scheduled load pipeline in the value pass.

The exact-row loops (bf16 rows and 8-bit rows) issue their loads through inline assembly and waits for them by count.
The compiler does not know those registers are in flight, so nothing it emits may touch a
destination register between the load and the matching wait.  This test compiles the kernel to
gfx950 assembly and replays the instruction stream of every instantiation that uses the pipeline.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2506_13059_amd", "csrc", "mp_value.hip")


def _regs(text):
    out = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text):
        out.update(range(int(a), int(b) + 1))
    for a in re.findall(r"\bv(\d+)\b", text):
        out.add(int(a))
    return out


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_no_instruction_touches_a_register_that_is_still_in_flight(tmp_path):
    asm = tmp_path / "mp_value.s"
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(asm), SRC],
                          stderr=subprocess.DEVNULL)
    lines = asm.read_text().splitlines()
    checked = 0
    i = 0
    while i < len(lines):
        m = re.match(r"^(_ZN2mp\S*value_pass_kernelILi(\d+)ELb(\d)E\S*):", lines[i])
        if not m:
            i += 1
            continue
        G, eight_bit = int(m.group(2)), m.group(3) == "1"
        j = i + 1
        pending = []            # destination register sets of the in-flight asm loads, oldest first
        in_asm = False
        n_loads = n_waits = 0
        while j < len(lines) and not lines[j].startswith(".Lfunc_end"):
            ln = lines[j].strip()
            j += 1
            if ln.startswith(";;#ASMSTART"):
                in_asm = True
                continue
            if ln.startswith(";;#ASMEND"):
                in_asm = False
                continue
            if not ln or ln.startswith(";") or ln.startswith(".") or ln.endswith(":"):
                continue
            if in_asm and ln.startswith("global_load_dwordx"):
                dst = re.match(r"global_load_dwordx[24] v\[(\d+):(\d+)\]", ln)
                regs = set(range(int(dst.group(1)), int(dst.group(2)) + 1))
                addr = _regs(ln.split(",", 1)[1])
                for pset in pending:
                    assert not (pset & (regs | addr)), f"G={G}: {ln} overlaps an in-flight load"
                pending.append(regs)
                n_loads += 1
                continue
            if in_asm and ln.startswith("s_waitcnt vmcnt"):
                n = int(re.search(r"vmcnt\((\d+)\)", ln).group(1))
                while len(pending) > n:
                    pending.pop(0)
                n_waits += 1
                continue
            if ln.startswith("s_waitcnt") and "vmcnt(0)" in ln:
                pending.clear()
                continue
            used = _regs(ln)
            for pset in pending:
                assert not (pset & used), f"G={G}: `{ln}` touches a register of a load still in flight"
        # every group size runs the pipelines (groups of more than five heads as two half-groups), in strips of
        # eight and of two iterations.  bf16 rows: eight loads an iteration.  The kernel of launches with 8-bit
        # rows: six loads an iteration plus the ready-made logit shares of the two rows (one 16-byte load each
        # for up to four heads a wave, two for five), and the two-iteration bf16 strip for the unclustered tail.
        if eight_bit:
            per_iter8 = 6 + 2 * (2 if G == 5 else 1)
            assert n_loads == 16 + 10 * per_iter8 and n_waits == 2 + (8 + 2), (G, n_loads, n_waits)
        else:
            assert n_loads == 64 + 16 and n_waits == 8 + 2, (G, n_loads, n_waits)
        checked += 1
        i = j
    assert checked == 16
