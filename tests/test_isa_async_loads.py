"""The attention kernel requests its Q fragments with hand-written load instructions that the compiler does not
track (so that nothing waits for them before the first K/V tile has been requested); the registers they fill must
not be read before the kernel's own s_waitcnt.  The source arranges that with in/out operands on the wait, but
nothing in the language forbids the compiler to copy such a register early, so the generated code is checked:
compile csrc/tree_attn.hip to gfx950 assembly and scan every attn_mfma_kernel instantiation."""
import os
import re
import subprocess

import pytest

from paper_2406_17276_amd import build as B


def _regs(tok):
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def find_early_reads(asm_text):
    """[(kernel, line number, instruction)] of instructions that touch a register filled by a hand-issued
    global_load_dwordx{2,4} (inside an inline-assembly block) before any s_waitcnt vmcnt follows the load."""
    kernel, pending, in_asm, bad, seen = None, {}, False, [], 0
    for no, line in enumerate(asm_text.split("\n"), 1):
        m = re.match(r"^(_Z\S+):", line)
        if m:
            kernel, pending = m.group(1), {}
        if ";;#ASMSTART" in line:
            in_asm = True
        if ";;#ASMEND" in line:
            in_asm = False
        m = re.match(r"^([a-z_0-9]+)\s+(.*)$", line.strip())
        if not m or not kernel or "attn_mfma_kernel" not in kernel:
            continue
        op, ops = m.group(1), [x.strip() for x in m.group(2).split(",")]
        if in_asm and op in ("global_load_dwordx4", "global_load_dwordx2"):
            seen += 1
            for r in _regs(ops[0]):
                pending[r] = no
        elif op == "s_waitcnt" and "vmcnt" in m.group(2):
            pending = {}
        elif pending:
            used = set()
            for o in ops:
                used |= _regs(o.split(" ")[0])
            if used & set(pending):
                bad.append((kernel, no, line.strip()))
    return bad, seen


def test_checker_sees_a_planted_early_read():
    planted = "\n".join(["_ZN2ot16attn_mfma_kernelEv:", "\t;;#ASMSTART", "\tglobal_load_dwordx4 v[4:7], v[2:3], off", "\t;;#ASMEND",
                         "\tv_mov_b32_e32 v9, v5", "\ts_waitcnt vmcnt(0)", "\tv_mov_b32_e32 v10, v6"])
    bad, seen = find_early_reads(planted)
    assert seen == 1 and len(bad) == 1 and bad[0][1] == 5


@pytest.mark.timeout(600)
def test_registers_of_hand_issued_loads_are_not_read_before_the_wait(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    out = tmp_path / "tree_attn.s"
    flags = [f for f in B.FLAGS if f != "-fPIC"]
    subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only", os.path.join(B.CSRC, "tree_attn.hip"), "-o", str(out)],
                   check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    bad, seen = find_early_reads(out.read_text())
    assert seen >= 4 * 4, "the hand-issued Q loads were not found in the assembly: the check is out of date"
    assert not bad, bad[:5]
