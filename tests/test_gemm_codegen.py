"""The prefill GEMM issues its LDS operand reads as inline assembly with hand-counted waits.  The compiler cannot see
such a read: until the wait it takes the destination registers for valid, and it may copy them, e.g. where two code
regions disagree on the register assignment.  The kernel is written so that no hand-issued read is in flight across a
branch; this test checks the code the compiler actually produced: in every instantiation of that kernel, between a
hand-issued read and the wait for it, no instruction reads the registers the read is going to write.

Compiles the library's device code to assembly with the library's own flags (no GPU needed, about a minute)."""
import os
import re
import subprocess

import pytest

from paper_2507_06608_amd import build as nbuild

SRC = os.path.join(nbuild.CSRC, "nexus_lib.hip")


@pytest.fixture(scope="module")
def device_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "nexus_lib.s"
    flags = [f for f in nbuild.FLAGS if f not in ("-fPIC", "-shared")]
    r = subprocess.run(["hipcc"] + flags + ["-S", "--cuda-device-only", "-o", str(out), SRC], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text().split("\n")


def _registers(operands: str):
    regs = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", operands):
        regs |= set(range(int(a), int(b) + 1))
    for a in re.findall(r"\bv(\d+)\b", operands):
        regs.add(int(a))
    return regs


def test_no_instruction_reads_a_register_with_a_hand_issued_lds_read_in_flight(device_asm):
    lines = device_asm
    starts = [i for i, l in enumerate(lines) if re.match(r"_ZN5nexus14gemm_dl_kernel\S*:", l)]
    assert starts, "no gemm_dl_kernel instantiation found in the device code"
    checked = 0
    for s in starts:
        name = lines[s].split(":")[0]
        m = re.search(r"ILi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELb(\d)ELi(\d+)ELb(\d)", name)
        assert m, name
        bkt, asm_reads = int(m.group(5)), m.group(8) == "1"
        if not asm_reads or bkt != 2:
            continue    # the other instantiations wait with partial counts the scan below does not model
        end = next(i for i in range(s, len(lines)) if lines[i].startswith(".Lfunc_end"))
        pending, n_reads, issues = set(), 0, []
        for i in range(s, end):
            code = lines[i].split(";")[0].strip()
            if not code or code.startswith(".") or code.endswith(":"):
                continue
            m2 = re.match(r"ds_read_b128 v\[(\d+):(\d+)\]", code)
            if m2:
                pending |= set(range(int(m2.group(1)), int(m2.group(2)) + 1))
                n_reads += 1
                continue
            if code.startswith("s_waitcnt") and "lgkmcnt(0)" in code:
                pending = set()
                continue
            if pending and "," in code:
                if _registers(code.split(",", 1)[1]) & pending:
                    issues.append((i + 1, code))
        assert n_reads > 0, name
        assert not issues, f"{name}: {issues[:5]}"
        checked += 1
    assert checked >= 3     # 256 x 256, 256 x 128 and 128 x 128 tiles, each with several epilogues
