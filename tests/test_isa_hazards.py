"""Checks on the gfx950 assembly that hipcc generates for the fused kernel (no GPU needed).

The query-weight broadcast of the fused kernel is a DPP modifier on v_fmac_f32, written as inline assembly.  The
CDNA ISA asks for two wait states between a VALU instruction that writes a VGPR and a DPP instruction that reads
it; the hardware does not interlock and the compiler's hazard recogniser does not look into inline assembly.  The
weights come from LDS reads, so no such pair should exist: this test fails if a compiler change ever creates one.
"""
import re

import pytest

from paper_2509_00579_amd import build as B

_VREG = re.compile(r"^v(\d+)$")
_VRANGE = re.compile(r"^v\[(\d+):(\d+)\]$")


def _regs(op):
    op = op.strip().rstrip(",")
    m = _VREG.match(op)
    if m:
        return {int(m.group(1))}
    m = _VRANGE.match(op)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return set()


@pytest.fixture(scope="module")
def asm():
    return B.device_assembly("attn_fused.hip")


def test_dpp_fma_source_is_not_written_by_the_two_preceding_valu_instructions(asm):
    insts = []
    for line in asm.splitlines():
        line = line.split(";")[0].strip()
        if not line or line.startswith(".") or line.endswith(":"):
            continue
        insts.append(line)
    n_dpp = 0
    for i, ins in enumerate(insts):
        if not ins.startswith("v_fmac_f32_dpp"):
            continue
        n_dpp += 1
        ops = ins.split(None, 1)[1].split(",")
        dpp_src = _regs(ops[1].split()[0])
        assert dpp_src, ins
        wait = 0
        j = i - 1
        while j >= 0 and wait < 2:
            prev = insts[j]
            name = prev.split()[0]
            if name == "s_nop":
                wait += int(prev.split()[1], 0) + 1
            else:
                if name.startswith("v_") and not name.startswith("v_cmp"):
                    dst = _regs(prev.split(None, 1)[1].split(",")[0])
                    assert not (dst & dpp_src), f"VALU write too close to a DPP read:\n  {prev}\n  {ins}"
                wait += 1
            j -= 1
    assert n_dpp > 0, "the fused kernel no longer uses v_fmac_f32_dpp: drop or adapt this test"
