"""Checks on the gfx950 assembly that hipcc generates for the fused kernel (no GPU needed).

The query-weight broadcast of the fused kernel is a DPP modifier on v_fmac_f32, written as inline assembly.  The
CDNA ISA asks for two wait states between a VALU instruction that writes a VGPR and a DPP instruction that reads
it; the hardware does not interlock and the compiler's hazard recogniser does not look into inline assembly.  The
weights come from LDS reads, so no such pair should exist: this test fails if a compiler change ever creates one.
The walk follows the control flow backwards (fall-through and every branch into a label), not just the text order.
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


def _parse(asm):
    """Instructions in program order, the label positions, and for every label the instructions that branch to it."""
    insts, labels = [], {}
    for line in asm.splitlines():
        line = line.split(";")[0].strip()
        if not line or line.startswith("."):
            if line.endswith(":"):          # local labels look like .LBB0_12:
                labels[line[:-1]] = len(insts)
            continue
        if line.endswith(":"):
            labels[line[:-1]] = len(insts)
            continue
        insts.append(line)
    at = {}
    for lab, pos in labels.items():
        at.setdefault(pos, []).append(lab)
    branches = {}
    for i, ins in enumerate(insts):
        name = ins.split()[0]
        if name == "s_branch" or name.startswith("s_cbranch"):
            branches.setdefault(ins.split()[1], []).append(i)
    return insts, at, branches


def _check_back(insts, at, branches, i, wait, dpp_src, ins, seen):
    """Walk backwards from instruction i (exclusive) over every path that can reach it, `wait` wait states so far."""
    while wait < 2:
        # predecessors through branches to a label that sits right before instruction i
        for lab in at.get(i, []):
            for b in branches.get(lab, []):
                if (b, wait) not in seen:
                    seen.add((b, wait))
                    _check_back(insts, at, branches, b + 1, wait, dpp_src, ins, seen)
        j = i - 1
        if j < 0:
            return
        prev = insts[j]
        name = prev.split()[0]
        if name in ("s_branch", "s_endpgm", "s_setpc_b64") and at.get(i):
            return                          # no fall-through into the label: only the branches above lead here
        if name == "s_nop":
            wait += int(prev.split()[1], 0) + 1
        else:
            if name.startswith("v_") and not name.startswith("v_cmp"):
                dst = _regs(prev.split(None, 1)[1].split(",")[0])
                assert not (dst & dpp_src), f"VALU write too close to a DPP read:\n  {prev}\n  {ins}"
            wait += 1
        i = j


def test_dpp_fma_source_is_not_written_by_the_two_preceding_valu_instructions(asm):
    """Backwards from every v_fmac_f32_dpp over two wait states, along the straight line and along every branch that
    enters a label on the way (so a write at the end of a predecessor block counts too)."""
    insts, at, branches = _parse(asm)
    n_dpp = 0
    for i, ins in enumerate(insts):
        if not ins.startswith("v_fmac_f32_dpp"):
            continue
        n_dpp += 1
        ops = ins.split(None, 1)[1].split(",")
        dpp_src = _regs(ops[1].split()[0])
        assert dpp_src, ins
        _check_back(insts, at, branches, i, 0, dpp_src, ins, set())
    assert n_dpp > 0, "the fused kernel no longer uses v_fmac_f32_dpp: drop or adapt this test"


def test_the_walk_sees_a_write_at_the_end_of_a_predecessor_block():
    """The checker itself, on hand-written snippets: a VALU write that reaches the DPP read through a branch is found,
    one that is two wait states away is not."""
    bad = """
        v_mov_b32 v5, v9
        s_cbranch_scc1 .LBB0_2
    .LBB0_1:
        s_nop 0
        s_branch .LBB0_3
    .LBB0_2:
        v_fmac_f32_dpp v1, v5, v2 quad_perm:[0,0,0,0] row_mask:0xf bank_mask:0xf
    .LBB0_3:
        s_endpgm
    """
    insts, at, branches = _parse(bad)
    i = next(k for k, x in enumerate(insts) if x.startswith("v_fmac_f32_dpp"))
    with pytest.raises(AssertionError):
        _check_back(insts, at, branches, i, 0, {5}, insts[i], set())
    good = bad.replace("s_cbranch_scc1 .LBB0_2", "s_nop 1\n        s_cbranch_scc1 .LBB0_2")
    insts, at, branches = _parse(good)
    i = next(k for k, x in enumerate(insts) if x.startswith("v_fmac_f32_dpp"))
    _check_back(insts, at, branches, i, 0, {5}, insts[i], set())


@pytest.mark.parametrize("source", ["quantize.hip", "encode.hip"])
def test_row_reductions_of_the_store_kernels_carry_their_wait_states(source):
    """The store kernels reduce a token's row with v_min_f32_dpp / v_max_f32_dpp (inline assembly, csrc/tile_quant.cuh);
    each of these reads the register the instruction before it wrote, so the assembly puts an s_nop of at least two
    wait states (s_nop 1) directly in front of every one: checked on what the compiler emitted."""
    lines = [l.split(";")[0].strip() for l in B.device_assembly(source).splitlines()]
    lines = [l for l in lines if l and not l.startswith(".") and not l.endswith(":")]
    found = 0
    for i, ins in enumerate(lines):
        if ins.split()[0] in ("v_min_f32_dpp", "v_max_f32_dpp"):
            found += 1
            prev = lines[i - 1].split()
            assert prev[0] == "s_nop" and int(prev[1], 0) >= 1, (i, lines[i - 1], ins)
    assert found >= 8   # the V quantizer is in every store kernel of both files
