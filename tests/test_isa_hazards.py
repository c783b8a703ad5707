"""Static check of the hand-scheduled kernels' instruction streams (no GPU needed).

The hand-scheduled translation units issue their matrix-core products from inline assembly, which
the compiler's hazard recognizer does not look into.  Four hazards are therefore ours to keep out
(the hardware interlocks neither):
  1. a matrix-core instruction must not read a register that a VALU instruction wrote in one of
     the two issue slots before it (s_nop N fills N+1 slots);
  2. nothing but a matrix-core accumulate into the same registers may touch the result registers
     of a matrix-core instruction until it has finished: 12 issue slots, a further matrix-core
     instruction counting as the 8 passes it keeps the pipe for.
  3. the VALU instruction right behind a transcendental one (v_exp_f32, ...) must not read its result;
     the compiler keeps this apart in its own code but does not look into inline assembly, and may put
     a register copy right behind an assembly statement that ends in one.
  4. the asynchronous global->LDS loads take their LDS address from M0: one wait state between the scalar
     write of M0 and the load (both sit in one assembly statement, out of the compiler's sight).
The compiler is free to put register copies right in front of or right behind an inline-assembly
statement (at a loop exit, say), so this is checked on the generated assembly of every
instantiation rather than argued from the source.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2511_19797_amd import build

CSRC = os.path.join(os.path.dirname(build.__file__), "csrc")
HAND_SCHEDULED = ["bwd_row_pipe.hip", "bwd_col_pipe.hip", "bwd_row_pipe_tangent.hip", "bwd_col_pipe_tangent.hip",
                  "bwd_row_pipe_qknorm.hip", "bwd_col_pipe_qknorm.hip", "bwd_pass.hip"]

REG = re.compile(r"\b([va])(?:(\d+)|\[(\d+):(\d+)\])")


def regs(operand):
    out = set()
    for m in REG.finditer(operand):
        f = m.group(1)
        if m.group(2) is not None:
            out.add((f, int(m.group(2))))
        else:
            out.update((f, i) for i in range(int(m.group(3)), int(m.group(4)) + 1))
    return out


def instructions(asm_text):
    """(mnemonic, [operands]) of every instruction, in file order (labels, directives, comments dropped)."""
    for line in asm_text.splitlines():
        t = line.split(";")[0].strip()
        if not t or t.startswith(".") or t.endswith(":") or t.startswith("//"):
            continue
        parts = t.split(None, 1)
        ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
        yield parts[0], ops


def violations(asm_text):
    ins = list(instructions(asm_text))
    bad = []
    for i, (op, ops) in enumerate(ins):
        if not op.startswith("v_mfma"):
            continue
        srcs = set().union(*[regs(o) for o in ops[1:]])
        slots = 0
        j = i - 1
        while j >= 0 and slots < 2:
            pop, pops = ins[j]
            if pop == "s_nop":
                slots += int(pops[0], 0) + 1
            else:
                is_valu = pop.startswith("v_") and not pop.startswith("v_mfma")
                if is_valu and pops and regs(pops[0]) & srcs:
                    bad.append((i, " ".join([pop] + pops), " ".join([op] + ops)))
                slots += 1
            j -= 1
    return bad


def result_violations(asm_text, need=12):
    """Hazard 2: (index, toucher, mfma) for every instruction that touches an unfinished result."""
    ins = list(instructions(asm_text))
    bad = []
    for i, (op, ops) in enumerate(ins):
        if not op.startswith("v_mfma"):
            continue
        dst = regs(ops[0])
        slots = 0
        for j in range(i + 1, len(ins)):
            nop, nops = ins[j]
            if nop.startswith("v_mfma"):
                same_acc = regs(nops[0]) == dst and regs(nops[-1]) == dst
                srcs = set().union(*[regs(o) for o in nops[1:3]])
                if (srcs & dst) or (not same_acc and (regs(nops[0]) | regs(nops[-1])) & dst):
                    bad.append((i, " ".join([nop] + nops), " ".join([op] + ops)))
                slots += 8
            elif nop == "s_nop":
                slots += int(nops[0], 0) + 1
            else:
                touched = set().union(*[regs(o) for o in nops]) if nops else set()
                if touched & dst:
                    bad.append((i, " ".join([nop] + nops), " ".join([op] + ops)))
                slots += 1
            if slots >= need:
                break
    return bad


TRANS = ("v_exp_", "v_log_", "v_rcp_", "v_rsq_", "v_sqrt_", "v_sin_", "v_cos_")


def trans_violations(asm_text):
    """Hazard 3: (index, reader, transcendental) for every VALU read of a transcendental result in the next slot."""
    ins = list(instructions(asm_text))
    bad = []
    for i, (op, ops) in enumerate(ins[:-1]):
        if not op.startswith(TRANS):
            continue
        nop, nops = ins[i + 1]
        if not nop.startswith("v_") or nop.startswith(TRANS):
            continue
        srcs = set().union(*[regs(o) for o in nops[1:]]) if len(nops) > 1 else set()
        if nop.startswith(("v_fmac", "v_mac")) or nop.startswith("v_mfma"):
            srcs |= regs(nops[0]) | (regs(nops[-1]) if nop.startswith("v_mfma") else set())
        if regs(ops[0]) & srcs:
            bad.append((i, " ".join([nop] + nops), " ".join([op] + ops)))
    return bad


def m0_violations(asm_text):
    """A load that takes its LDS address from M0 right behind the scalar write of M0 (one wait state is due)."""
    ins = list(instructions(asm_text))
    return [(i, ins[i + 1][0]) for i, (op, ops) in enumerate(ins[:-1])
            if op.startswith("s_mov") and ops and ops[0] == "m0" and "load_lds" in ins[i + 1][0]]


def test_parser_flags_a_planted_hazard():
    planted = """
    v_accvgpr_write_b32 a4, v9
    s_mov_b32 s0, 1
    v_mfma_f32_32x32x16_bf16 v[0:15], v[20:23], a[4:7], v[0:15]
    """
    assert len(violations(planted)) == 1
    padded = planted.replace("s_mov_b32 s0, 1", "s_nop 1")
    assert violations(padded) == []
    far = planted.replace("s_mov_b32 s0, 1", "s_mov_b32 s0, 1\n v_add_u32 v100, v101, v102")
    assert violations(far) == []
    early = """
    v_mfma_f32_32x32x16_bf16 a[64:79], v[2:5], v[22:25], a[64:79]
    ds_read_b128 v[2:5], v100
    v_accvgpr_mov_b32 a48, a64
    """
    assert len(result_violations(early)) == 1
    chained = """
    v_mfma_f32_32x32x16_bf16 a[64:79], v[2:5], v[22:25], a[64:79]
    v_mfma_f32_32x32x16_bf16 a[64:79], v[6:9], v[22:25], a[64:79]
    v_mfma_f32_32x32x16_bf16 a[0:15], v[6:9], v[22:25], a[0:15]
    v_mfma_f32_32x32x16_bf16 a[16:31], v[6:9], v[22:25], a[16:31]
    v_accvgpr_mov_b32 a48, a64
    """
    assert result_violations(chained) == []
    trans = """
    v_exp_f32 v3, v4
    v_accvgpr_write_b32 a9, v3
    """
    assert len(trans_violations(trans)) == 1
    assert trans_violations(trans.replace("v_accvgpr", "v_fma_f32 v7, v8, v9, v10\n v_accvgpr")) == []
    assert trans_violations("v_exp_f32 v3, v4\n v_exp_f32 v5, v3") == []
    assert len(m0_violations("s_mov_b32 m0, s3\n global_load_lds_dwordx4 v1, s[4:5]")) == 1
    assert m0_violations("s_mov_b32 m0, s3\n s_nop 0\n global_load_lds_dwordx4 v1, s[4:5]") == []


@pytest.mark.parametrize("name", HAND_SCHEDULED)
def test_no_valu_write_feeds_next_matrix_instruction(name):
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, name + ".s")
        cmd = ["hipcc", *build.COMMON, *build.PER_FILE.get(name, []), "--cuda-device-only", "-S",
               os.path.join(CSRC, name), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(out).read()
    assert text.count("v_mfma") > 100, "expected the matrix-core kernels in the assembly"
    bad = violations(text)
    assert not bad, f"{len(bad)} VALU->MFMA hazards, first: {bad[:3]}"
    bad = result_violations(text)
    assert not bad, f"{len(bad)} touches of unfinished matrix-core results, first: {bad[:3]}"
    bad = trans_violations(text)
    assert not bad, f"{len(bad)} reads of a transcendental result in the next slot, first: {bad[:3]}"
    assert text.count("load_lds") > 10 and not m0_violations(text)
