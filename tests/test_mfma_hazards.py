"""Static guard for the hand-written MFMA statements (host only: compiles to assembly, runs nothing).

The long-lived accumulators of the d = 128 kernels are pinned to AGPRs through inline-assembly
MFMAs.  Inline assembly is opaque to the compiler's hazard recognizer, so two rules that the
compiler keeps by itself for its own MFMAs are kept by hand there (csrc/burst_common.h):
  1. a register written by a vector instruction must not be an MFMA source operand within the next
     two wait states (the statements start with `s_nop 1`, or with two vector instructions of the
     slice that do not feed the MFMA);
  2. nothing but another MFMA may touch an accumulator of such a statement while MFMAs on it may
     still be in flight (readers go through mfma_acc_fence / mfma_vgpr_fence: `s_nop`s that
     cover the MFMA's passes).
  3. a vector instruction written inside such a statement (the slices' own arithmetic) must not
     read or overwrite a register that any MFMA, the compiler's included, wrote less than a drained
     MFMA ago: the compiler waits before the instructions it schedules itself, it cannot before
     those it does not see.
A compiler upgrade may place register copies differently.  This test compiles the kernels to
assembly and checks rule 1 for every MFMA inside an inline-assembly block, rule 2 for every
non-MFMA instruction that reads or writes a register an inline-assembly MFMA accumulates into, and
rule 3 for every vector instruction inside an inline-assembly block.
"""
import os
import re
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from paper_2403_09347_amd import build as B  # noqa: E402

KERNEL_SOURCES = ["burst_fwd_mfma.hip", "burst_bwd_dq_mfma.hip", "burst_bwd_dkv_mfma.hip"]
DRAIN = 18                # wait states after which a 32x32x16 MFMA (8 passes) has written its accumulator

REG = re.compile(r"\b([va])(\d+)\b|\b([va])\[(\d+):(\d+)\]")


def regs(operand):
    """Set of (file, index) named by an operand such as v12, a[0:15], v[4:7]."""
    out = set()
    for m in REG.finditer(operand):
        if m.group(1):
            out.add((m.group(1), int(m.group(2))))
        else:
            out.update((m.group(3), i) for i in range(int(m.group(4)), int(m.group(5)) + 1))
    return out


def parse(asm_text):
    """Yields (kernel, [(mnemonic, operands, in_inline_asm)]) per function, instructions in file order."""
    kernel, body, inside = None, [], False
    for raw in asm_text.splitlines():
        line = raw.split(";")[0].strip() if "#ASM" not in raw else raw.strip()
        if "#ASMSTART" in raw:
            inside = True
            continue
        if "#ASMEND" in raw:
            inside = False
            continue
        m = re.match(r"^(_ZN5burst\w+):", line)
        if m:
            kernel, body = m.group(1), []
            continue
        if line.startswith(".Lfunc_end") and kernel:
            yield kernel, body
            kernel = None
            continue
        if kernel is None or not line or line.startswith(".") or line.endswith(":"):
            continue
        parts = line.split(None, 1)
        ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
        body.append((parts[0], ops, inside))


def wait_states(mnemonic, ops):
    if mnemonic == "s_nop":
        return int(ops[0], 0) + 1
    return 1


def check_kernel(name, body):
    problems = []
    asm_acc = set()                                   # registers that inline-assembly MFMAs accumulate into
    for mn, ops, inside in body:
        if inside and mn.startswith("v_mfma"):
            asm_acc |= regs(ops[0])
    n_asm_mfma = 0
    for i, (mn, ops, inside) in enumerate(body):
        if mn.startswith("v_mfma") and inside:
            n_asm_mfma += 1
            sources = set().union(*(regs(o) for o in ops[1:4]))
            gap = 0
            for pmn, pops, _ in reversed(body[max(0, i - 3):i]):
                if gap >= 2:
                    break
                is_valu = pmn.startswith("v_") and not pmn.startswith("v_mfma")
                if is_valu and pops and regs(pops[0]) & sources:
                    problems.append(f"{name}: instruction {i}: {pmn} {pops[0]} feeds an inline-asm MFMA {gap} wait states later")
                gap += wait_states(pmn, pops)
        if inside and mn.startswith("v_") and not mn.startswith("v_mfma"):      # rule 3
            touched = set().union(*(regs(o) for o in ops)) if ops else set()
            gap = 0
            for pmn, pops, _ in reversed(body[max(0, i - 64):i]):
                if gap >= DRAIN:
                    break
                if pmn.startswith("v_mfma") and regs(pops[0]) & touched:
                    problems.append(f"{name}: instruction {i}: {mn} inside an asm statement touches "
                                    f"{sorted(touched & regs(pops[0]))[:2]} {gap} wait states after an MFMA wrote it")
                    break
                gap += wait_states(pmn, pops)
        if not mn.startswith("v_mfma") and asm_acc:
            touched = set().union(*(regs(o) for o in ops)) if ops else set()
            if touched & asm_acc:
                gap = 0
                for pmn, pops, pin in reversed(body[max(0, i - 64):i]):
                    if gap >= DRAIN:
                        break
                    if pmn.startswith("v_mfma") and pin and regs(pops[0]) & touched:
                        problems.append(f"{name}: instruction {i}: {mn} touches {sorted(touched & asm_acc)[:2]} "
                                        f"{gap} wait states after an inline-asm MFMA on it")
                        break
                    gap += wait_states(pmn, pops)
    return n_asm_mfma, problems


@pytest.mark.parametrize("source", KERNEL_SOURCES)
def test_inline_asm_mfma_hazards(source):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [hipcc, *B.FLAGS, "--cuda-device-only", "-S", os.path.join(B.CSRC, source), "-o", out]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-3000:]
        text = open(out).read()
    total, problems = 0, []
    for kernel, body in parse(text):
        n, p = check_kernel(kernel, body)
        total += n
        problems += p
    assert total >= 32, f"{source}: expected inline-assembly MFMAs, found {total}"
    assert not problems, "\n".join(problems[:20])


def test_checker_finds_planted_hazards():
    """The checker itself, on hand-made instruction lists."""
    mf = ("v_mfma_f32_32x32x16_bf16", ["a[0:15]", "v[4:7]", "v[8:11]", "a[0:15]"], True)
    ok = [("v_mov_b32_e32", ["v4", "v20"], False), ("s_nop", ["1"], True), mf]
    assert check_kernel("k", ok) == (1, [])
    bad = [("v_mov_b32_e32", ["v4", "v20"], False), ("s_nop", ["0"], True), mf]
    assert len(check_kernel("k", bad)[1]) == 1
    also_ok = [("v_mov_b32_e32", ["v4", "v20"], False), ("v_exp_f32_e32", ["v30", "v30"], True),
               ("v_exp_f32_e32", ["v31", "v31"], True), mf]
    assert check_kernel("k", also_ok) == (1, [])
    early_read = [mf, ("s_nop", ["15"], False), ("v_accvgpr_read_b32", ["v1", "a3"], False)]
    assert len(check_kernel("k", early_read)[1]) == 1
    builtin = ("v_mfma_f32_32x32x16_bf16", ["v[32:47]", "v[4:7]", "v[8:11]", "v[32:47]"], False)
    hidden_read = [builtin, ("s_nop", ["7"], False), ("v_fma_f32", ["v60", "v33", "s1", "v61"], True)]
    assert len(check_kernel("k", hidden_read)[1]) == 1
    late_read = [builtin] + [("s_nop", ["7"], False)] * 3 + [("v_fma_f32", ["v60", "v33", "s1", "v61"], True)]
    assert check_kernel("k", late_read) == (0, [])
    fenced = [mf, ("s_nop", ["15"], False), ("s_nop", ["15"], False), ("v_accvgpr_read_b32", ["v1", "a3"], False)]
    assert check_kernel("k", fenced) == (1, [])
