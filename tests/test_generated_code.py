"""The 16x16x32 GEMM kernels issue their MFMAs as inline assembly (see mfma16 in kernels_bf16.hip), so the compiler
does not know that the accumulators it sees are written by instructions whose results take time to land.  Nothing
but those MFMAs may touch an accumulator register within 16 wait states of the MFMA that wrote it: this test compiles
the kernels to assembly (no GPU needed) and follows every path through the code to check that."""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

from paper_2604_16400_amd import build

SETTLE = 16  # wait states; what mfma16_settle() provides
COPY_SETTLE = 4  # wait states between an ordinary write of an accumulator register and an MFMA that reads it
FAR = 10 ** 6


def _device_asm() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(build.CSRC, "kernels_bf16.hip")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = [hipcc] + [f for f in build.FLAGS if f != "-fPIC"] + ["-x", "hip", "-S", "--cuda-device-only", src, "-o", out]
        subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        with open(out) as f:
            return f.read()


def _kernels(asm: str):
    """(name, instructions) of every kernel; an instruction is (text, is_asm_mfma, label or None)."""
    for m in re.finditer(r"^(_ZN5collm\w+):[^\n]*\n(.*?)\n\s*s_endpgm", asm, re.S | re.M):
        ins, in_asm = [], False
        for line in m.group(2).split("\n"):
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
            elif t.startswith(";;#ASMEND"):
                in_asm = False
            if not t or t.startswith(";"):
                continue
            if re.match(r"^\.LBB\d+_\d+:$", t):
                ins.append((t[:-1], False, t[:-1]))
            elif not t.startswith("."):
                ins.append((t, in_asm and t.startswith("v_mfma"), None))
        yield m.group(1), ins


def _acc_regs(text: str):
    """Accumulator registers an instruction names: a7, a[4:7]."""
    regs = set()
    for lo, hi in re.findall(r"\ba\[(\d+):(\d+)\]", text):
        regs.update(range(int(lo), int(hi) + 1))
    regs.update(int(r) for r in re.findall(r"\ba(\d+)\b", text))
    return regs


def _violations(ins):
    """Forward data flow over the instruction list.  State: for every accumulator register written by an
    inline-assembly MFMA less than SETTLE wait states ago, the wait states since (the minimum over all ways to reach
    the instruction).  Any other instruction that names such a register is a violation."""
    label_at = {lab: i for i, (_, _, lab) in enumerate(ins) if lab}
    at_label = {lab: {} for lab in label_at}

    def merge(into, frm):
        changed = False
        for r, d in frm.items():
            if d < into.get(r, FAR):
                into[r] = d
                changed = True
        return changed

    bad = {}
    for _ in range(12):  # until the label states stop changing
        changed, state = False, {}
        for i, (t, is_mfma, lab) in enumerate(ins):
            if lab:
                merge(state, at_label[lab])
                continue
            op = t.split()[0]
            if is_mfma:
                # (negative keys: accumulator registers written by an ordinary instruction, see below)
                dst = re.match(r"\S+\s+a\[(\d+):(\d+)\]", t)
                early = [(r, state[-1 - r]) for r in range(int(dst.group(1)), int(dst.group(2)) + 1) if -1 - r in state]
                if early:
                    bad[i] = (min(d for _, d in early), t)
                step = 1
                state = {r: d + step for r, d in state.items() if d + step < (SETTLE if r >= 0 else COPY_SETTLE)}
                for r in range(int(dst.group(1)), int(dst.group(2)) + 1):
                    state[r] = 0
                continue
            hit = [(r, state[r]) for r in _acc_regs(t) if r in state]
            if hit:
                bad[i] = (min(d for _, d in hit), t)
            step = int(t.split()[1]) + 1 if op == "s_nop" else 1
            state = {r: d + step for r, d in state.items() if d + step < (SETTLE if r >= 0 else COPY_SETTLE)}
            if op.startswith("v_accvgpr_write") or op.startswith("v_accvgpr_mov"):
                # the other direction: an ordinary write of an accumulator register, and the compiler does not know
                # that an MFMA reads it next (it would keep COPY_SETTLE wait states between them)
                state[-1 - int(re.match(r"\S+\s+a(\d+)", t).group(1))] = 0
            tgt = re.search(r"(\.LBB\d+_\d+)", t) if op.startswith(("s_branch", "s_cbranch")) else None
            if tgt and tgt.group(1) in at_label and merge(at_label[tgt.group(1)], state):
                changed = True
            if op in ("s_branch", "s_setpc_b64"):
                state = {}  # nothing falls through
        if not changed:
            break
    return bad


def test_no_accumulator_access_close_behind_an_inline_mfma():
    asm = _device_asm()
    checked = 0
    for name, ins in _kernels(asm):
        if not any(is_mfma for _, is_mfma, _ in ins):
            continue
        checked += 1
        bad = _violations(ins)
        assert not bad, f"{name}: accumulator touched {sorted(bad.items())[:5]} wait states behind an inline MFMA"
    assert checked >= 1, "no kernel with inline-assembly MFMAs was found"


def test_the_checker_sees_a_planted_violation():
    mfma = ("v_mfma_f32_16x16x32_bf16 a[0:3], v[0:3], v[4:7], a[0:3]", True, None)
    read = ("v_accvgpr_read_b32 v9, a2", False, None)
    nop = ("s_nop 7", False, None)
    assert _violations([mfma, read])
    assert _violations([mfma, nop, read])
    assert not _violations([mfma, nop, nop, read])
    assert not _violations([mfma, ("v_accvgpr_read_b32 v9, a8", False, None)])  # another accumulator
    copy = ("v_accvgpr_mov_b32 a1, a40", False, None)
    assert _violations([copy, mfma])
    assert not _violations([copy, ("s_nop 3", False, None), mfma])
    # through a jump: the MFMA is far behind in the text but close on the path that jumps to the label
    far = [("v_add_u32_e32 v1, v2, v3", False, None)] * 20
    jump = [mfma, ("s_cbranch_scc1 .LBB0_7", False, None)] + far + [("s_branch .LBB0_9", False, None),
            (".LBB0_7", False, ".LBB0_7"), read, (".LBB0_9", False, ".LBB0_9")]
    assert _violations(jump)
    # a copy behind a loop's back edge
    loop = [(".LBB0_1", False, ".LBB0_1"), ("v_accvgpr_mov_b32 a8, a0", False, None)] + far + [mfma, ("s_cbranch_vccnz .LBB0_1", False, None)]
    assert _violations(loop)
