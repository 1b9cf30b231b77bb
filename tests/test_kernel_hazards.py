"""A check of the compiled kernels, on the CPU: no MFMA result is read too soon on ANY path through the code.

An MFMA's result may be read (or overwritten) by another kind of instruction only some wait states after the MFMA
was issued.  In straight-line code the compiler's hazard recogniser sees to that (it puts `s_nop`s where nothing else
fills the gap); this test does not trust it across control flow.  It compiles the device code to assembly and walks
the control-flow graph of every kernel: from each MFMA it follows the fall-through, every branch target and every
back-edge, counts the wait states along each path (an instruction is one, `s_nop n` is n + 1) and reports any
instruction other than an MFMA that touches the result registers before the required number has passed.  A branch
whose target it cannot resolve (an indirect jump) inside such a window fails the test too.

The number required is not typed in: per MFMA opcode it is the gap the compiler itself leaves, in this very
assembly, between an MFMA and a dependent instruction that follows it with nothing but `s_nop` in between (the
smallest such gap: the compiler inserts exactly what the hardware needs, hand-written `s_nop`s only add to it;
with the 16x16x32 bf16 shape it is eight, for vector-ALU and LDS consumers alike).

History: the decoder with two workgroups per compute unit once decoded wrongly now and then (different from run to
run) when a scalar branch sat between a block's last MFMA and the first read of its accumulators; the kernels now
finish every block (activation, split, store) inside the branch region that computed it, which this walk confirms
for whatever the compiler lays out."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

from paper_2212_01185_amd import build as pcc_build

FALLBACK_NEEDED = 8      # used for an opcode the assembly holds no calibration case for (and as the floor of the planted test)


def _regs(tok):
    """Vector registers (v) and accumulation registers (a, numbered from 1000) named by one operand."""
    tok = tok.strip().rstrip(",")
    m = re.match(r"([va])\[(\d+):(\d+)\]$", tok)
    if m:
        base = 1000 if m.group(1) == "a" else 0
        return set(range(base + int(m.group(2)), base + int(m.group(3)) + 1))
    m = re.match(r"([va])(\d+)$", tok)
    return {(1000 if m.group(1) == "a" else 0) + int(m.group(2))} if m else set()


def _touched(ins):
    """Vector registers an instruction reads or writes (operand modifiers are ignored; memory and DPP forms included)."""
    ops = ins.replace(",", " ").split()[1:]
    out = set()
    for o in ops:
        out |= _regs(o)
    return out


def _functions(lines):
    starts = [i for i, l in enumerate(lines) if l.startswith("_Z") and "kernel" in l and ": " in l]
    for start in starts:
        end = next(i for i in range(start, len(lines)) if lines[i].strip().startswith(".Lfunc_end"))
        body, labels = [], {}
        for l in lines[start + 1:end]:
            s = l.strip()
            if not s or s.startswith(";"):
                continue
            m = re.match(r"(\.LBB\d+_\d+):", s)
            if m:
                labels[m.group(1)] = len(body)
            elif not s.startswith("."):
                body.append(s)
        yield lines[start].split(":")[0], body, labels


def _states(ins):
    return int(ins.split()[1]) + 1 if ins.startswith("s_nop") else 1


def calibrate(functions):
    """opcode -> number of wait states the compiler puts between an MFMA and a dependent instruction that follows it
    behind nothing but s_nop (the smallest seen: hand-written nops only ever add to the compiler's)."""
    need = {}
    for _, body, _ in functions:
        for i, ins in enumerate(body):
            if not ins.startswith("v_mfma"):
                continue
            dst = _regs(ins.split()[1])
            k, gap = i + 1, 0
            while k < len(body) and body[k].startswith("s_nop"):
                gap += _states(body[k])
                k += 1
            if gap and k < len(body) and not body[k].startswith("v_mfma") and _touched(body[k]) & dst:
                op = ins.split()[0]
                need[op] = min(need.get(op, 1 << 30), gap)
    return need


def early_reads(asm_text, needed=None):
    """[(wait states, needed, description)] for every path on which an MFMA's result is touched too soon."""
    functions = list(_functions(asm_text.split("\n")))
    need = dict(calibrate(functions))
    if needed is not None:
        need = {op: needed for op in need} or {}
    default = needed if needed is not None else max(list(need.values()) + [FALLBACK_NEEDED])
    out = []
    for name, body, labels in functions:
        for i, ins in enumerate(body):
            if not ins.startswith("v_mfma"):
                continue
            op = ins.split()[0]
            want = need.get(op, default)
            dst = _regs(ins.split()[1])
            best = {}
            stack = [(i + 1, 0)]
            while stack:
                pc, st = stack.pop()
                while pc < len(body) and st < want:
                    if best.get(pc, 1 << 30) <= st:
                        break
                    best[pc] = st
                    cur = body[pc]
                    if cur.startswith("v_mfma"):
                        if _regs(cur.split()[1]) >= dst:
                            break                      # the accumulators pass on to the next MFMA: its own window starts there
                    elif _touched(cur) & dst:
                        out.append((st, want, "%s: %s ... %s" % (name[:70], ins, cur)))
                        break
                    if cur.startswith("s_endpgm"):
                        break
                    if cur.startswith(("s_setpc", "s_swappc", "s_call")):
                        out.append((st, want, "%s: %s ... unresolvable jump %s" % (name[:70], ins, cur)))
                        break
                    if cur.startswith("s_branch") or cur.startswith("s_cbranch"):
                        target = labels.get(cur.split()[-1])
                        if target is None:
                            out.append((st, want, "%s: %s ... unknown label in %s" % (name[:70], ins, cur)))
                            break
                        stack.append((target, st + 1))
                        if cur.startswith("s_branch"):
                            break
                    st += _states(cur)
                    pc += 1
    return out, need


def test_scanner_finds_planted_cases():
    asm = "\n".join([
        "_Z6kernelv: ; @_Z6kernelv",
        "\tv_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]",
        "\ts_cbranch_vccnz .LBB0_2",
        "\ts_nop 7",
        "\tv_add_f32_e32 v0, v4, v1",
        ".LBB0_2:",
        "\ts_nop 1",
        "\tv_max_f32_e32 v2, v5, v5",
        "\ts_endpgm",
        ".Lfunc_end0:",
    ])
    found, _ = early_reads(asm, needed=8)
    assert [f[0] for f in found] == [3]                   # the branch, then s_nop 1: three wait states on the taken path
    assert not early_reads(asm.replace("s_nop 1", "s_nop 7"), needed=8)[0]
    # a back-edge: the loop's first instruction reads the accumulators of the MFMA at its end
    loop = "\n".join([
        "_Z6kernelv: ; @_Z6kernelv",
        ".LBB0_1:",
        "\tv_mul_f32_e32 v0, v4, v4",
        "\ts_nop 7",
        "\tv_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]",
        "\ts_cbranch_scc1 .LBB0_1",
        "\ts_nop 7",
        "\ts_endpgm",
        ".Lfunc_end0:",
    ])
    found, _ = early_reads(loop, needed=8)
    assert [f[0] for f in found] == [1]
    # a jump the walk cannot follow inside the window
    jump = asm.replace("s_cbranch_vccnz .LBB0_2", "s_setpc_b64 s[4:5]")
    assert "unresolvable" in early_reads(jump, needed=8)[0][0][2]
    # calibration: the planted straight-line case says eight
    assert calibrate(list(_functions(asm.replace("\ts_cbranch_vccnz .LBB0_2\n", "").split("\n"))))["v_mfma_f32_16x16x32_bf16"] == 8


@pytest.mark.skipif(shutil.which(pcc_build.HIPCC) is None and not os.path.exists(pcc_build.HIPCC), reason="no hipcc")
def test_no_mfma_result_is_touched_early_on_any_path():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "pcc.s")
        flags = [f for f in pcc_build.FLAGS if f not in ("-shared", "-fPIC")]
        cmd = [pcc_build.HIPCC] + flags + ["--cuda-device-only", "-S", "-o", out, pcc_build.SRC]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout[-2000:]
        asm = open(out).read()
    assert asm.count("v_mfma_f32_16x16x32_bf16") > 1000          # the kernels are in there
    found, need = early_reads(asm)
    print("wait states the compiler leaves in straight-line code:", need)
    assert need.get("v_mfma_f32_16x16x32_bf16", 0) >= 4, need     # calibration cases exist for the shape the kernels use
    assert not found, "MFMA results touched too soon:\n" + "\n".join("%d of %d wait states: %s" % f for f in sorted(found)[:10])
