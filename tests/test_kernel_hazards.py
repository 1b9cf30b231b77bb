"""A check of the compiled kernels, on the CPU: no MFMA result is read too soon along a taken branch.

An MFMA's result may be read by another kind of instruction only some wait states after the MFMA was issued
(eight for the 16x16x32 bf16 shape as this compiler counts them: it puts `s_nop 7` between the two when nothing else
is there).  The compiler counts those wait states along the instruction stream as laid out; where a branch follows
the MFMA closely and is taken, the instructions it skipped do not count, and the hardware then reads accumulators
that are not written yet.  The decoder with two workgroups per compute unit once had such a place (wrong decodes
now and then, different from run to run).  This test compiles the device code to assembly and looks for the pattern
in every kernel."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

from paper_2212_01185_amd import build as pcc_build

WINDOW = 14          # instructions looked at behind an MFMA and behind a branch target
NEEDED = 8           # wait states between an MFMA and the first read of its result by a non-MFMA instruction


def _regs(tok):
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


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


def _wait_states(instrs):
    return sum(int(x.split()[1]) + 1 if x.startswith("s_nop") else 1 for x in instrs)


def shortest_taken_paths(asm_text):
    """(wait states, description) of every place where a non-MFMA instruction reads an MFMA's result close behind
    a branch that was taken close behind that MFMA."""
    out = []
    for name, body, labels in _functions(asm_text.split("\n")):
        for i, ins in enumerate(body):
            if not ins.startswith("v_mfma"):
                continue
            dst = _regs(ins.split()[1].rstrip(","))
            for d in range(1, WINDOW):
                if i + d >= len(body):
                    break
                br = body[i + d]
                if not (br.startswith("s_cbranch") or br.startswith("s_branch")):
                    continue
                target = labels.get(br.split()[-1])
                if target is None:
                    continue
                for e in range(WINDOW):
                    if target + e >= len(body):
                        break
                    use = body[target + e]
                    ops = use.replace(",", " ").split()[1:]
                    is_store = use.startswith(("ds_write", "global_store", "global_atomic", "buffer_store", "scratch_store"))
                    srcs = ops if is_store else ops[1:]
                    read = set().union(*[_regs(o) for o in srcs]) if srcs else set()
                    if read & dst and not use.startswith("v_mfma"):
                        # between the two: the instructions behind the MFMA up to and with the branch, then the target's
                        states = _wait_states(body[i + 1:i + d + 1]) + _wait_states(body[target:target + e])
                        out.append((states, "%s: %s ... %s ... %s" % (name[:60], ins.split()[0], br, use)))
                        break
    return out


def test_scanner_finds_a_planted_case():
    asm = "\n".join([
        "_Z6kernelv: ; @_Z6kernelv",
        "\tv_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]",
        "\ts_cbranch_vccnz .LBB0_2",
        "\ts_nop 7",
        "\tv_add_f32_e32 v0, v4, v1",
        ".LBB0_2:",
        "\ts_nop 1",
        "\tv_max_f32_e32 v2, v5, v5",
        ".Lfunc_end0:",
    ])
    found = shortest_taken_paths(asm)
    assert len(found) == 1 and found[0][0] == 3          # the branch, then s_nop 1: three wait states
    safe = asm.replace("s_nop 1", "s_nop 7")
    assert shortest_taken_paths(safe)[0][0] == 9


@pytest.mark.skipif(shutil.which(pcc_build.HIPCC) is None and not os.path.exists(pcc_build.HIPCC), reason="no hipcc")
def test_no_mfma_result_is_read_early_behind_a_taken_branch():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "pcc.s")
        flags = [f for f in pcc_build.FLAGS if f not in ("-shared", "-fPIC")]
        cmd = [pcc_build.HIPCC] + flags + ["--cuda-device-only", "-S", "-o", out, pcc_build.SRC]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout[-2000:]
        asm = open(out).read()
    assert asm.count("v_mfma_f32_16x16x32_bf16") > 1000          # the kernels are in there
    found = shortest_taken_paths(asm)
    short = sorted(f for f in found if f[0] < NEEDED)
    assert not short, "MFMA results read too soon behind a taken branch:\n" + "\n".join("%d wait states: %s" % f for f in short[:10])
