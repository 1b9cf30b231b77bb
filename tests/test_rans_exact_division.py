"""CPU check of the row coder's division through fp64 (csrc/rans_arith.h, the source the kernels compile).

The GPU coder replaces the 64-bit x / f of the rANS push by an fp64 estimate rounded toward zero and one
integer correction.  The host program under tests/host_checks builds that same header with g++ and compares
it with integer division for every frequency 1 .. 65536 and states at both ends of the range, around
multiples of f, around powers of two and at random (9.4 million pushes, three reciprocal seeds).
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_rans_push_equals_integer_division(tmp_path):
    exe = str(tmp_path / "rans_push_check")
    src = os.path.join(ROOT, "tests", "host_checks", "rans_push_check.cpp")
    inc = os.path.join(ROOT, "paper_2212_01185_amd", "csrc")
    # -frounding-math: the program switches rounding modes; -ffp-contract=off: as the kernels are built
    subprocess.run(["g++", "-O2", "-std=c++17", "-frounding-math", "-ffp-contract=off", "-I" + inc, src, "-o", exe], check=True)
    res = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
    print(res.stdout)
    assert res.returncode == 0, res.stdout
    last = res.stdout.strip().splitlines()[-1].split()
    assert last[0] == "checked" and int(last[1]) > 9_000_000 and last[2:] == ["failures", "0", "recip_out_of_bounds", "0"]
