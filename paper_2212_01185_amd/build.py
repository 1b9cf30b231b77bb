"""Build libpcc.so (HIP, gfx950) in-tree next to the package."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SRC = os.path.join(_HERE, "csrc", "pcc.hip")
LIB = os.path.join(_HERE, "libpcc.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # encoder and decoder must round identically: no contraction the source does not spell out
    "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results land in vector registers proper (the vector ALU reads them without a copy per register); the
    # decoder's resident weights, which only the matrix cores read, go to the accumulation registers instead
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-function",
    "-I" + os.path.join(ROOT, "include"),
    "-I" + os.path.join(_HERE, "csrc"),
]


def build(verbose: bool = False, extra=(), lib: str = LIB) -> str:
    """Compile the library to `lib` (default: libpcc.so next to the package).  `extra` are more hipcc flags, e.g.
    -DPCC_PHASE_TIMING for the measurement build that counts the decode step's cycles per phase."""
    LIB = lib
    os.makedirs(os.path.dirname(os.path.abspath(LIB)), exist_ok=True)
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC] + FLAGS + list(extra) + ["-o", tmp, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    # python -m paper_2212_01185_amd.build [--out PATH] [hipcc flags ...]
    argv = sys.argv[1:]
    out = LIB
    if argv[:1] == ["--out"]:
        out, argv = os.path.abspath(argv[1]), argv[2:]
    print(build(verbose=True, extra=argv, lib=out))
