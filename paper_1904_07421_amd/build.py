"""Compile libjitdb.so (hand-written HIP for gfx950) next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libjitdb.so")
SOURCES = ["schedule.hip", "forward.hip", "api.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-Rpass-analysis=kernel-resource-usage",
]


def _check_no_scratch(lines) -> None:
    """No kernel may use scratch memory.  The level kernel issues LDS reads from inline asm
    and waits for them by hand; a register spill between the read and its wait would store
    a value that has not arrived yet, so a spilling build is refused rather than run."""
    name = None
    for l in lines:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in l:
            size = int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0].strip())
            if size != 0:
                raise RuntimeError(f"kernel {name} uses {size} bytes/lane of scratch memory (register spill)")


def build(verbose: bool = False) -> str:
    """Always recompiles every source; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l]
    out = "\n".join(l for l in lines if "-Rpass-analysis" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    _check_no_scratch(lines)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
