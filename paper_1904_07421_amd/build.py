"""Compile libjitdb.so (hand-written HIP for gfx950) next to this file."""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libjitdb.so")
SOURCES = ["schedule.hip", "forward.hip", "level256.hip", "cells.hip", "backward.hip", "cache.hip", "probe.hip", "api.hip"]

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


_VREG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")


def _vregs(text: str) -> set:
    out = set()
    for m in _VREG.finditer(text):
        if m.group(1) is not None:
            out.add(int(m.group(1)))
        else:
            out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def _join(a, b):
    """Upper bound of two FIFO states (oldest first): align at the youngest end, unite per slot."""
    if a is None:
        return b
    if b is None:
        return a
    n = max(len(a), len(b))
    a = (frozenset(),) * (n - len(a)) + a
    b = (frozenset(),) * (n - len(b)) + b
    return tuple(x | y for x, y in zip(a, b))


def check_lds_read_waits(asm_text: str, kernel_substr: str = "level_kernel") -> int:
    """Static check of the generated code of the level kernel, whose LDS fragment reads are
    inline asm the compiler knows nothing about: between a ds_read and the s_waitcnt
    lgkmcnt that covers it, no other instruction may touch the registers it will write (a
    compiler-made copy or spill there would move data that has not arrived).  LDS and
    scalar-memory operations of a wave are counted by one in-order counter, modelled as a
    FIFO of destination-register sets; the states are propagated over the control-flow
    graph of each kernel to a fixed point.  Returns the number of ds_read instructions seen."""
    # split into kernels, then basic blocks
    kernels, cur = [], None
    for raw in asm_text.splitlines():
        line = raw.split(";")[0].strip()
        if not line:
            continue
        if line.endswith(":") and not line.startswith("."):
            cur = [] if kernel_substr in line else None
            if cur is not None:
                kernels.append(cur)
            continue
        if cur is None or (line.startswith(".") and not line.endswith(":")):
            continue
        cur.append(line)
    seen = 0
    for body in kernels:
        blocks, names = [[]], {}
        for line in body:
            if line.endswith(":"):
                if blocks[-1]:
                    blocks.append([])
                names[line[:-1]] = len(blocks) - 1
                continue
            blocks[-1].append(line)
            op = line.split(" ")[0]
            if op.startswith("s_cbranch") or op in ("s_branch", "s_endpgm"):
                blocks.append([])
        succ = []
        for bi, blk in enumerate(blocks):
            last = blk[-1].split() if blk else []
            nxt = [bi + 1] if bi + 1 < len(blocks) else []
            if last and last[0] == "s_branch":
                succ.append([names[last[1]]])
            elif last and last[0].startswith("s_cbranch"):
                succ.append([names[last[1]]] + nxt)
            elif last and last[0] == "s_endpgm":
                succ.append([])
            else:
                succ.append(nxt)
        state_in = [None] * len(blocks)
        state_in[0] = ()
        work = [0]
        while work:
            bi = work.pop()
            pending = list(state_in[bi])
            for line in blocks[bi]:
                op, _, rest = line.partition(" ")
                if op == "s_waitcnt":
                    m = re.search(r"lgkmcnt\((\d+)\)", rest)
                    if m and int(m.group(1)) < len(pending):
                        pending = pending[len(pending) - int(m.group(1)):]
                    continue
                busy = frozenset().union(*pending) if pending else frozenset()
                if busy:
                    touched = _vregs(rest)
                    if op.startswith("ds_read"):          # its address may be a register it overwrites
                        touched = _vregs(rest.split(",")[0])
                    if touched & busy:
                        raise RuntimeError("register of an LDS read in flight is touched before its wait: " + line)
                if op.startswith("ds_read"):
                    pending.append(frozenset(_vregs(rest.split(",")[0])))
                elif op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load"):
                    pending.append(frozenset())
                pending = pending[-64:]
            out = tuple(pending)
            for t in succ[bi]:
                joined = _join(state_in[t], out)
                if joined != state_in[t]:
                    state_in[t] = joined
                    work.append(t)
        seen += sum(1 for line in body if line.startswith("ds_read"))
    return seen


_VMEM = re.compile(r"(global|buffer|flat|scratch)_(load|store|atomic)")


def check_stage_loads(asm_text: str, kernel_substr: str = "level_kernel") -> int:
    """Static check of the K loops of the kernels that move pipeline stages with direct-to-LDS loads
    and wait for them with hand-written `s_waitcnt vmcnt(N)`: N is a number of loads of a YOUNGER
    stage that may stay in flight, so it is only right if every wave issues exactly the expected
    loads per stage and nothing else joins the same counter in between.  For every innermost loop
    that holds MFMAs, the only vector-memory instructions must be global_load_lds_dwordx4, and their
    number must be (loads per wave and stage) x (barriers in the loop): 5 for the leaf level kernel
    (its blocks skip the forget rows), 6 otherwise.  Returns the number of loops examined."""
    kernels, cur, name = [], None, None
    for raw in asm_text.splitlines():
        line = raw.split(";")[0].strip()
        if not line:
            continue
        if line.endswith(":") and not line.startswith("."):
            cur = [] if kernel_substr in line else None
            if cur is not None:
                kernels.append((line[:-1], cur))
            continue
        if cur is None or (line.startswith(".") and not line.endswith(":")):
            continue
        cur.append(line)
    examined = 0
    for name, body in kernels:
        m = re.search(r"level_kernelI[a-z]Li(\d)E", name)
        per_stage = 5 if (m and m.group(1) == "0") else 6
        labels = {l[:-1]: i for i, l in enumerate(body) if l.endswith(":")}
        loops = {}
        for i, l in enumerate(body):
            p = l.split()
            if len(p) >= 2 and (p[0].startswith("s_cbranch") or p[0] == "s_branch") and p[1] in labels and labels[p[1]] <= i:
                head = labels[p[1]]
                loops[head] = max(loops.get(head, head), i)
        with_mfma = [(a, b) for a, b in loops.items() if any(l.startswith("v_mfma") for l in body[a:b + 1])]
        for a, b in with_mfma:
            if any(a < a2 and b2 <= b for a2, b2 in with_mfma):
                continue                                   # not innermost
            seg = body[a:b + 1]
            other = [l for l in seg if _VMEM.match(l) and not l.startswith("global_load_lds_dwordx4")]
            if other:
                raise RuntimeError(f"{name}: a K loop holds a vector-memory instruction besides the stage loads: {other[0]}")
            n_dma = sum(1 for l in seg if l.startswith("global_load_lds_dwordx4"))
            n_bar = sum(1 for l in seg if l.startswith("s_barrier"))
            if n_dma == 0 and n_bar == 0:
                continue                                   # a loop of MFMAs on operands that do not come through stages
            if n_bar == 0 or n_dma != per_stage * n_bar:
                raise RuntimeError(f"{name}: a K loop issues {n_dma} stage loads for {n_bar} barrier(s); "
                                   f"the hand-placed waits assume {per_stage} per stage")
            examined += 1
    return examined


def build(verbose: bool = False) -> str:
    """Always recompiles every source; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    cmd = [hipcc, *HIPCC_FLAGS, "--save-temps", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    tmp = tempfile.mkdtemp(prefix="jitdb_build_")
    try:
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, cwd=tmp)
        asm_texts = {}
        for stem in ("forward", "level256"):
            asm_path = os.path.join(tmp, stem + "-hip-amdgcn-amd-amdhsa-gfx950.s")
            asm_texts[stem] = open(asm_path).read() if os.path.exists(asm_path) else None
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l]
    out = "\n".join(l for l in lines if "-Rpass-analysis" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    _check_no_scratch(lines)
    # the kernels whose LDS reads (and, for the 256 x 256 tile kernel, weight loads) are inline asm
    # (names with their length prefix, as they are mangled: "level_kernel" alone would also match fused_level_kernel)
    for stem, name in (("forward", "12level_kernel"), ("forward", "14gemm_kb_kernel"), ("forward", "17nary_level_kernel"),
                       ("level256", "14tile256_kernel")):
        if asm_texts.get(stem) is None:
            raise RuntimeError(f"the device assembly of {stem}.hip was not produced; cannot check it")
        if check_lds_read_waits(asm_texts[stem], name) == 0:
            raise RuntimeError(f"no LDS reads found in the assembly of {name}: the check is not looking at it")
    # the K loops whose waits for direct-to-LDS stage loads are hand-counted
    for name in ("12level_kernel", "14gemm_kb_kernel", "17nary_level_kernel"):
        if check_stage_loads(asm_texts["forward"], name) == 0:
            raise RuntimeError(f"no K loop with stage loads found in the assembly of {name}: the check is not looking at it")
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
