"""Builds liblrsa.so (the C-ABI library of the LRSA hot path) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblrsa.so")

HIPCC = "/opt/rocm/bin/hipcc"
# packed-fp32 VALU forms are switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Kernels that count their own outstanding vector-memory operations (s_waitcnt vmcnt(n) around an
# asynchronous LDS ring) must not spill: scratch traffic would be counted by the same counter.
# Scratch (register spill) limits in bytes per lane.  The forward ring waits with partial vmcnt counts, which
# spill traffic would throw off: none allowed.  The backward kernels wait for vmcnt(0) at every step, so a spill
# cannot break them; a few dwords that are stored before the main loop and reloaded after it (the unified
# dK/dV kernel keeps two address pairs that way) are tolerated, anything larger means spills inside the loop.
SCRATCH_LIMIT = {"k_fwd_mfma": 0, "k_bwd_dq": 0, "k_bwd_dkv": 32}


def _check_scratch(remarks: str, src: str) -> None:
    name = None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if not (m and name) or "generic" in name or "reduce" in name:
            continue
        for key, limit in SCRATCH_LIMIT.items():
            if key in name and int(m.group(1)) > limit:
                raise RuntimeError(f"{src}: kernel {name} spills {m.group(1)} bytes/lane to scratch (limit {limit})")


# Scalar loads issued from inline assembly (smem_load in mfma_tiles.h) land behind the compiler's back.  If it
# sees their result as unused it reuses the destination register at once, and if it copies the result before the
# kernel's own wait the copy is stale; either way a kernel could compute an address from garbage.  So the
# generated assembly of every source that uses them is scanned: between such a load and the next
# `s_waitcnt lgkmcnt(0)` (text order) no other instruction may touch the load's destination register.
def _check_scalar_loads(src: str) -> None:
    asm = os.path.join(OBJ, os.path.basename(src) + ".s")
    r = subprocess.run([HIPCC, *FLAGS, "-S", "--cuda-device-only", src, "-o", asm], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc -S failed on {src}")
    ins = [(i, t.strip()) for i, t in enumerate(open(asm).read().split("\n")) if t.strip() and not t.strip().startswith(";")]
    for k, (i, t) in enumerate(ins):
        m = re.match(r"s_load_dword (s\d+),", t)
        if not m:
            continue
        dest = m.group(1)
        for j, u in ins[k + 1:k + 600]:
            if "lgkmcnt(0)" in u:
                break
            if u.startswith("."):
                continue
            ops = u.split(None, 1)
            if len(ops) < 2:
                continue
            used = set()
            for a, b, c in re.findall(r"\bs\[(\d+):(\d+)\]|\b(s\d+)\b", ops[1]):
                used.update([c] if c else [f"s{n}" for n in range(int(a), int(b) + 1)])
            if dest in used:
                raise RuntimeError(f"{src}: line {i + 1} of {asm}: `{t}` -- {dest} is touched by `{u}` (line {j + 1}) "
                                   f"before the load is waited for")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    remarks = [l for l in r.stderr.splitlines() if "remark:" in l]
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(l for l in r.stderr.splitlines() if noise not in l and "remark:" not in l))
    err = "\n".join(l for l in r.stderr.splitlines() if "warning:" in l and noise not in l)
    _check_scratch("\n".join(remarks), src)
    if "smem_load(" in open(src).read():
        _check_scalar_loads(src)
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    """Compile every csrc/*.hip and link liblrsa.so.  Always recompiles."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    return LIB


if __name__ == "__main__":
    build()
