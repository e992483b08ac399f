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
