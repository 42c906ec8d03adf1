"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libelattn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    # m0 is on the clobber list of the LDS-DMA asm statements on purpose; clang flags every reserved register there
    "-Wno-inline-asm",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", tmp, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    # The resource remarks are read back: the attention core keeps 32 rows of expanded queries or a quarter of the
    # accumulators in each wavefront's registers, and a change that makes the compiler spill any of them costs a
    # fifth of the kernel's speed without failing a single test.  A spill there fails the build instead.
    res = subprocess.run(cmd + ["-Rpass-analysis=kernel-resource-usage"], stderr=subprocess.PIPE, text=True)
    spilled = check_core_spills(res.stderr)
    lines = res.stderr.splitlines()
    if res.returncode != 0:      # everything but the remarks (each is followed by a source line and a caret)
        skip = 0
        for ln in lines:
            if "remark:" in ln:
                skip = 2
            elif skip:
                skip -= 1
            else:
                print(ln, file=sys.stderr)
    elif verbose:
        for ln in lines:
            if "warning:" in ln or "error:" in ln:
                print(ln, file=sys.stderr)
    sys.stderr.flush()
    if res.returncode != 0:
        raise subprocess.CalledProcessError(res.returncode, cmd)
    if spilled:
        os.remove(tmp)
        raise RuntimeError("register spills in the attention core: " + ", ".join(f"{k}: {v}" for k, v in spilled.items()))
    os.replace(tmp, LIB)
    return LIB


def check_core_spills(remarks: str) -> dict:
    """{kernel name: spilled VGPRs} for the instances of k_core_stream that spill, from hipcc's
    -Rpass-analysis=kernel-resource-usage remarks (a 'Function Name:' line opens each kernel's block)."""
    import re
    out, name = {}, None
    for ln in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", ln)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"VGPRs Spill: (\d+)", ln)
        if m and name and "k_core_stream" in name and int(m.group(1)) > 0:
            out[name] = int(m.group(1))
    return out


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
