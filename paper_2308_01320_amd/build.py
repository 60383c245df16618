"""Builds libhe.so (the C-ABI engine) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhe.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # keep the compiler from forming packed-fp32 instructions (v_pk_*_f32)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # per-kernel register / scratch report, scanned below: a kernel that spills registers to scratch
    # memory is a performance bug here (it has happened silently to one launch shape)
    "-Rpass-analysis=kernel-resource-usage",
    # the first kernel arguments (the operand pointers and sizes) arrive in scalar registers with the launch
    # instead of being loaded by the kernel's first instructions: each kernel starts its loads ~0.4 us earlier
    "-mllvm", "-amdgpu-kernarg-preload-count=12",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, jobs: int = 8) -> str:
    """Compiles every .hip source and links libhe.so next to this file."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()
    procs = []
    objs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [cc, *FLAGS, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _wait(procs, verbose)
    _wait(procs, verbose)
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def _wait(procs, verbose):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        lines = out.splitlines()
        # the resource report: remember which kernels use scratch memory, drop the rest of it
        spilled, name = [], "?"
        for l in lines:
            if "remark: Function Name:" in l:
                name = l.split("Function Name:")[1].split("[")[0].strip()
            elif "remark:     ScratchSize [bytes/lane]:" in l:
                if int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0]) > 0:
                    spilled.append(name)
        keep, skip = [], 0
        for l in lines:
            # hipcc's host pass does not know the packed-fp32 feature name: harmless
            if "packed-fp32-ops" in l:
                continue
            if "[-Rpass-analysis=kernel-resource-usage]" in l:
                skip = 2  # the remark and the two source-context lines after it
                continue
            if skip:
                skip -= 1
                continue
            keep.append(l)
        out = "\n".join(keep)
        if out.strip() and (verbose or p.returncode):
            print(out)
        if p.returncode:
            raise RuntimeError(f"hipcc failed on {src}")
        if spilled:
            raise RuntimeError(f"{os.path.basename(src)}: kernels spilling registers to scratch memory: " + ", ".join(spilled))


if __name__ == "__main__":
    build()
    print(LIB)
