"""Build libkeydiff.so (gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkeydiff.so")
SOURCES = ["attention.hip", "evict.hip", "keydiff_abi.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-ffp-contract=off",   # the deciding score is plain IEEE double arithmetic
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-Rpass-analysis=kernel-resource-usage",   # the compiler reports every kernel's registers and scratch: checked below
]


TIMELINE_LIB = os.path.join(HERE, "libkeydiff_timeline.so")


def scratch_users(remarks):
    """(kernel, bytes per lane) of every kernel whose resource-usage remarks report scratch memory."""
    found, name = [], None
    for l in remarks:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in l:
            n = int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if n:
                found.append((name, n))
    return found


def build(verbose: bool = False, timeline: bool = False) -> str:
    """timeline=True builds the profiling variant (libkeydiff_timeline.so, -DKD_TIMELINE: wall-clock stamps
    inside step_main and the carried selection, read by `python -m paper_2504_15364_amd.timeline`)."""
    objs = []
    procs = []
    extra = ["-DKD_TIMELINE"] if timeline else []
    suffix = ".timeline.o" if timeline else ".o"
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", suffix))
        cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        lines = out.splitlines()
        spilled = scratch_users(lines)
        out = "\n".join(l for l in lines if "not a recognized feature" not in l and "kernel-resource-usage" not in l)
        if p.returncode:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if spilled and timeline:
            # (the stamps cost registers: tolerated in the profiling build, whose timings of such a kernel do not count)
            print(f"warning: {src}: kernels that use scratch memory in the profiling build: "
                  + ", ".join(f"{k} ({b} bytes/lane)" for k, b in spilled), file=sys.stderr)
        elif spilled:
            # A kernel that touches scratch memory (spilled registers, or a parameter block the compiler
            # could not keep in registers) runs several times slower on this chip (measured: 4x on the
            # generation-phase attention, 30x on the ordered shift): refuse to build one.
            raise RuntimeError(f"{src}: kernels that use scratch memory: " + ", ".join(f"{k} ({b} bytes/lane)" for k, b in spilled))
        if verbose and out.strip():
            print(out)
    lib = TIMELINE_LIB if timeline else LIB
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    subprocess.run(link, check=True)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, timeline="--timeline" in sys.argv))
