"""Build libglowq.so (the C-ABI library) for gfx950 with hipcc.

    python paper_2603_25385_amd/csrc/build.py

The library lands in paper_2603_25385_amd/lib/ (git-ignored, in-tree so that a
snapshot of the tree carries it to the GPU machine).  This file is a plain script on
purpose: it must run when the library does not exist yet, so it cannot live
behind the package import, which loads the library.
"""
from __future__ import annotations

import os
import subprocess
import sys

CSRC = os.path.dirname(os.path.abspath(__file__))
LIB_DIR = os.path.join(os.path.dirname(CSRC), "lib")
LIB = os.path.join(LIB_DIR, "libglowq.so")
SOURCES = ["api.hip", "prepare.hip", "proj.hip", "decode.hip", "prefill.hip"]
# packed-fp32 instructions are switched off for device code on purpose
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False, extra: list | None = None) -> str:
    os.makedirs(LIB_DIR, exist_ok=True)
    extra = list(extra or []) + os.environ.get("GLOWQ_EXTRA_HIPCC_FLAGS", "").split()
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(LIB_DIR, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, *(extra or []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                                            text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "is not a recognized feature" not in l)
        if p.returncode != 0:
            failed = True
            print(f"--- {src} failed ---\n{out}", file=sys.stderr)
        elif out.strip() and verbose:
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
