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
SOURCES = ["api.hip", "prepare.hip", "proj.hip", "decode.hip", "prefill.hip", "probe.hip", "factorize.hip", "mx.hip"]
# packed-fp32 instructions are switched off for device code on purpose
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Rpass-analysis=kernel-resource-usage"]
# Per-file flags.  decode.hip: matrix-instruction results stay in ordinary vector registers
# (the few-token kernels issue one correction product per workgroup; with it in an
# accumulation register the 2- and 4-token kernels measured 4-7 % slower).
FILE_FLAGS = {"decode.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}
# Kernels that count their own outstanding memory operations (hand-placed s_waitcnt): a
# register spill would add loads of the compiler's to that count, so they must have none.
NO_SPILL = ("k_prefill",)


def check_no_spills(src: str, remarks: str) -> None:
    name = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].strip()
        elif "AGPRs:" in line and name and any(k in name for k in NO_SPILL):
            # values parked in accumulation registers are copies too, and a copy of a
            # register whose load is still in flight (hand-counted waits) reads garbage
            if int(line.split("AGPRs:")[1].split()[0]):
                raise RuntimeError(f"{src}: {name} uses accumulation registers; this kernel "
                                   "must keep everything in vector registers")
        elif "ScratchSize [bytes/lane]:" in line and name:
            n = int(line.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if n and any(k in name for k in NO_SPILL):
                raise RuntimeError(f"{src}: {name} uses {n} bytes of scratch per lane (register "
                                   "spills); this kernel must not spill")


def build(verbose: bool = False, extra: list | None = None) -> str:
    os.makedirs(LIB_DIR, exist_ok=True)
    extra = list(extra or []) + os.environ.get("GLOWQ_EXTRA_HIPCC_FLAGS", "").split()
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(LIB_DIR, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, *FILE_FLAGS.get(src, []), *(extra or []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                                            text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        check_no_spills(src, out)
        out = "\n".join(l for l in out.splitlines()
                        if "is not a recognized feature" not in l and "remark:" not in l)
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
