"""Build libdvm.so in-tree with hipcc for gfx950.

    python -m paper_2603_24239_amd.build

Flags: the interpreter is written for gfx950 only; packed-fp32 instructions are disabled
(-packed-fp32-ops); the vector-combine pass is disabled because it splits the 128-bit global
loads of the tile load handler into dword loads; control flow that is uniform across a wave is
left unstructured (the interpreter loop has no lane-divergent branch), which keeps the dispatch
as plain scalar jumps and lets every instruction update its destination registers in place.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdvm.so")

COMMON = ["-O3", "-std=c++20", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument"]
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-mllvm", "-disable-vector-combine", "-mllvm", "-structurizecfg-skip-uniform-regions=1",
          "-mllvm", "-simplifycfg-sink-common=false"]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    for src, extra in (("dvm_encode.cpp", []), ("dvm_fuser.cpp", []), ("dvm_vm.hip", DEVICE)):
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err)
        objs.append(obj)
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
