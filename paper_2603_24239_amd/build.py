"""Build libdvm.so in-tree with hipcc for gfx950.

    python -m paper_2603_24239_amd.build

Flags: the interpreter is written for gfx950 only; packed-fp32 instructions are disabled
(-packed-fp32-ops); the vector-combine pass is disabled because it splits the 128-bit global
loads of the tile load handler into dword loads; control flow that is uniform across a wave is
left unstructured (the interpreter loop has no lane-divergent branch), which keeps the dispatch
as plain scalar jumps and lets every instruction update its destination registers in place.
"""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdvm.so")

COMMON = ["-O3", "-std=c++20", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument"]
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-mllvm", "-disable-vector-combine", "-mllvm", "-structurizecfg-skip-uniform-regions=1",
          "-mllvm", "-simplifycfg-sink-common=false"]


def variants(which: str = "DVM_VARIANT_LIST"):
    """(K, NR, largest workgroup, waves per SIMD) of every interpreter variant, read from the device source
    (`DVM_CRED_VARIANT_LIST`: those also built as the instantiation that runs reductions along the penultimate axis)."""
    src = open(os.path.join(CSRC, "dvm_vm.hip")).read()
    body = src[src.index(f"#define {which}(X)"):]
    body = body[: body.index("\n\n")]
    out = [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+),\s*(\d+)\)", body)]
    if not out:
        raise RuntimeError("no interpreter variants found in dvm_vm.hip")
    return out


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    vm = os.path.join(CSRC, "dvm_vm.hip")
    jobs = [([hipcc, *COMMON, "-c", os.path.join(CSRC, "dvm_encode.cpp")], os.path.join(CSRC, "dvm_encode.o")),
            ([hipcc, *COMMON, "-c", os.path.join(CSRC, "dvm_fuser.cpp")], os.path.join(CSRC, "dvm_fuser.o")),
            ([hipcc, *COMMON, *DEVICE, "-c", vm], os.path.join(CSRC, "dvm_vm_host.o")),
            ([hipcc, *COMMON, *DEVICE, "-c", os.path.join(CSRC, "dvm_bench.hip")], os.path.join(CSRC, "dvm_bench.o"))]
    # every interpreter variant is a translation unit of its own, compiled side by side
    for k, nr, maxt, waves in variants():
        defs = [f"-DDVM_VARIANT_K={k}", f"-DDVM_VARIANT_NR={nr}", f"-DDVM_VARIANT_MAXT={maxt}", f"-DDVM_VARIANT_WAVES={waves}"]
        jobs.append(([hipcc, *COMMON, *DEVICE, *defs, "-c", vm], os.path.join(CSRC, f"dvm_vm_k{k}_r{nr}.o")))
    for k, nr, maxt, waves in variants():       # (the instantiation for launches whose rows all span whole waves)
        defs = [f"-DDVM_VARIANT_K={k}", f"-DDVM_VARIANT_NR={nr}", f"-DDVM_VARIANT_MAXT={maxt}", f"-DDVM_VARIANT_WAVES={waves}",
                "-DDVM_VARIANT_WIDE=1"]
        jobs.append(([hipcc, *COMMON, *DEVICE, *defs, "-c", vm], os.path.join(CSRC, f"dvm_vm_w_k{k}_r{nr}.o")))
    for k, nr, maxt, waves in variants("DVM_CRED_VARIANT_LIST"):
        defs = [f"-DDVM_VARIANT_K={k}", f"-DDVM_VARIANT_NR={nr}", f"-DDVM_VARIANT_MAXT={maxt}", f"-DDVM_VARIANT_WAVES={waves}",
                "-DDVM_VARIANT_CRED=1"]
        jobs.append(([hipcc, *COMMON, *DEVICE, *defs, "-c", vm], os.path.join(CSRC, f"dvm_vm_c_k{k}_r{nr}.o")))

    # the variants with the most registers take the longest to compile: start them first
    def weight(job):
        m = re.search(r"dvm_vm(?:_c|_w)?_k(\d+)_r(\d+)\.o$", job[1])
        return -(int(m.group(1)) * int(m.group(2))) if m else 0
    jobs.sort(key=weight)

    def run(job):
        cmd, obj = job
        cmd = cmd + ["-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {obj}:\n{err}")
        if verbose and err.strip():
            print(err)
        return obj

    workers = max(1, min(len(jobs), os.cpu_count() or 1, int(os.environ.get("MAX_JOBS", "16"))))
    with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
        objs = list(pool.map(run, jobs))
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
