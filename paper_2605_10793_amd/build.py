"""Build libconqur.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(PKG, "libconqur.so")
SOURCES = ["gemm_nt.hip", "kernels.hip", "head_step.hip", "head_polar.hip", "static_score.hip", "conqur.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-result",
         # fp32/fp64 atomicAdd as the hardware's L2 atomics (device memory is coarse grained);
         # the default lowers them to compare-and-swap loops, which crawl under contention
         "-munsafe-fp-atomics",
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # per-kernel register / scratch report, read below: a GEMM kernel that spills runs at half speed
         "-Rpass-analysis=kernel-resource-usage"]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def kernels_with_scratch(remarks: str):
    """(kernel, bytes per lane) for every kernel the compiler's resource report shows with private scratch memory."""
    found, name = [], None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line and name:
            n = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0].strip())
            if n:
                found.append((name, n))
    return found


def build_lib(verbose: bool = False) -> str:
    """Compile every source (always: this is the 'does it build' check) and link."""
    os.makedirs(OBJ, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, p in procs:
        out, _ = p.communicate()
        spills = kernels_with_scratch(out)
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        for name, nbytes in spills:
            print(f"build.py: WARNING {src}: kernel {name} uses {nbytes} bytes/lane of scratch (register spill)",
                  file=sys.stderr, flush=True)
        if verbose and out.strip():
            print(out)
        objs.append(obj)
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}")
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
