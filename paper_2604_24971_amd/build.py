"""Builds libpolykv.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2604_24971_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpolykv.so")
SOURCES = ["polykv_api.hip", "polykv_codec.hip", "polykv_attend.hip", "polykv_attend_mfma.hip"]
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed-fp32 VALU forms stay off on these machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), r.stdout))
    return r.stdout


def _check_no_scratch(remarks: str):
    """The matrix-core attention kernel keeps its accumulators, parked query operands and score tiles in all 512
    registers of a wave; builds in which the register allocator spilled part of that to scratch memory returned
    wrong results on the GPU.  Refuse such a build: every instantiation must come out without scratch."""
    name = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize" in line and name and "attend_mfma_kernel" in name:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size and not os.environ.get("POLYKV_BUILD_ALLOW_SCRATCH"):   # (the variable is for timing experiments only)
                raise RuntimeError("%s spills %d bytes per lane to scratch: reduce its register use" % (name, size))


def build_library(verbose: bool = True, extra_flags=()) -> str:
    """Compile every source and link the shared library; always recompiles."""
    hipcc = _hipcc()
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(i):
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, SOURCES[i]), "-o", objs[i]]
        if SOURCES[i] == "polykv_attend_mfma.hip":
            log = _run(cmd + ["-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics"])
            _check_no_scratch(log)
            return "\n".join(l for l in log.splitlines() if "kernel-resource-usage" not in l)
        return _run(cmd)

    with ThreadPoolExecutor(max_workers=4) as ex:
        logs = list(ex.map(compile_one, range(len(SOURCES))))
    logs.append(_run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB]))
    if verbose:
        for log in logs:
            if log.strip():
                print(log, file=sys.stderr)
        print("built", LIB, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build_library()
