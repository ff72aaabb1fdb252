"""Build libkvfuse.so (the product) and libkvfuse_probe.so (machine probes for benchmarks) in-tree with hipcc, for
gfx950 only.  No JIT, no torch extension machinery."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvfuse.so")
PROBE_LIB = os.path.join(HERE, "libkvfuse_probe.so")
SOURCES = ["host.hip", "norms.hip", "similarity.hip", "assign.hip", "merge.hip", "rewrite.hip", "decode.hip", "decode_shared.hip", "prefill.hip", "threshold.hip", "variants.hip"]
PROBE_SOURCES = ["probe.hip"]
# packed-fp32 instructions are switched off for every device object of this library
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, jobs: int = 8) -> str:
    """Compile every source (always; the caller decides when) and link the shared library."""
    hipcc = _hipcc()
    objs = []

    def one(src):
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(one, SOURCES + PROBE_SOURCES))
    for lib, part in ((LIB, objs[:len(SOURCES)]), (PROBE_LIB, objs[len(SOURCES):])):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *part]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB, PROBE_LIB)
