"""Builds libhmoe.so (HIP, gfx950 only) in-tree, next to this file.

    python paper_2504_05897_amd/build.py

Every source is compiled each time this runs; the library is what the Python binding, the
tests and the benchmark load.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhmoe.so")

SOURCES = ["api.hip", "route.hip", "permute.hip", "combine.hip", "ffn_reference.hip", "ffn_skinny.hip",
           "ffn_tiled.hip", "schedule.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def kernels_with_scratch(remarks: str):
    """Kernel names whose resource-usage remarks report private (scratch) memory, i.e. register spills."""
    bad, name = [], None
    for line in remarks.splitlines():
        if "remark:" not in line:
            continue
        text = line.split("remark:", 1)[1]
        if "Function Name:" in text:
            name = text.split("Function Name:", 1)[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in text and int(text.split(":", 1)[1].split("[")[0]) > 0:
            bad.append(name)
    return bad


def build(verbose: bool = False, extra_flags=()) -> str:
    os.makedirs(BUILD, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = [os.path.join(BUILD, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        return _run([hipcc, *FLAGS, "-Rpass-analysis=kernel-resource-usage", *extra_flags, "-c", os.path.join(CSRC, src),
                     "-o", obj])

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        logs = list(pool.map(compile_one, zip(SOURCES, objs)))
    # No kernel of this library may spill registers.  The prefill kernels issue their loads by hand and count the
    # outstanding ones themselves; the compiler treats the destination of such a load as written at once, so under
    # register pressure it may spill and reuse that register before the data lands (observed: a late load then
    # overwrote a pointer and the launch faulted).  A variant that does not fit the register file is a build error.
    spilled = [k for log in logs for k in kernels_with_scratch(log)]
    if spilled:
        raise RuntimeError("kernels that spill registers (private memory) are not allowed:\n  " + "\n  ".join(spilled))
    logs = ["\n".join(l for l in log.splitlines() if "kernel-resource-usage" not in l and not l.lstrip().startswith(("|", "^"))
                      and not l.strip()[:1].isdigit()) for log in logs]
    logs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]))
    if verbose:
        for log in logs:
            if log.strip():
                print(log)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=tuple(sys.argv[1:])))
