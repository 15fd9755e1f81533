"""Builds libhmoe.so (HIP, gfx950 only) in-tree, next to this file.

    python paper_2504_05897_amd/build.py

Every source is compiled each time this runs; the library is what the Python binding, the
tests and the benchmark load.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)
import asm_check  # noqa: E402  (a sibling file: this script also runs before the package can be imported)
sys.path.pop(0)
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhmoe.so")

SOURCES = ["api.hip", "route.hip", "permute.hip", "combine.hip", "ffn_reference.hip", "ffn_skinny.hip",
           "ffn_tiled.hip", "ffn_tiled_w4.hip", "schedule.hip"]
HAND_ISSUED_LOADS = ["ffn_tiled.hip"]   # sources whose kernels load into registers from inline assembly

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
        found = re.search(r"Function Name:\s*(\S+)", line)
        if found:
            name = found.group(1)
        found = re.search(r"ScratchSize \[bytes/lane\]:\s*(\d+)", line)
        if found and int(found.group(1)) > 0:
            bad.append(name)
    return bad


def build(verbose: bool = False, extra_flags=()) -> str:
    os.makedirs(BUILD, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = [os.path.join(BUILD, s.replace(".hip", ".o")) for s in SOURCES]
    listings = [os.path.join(BUILD, s.replace(".hip", ".s")) for s in HAND_ISSUED_LOADS]

    def compile_one(pair):
        src, out = pair
        if out.endswith(".s"):   # device assembly, for the in-flight register check below
            return _run([hipcc, *FLAGS, *extra_flags, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", out])
        return _run([hipcc, *FLAGS, "-Rpass-analysis=kernel-resource-usage", *extra_flags, "-c", os.path.join(CSRC, src),
                     "-o", out])

    jobs = list(zip(HAND_ISSUED_LOADS, listings)) + list(zip(SOURCES, objs))
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        logs = list(pool.map(compile_one, jobs))[len(listings):]
    # No register of a load issued from inline assembly may be written, or used as an address, before the wait
    # that covers the load (see asm_check.py).
    # Nor may the compiler put a vector-memory instruction of its own between them, and the hand-counted waits of the
    # main loops are recounted from the listing.
    hazards = []
    for path in listings:
        with open(path) as f:
            text = f.read()
        hazards += asm_check.find_inflight_hazards(text)
        hazards += asm_check.find_wait_count_errors(text)
        os.remove(path)
    if hazards:
        raise RuntimeError("hand-issued loads: the device assembly breaks the rules they rely on:\n  " + "\n  ".join(hazards[:20]))
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
