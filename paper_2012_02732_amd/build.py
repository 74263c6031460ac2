"""Build libnimble_graph.so (host scheduler + gfx950 kernels) in-tree with hipcc.

Every source is compiled to an object of its own (in parallel) and the objects are linked
into the shared library. ``build()`` recompiles everything; ``build(incremental=True)`` or
``python -m paper_2012_02732_amd.build --incremental`` skips objects that are newer than
their source and every header. ``--knobs`` adds -DNG_MEASUREMENT_KNOBS: the build that reads
the ablation switches from the environment (the product build reads no environment variable).
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libnimble_graph.so")
SOURCES = ["ng_graph.cpp", "ng_schedule.cpp", "ng_launch_graph.cpp", "ng_resident_plan.cpp", "ng_kernels.hip", "ng_runtime.hip"]


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; the HIP library cannot be built")


def _flags(knobs: bool):
    flags = ["-std=c++17", "-O3", "-fPIC", "--offload-arch=gfx950",
             # keep the compiler from forming packed-fp32 instructions
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-function", "-Wno-unused-const-variable",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    if knobs:
        flags.append("-DNG_MEASUREMENT_KNOBS")
    return flags


def build(verbose: bool = True, incremental: bool = False, knobs: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    sources = list(SOURCES)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(CSRC, "*.inc")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    stamp = os.path.join(OBJ, "flags.txt")
    flag_text = " ".join(_flags(knobs))
    if incremental and (not os.path.exists(stamp) or open(stamp).read() != flag_text):
        incremental = False
    jobs = []
    for s in sources:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        # .cpp files are host-only: compile them as plain C++ (no device pass)
        lang = ["-x", "hip"] if s.endswith(".hip") else ["-x", "c++"]
        jobs.append([hipcc()] + _flags(knobs) + lang + ["-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, max(len(jobs), 1))) as pool:
        list(pool.map(run, jobs))
    with open(stamp, "w") as f:
        f.write(flag_text)
    run([hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950"] + [os.path.join(OBJ, s + ".o") for s in sources] + ["-o", LIB])
    return LIB


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv, knobs="--knobs" in sys.argv)
    print("built", LIB)
    sys.exit(0)
