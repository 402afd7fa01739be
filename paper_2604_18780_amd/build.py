"""Compile the HIP sources of this package into ``libsemicrf.so`` (gfx950 only)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libsemicrf.so")
SOURCES = [os.path.join(HERE, "csrc", n) for n in ("semicrf.hip", "mscan.hip", "plan.cpp")]
OBJDIR = os.path.join(HERE, "_build")
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
    # packed fp32 VALU forms are not to be generated on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]


def build_library(verbose: bool = False, only=None) -> str:
    """Compile every source (in parallel, one hipcc per translation unit) and link the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    only = [os.path.basename(x) for x in only] if only else None
    jobs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
        objs.append(obj)
        if only is not None and os.path.basename(src) not in only and os.path.exists(obj):
            continue
        # plan.cpp is host-only C++: no offload flags
        flags = FLAGS if src.endswith(".hip") else [f for f in FLAGS if not f.startswith("--offload-arch")][:3] + [FLAGS[-1]]
        jobs.append((src, subprocess.Popen([hipcc] + flags + ["-c", "-o", obj, src], cwd=HERE,
                                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, proc in jobs:
        out, _ = proc.communicate()
        if verbose or proc.returncode != 0:
            print(out)
        failed = failed or proc.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed compiling the sources of libsemicrf.so")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, cwd=HERE,
                         capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed linking libsemicrf.so")
    return LIB


if __name__ == "__main__":
    import sys
    # `python -m paper_2604_18780_amd.build mscan.hip` recompiles only that unit (the others must have been built)
    print(build_library(verbose=True, only=sys.argv[1:] or None))
