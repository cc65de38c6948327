"""Builds libdsattn.so in-tree with hipcc for gfx950 (no JIT, no torch extension)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdsattn.so")
# the same library with the in-kernel stage stamps compiled in (bench.py --trace loads it)
LIB_TRACE = os.path.join(HERE, "libdsattn_trace.so")
SOURCES = ["ds_select.hip", "ds_attend.hip", "ds_misc.hip", "ds_api.cpp"]
HEADERS = ["ds_internal.h", "ds_device.h", "ds_attend_core.h"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 VALU forms are kept off for every device function of the library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", "ds_attn.h")]
    return any(os.path.getmtime(p) > t for p in deps)


def build(verbose: bool = True, trace: bool = False) -> str:
    """Compile every source and link the shared library; always recompiles.  With `trace` the
    stage-stamp variant (-DDS_TRACE) is built instead, into LIB_TRACE."""
    cc = hipcc()
    objs = []
    bdir = os.path.join(HERE, "_build", "trace" if trace else "plain")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src + ".o")
        cmd = [cc] + FLAGS + (["-DDS_TRACE"] if trace else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if src.endswith(".cpp"):
            cmd.insert(1, "-x"); cmd.insert(2, "hip")
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd)))
        objs.append(obj)
    for src, p in procs:
        if p.wait() != 0:
            raise RuntimeError(f"hipcc failed on {src}")
    lib = LIB_TRACE if trace else LIB
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(trace="--trace" in sys.argv[1:]))
