"""Builds libfp6_mi355x.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libfp6_mi355x.so"
SOURCES = ["fp6_api.hip"]
HEADERS = ["fp6_device.hpp", "linear_stream.hpp", "linear_tiled.hpp", "pack_unpack.hpp"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_library(verbose: bool = False, extra_flags=()) -> Path:
    """Always compiles (the caller decides when); returns the path of the shared library."""
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [
        hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
        # packed-fp32 VALU forms are kept out of the generated code on this target
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function", "-Rpass-analysis=kernel-resource-usage",
        *extra_flags,
        "-I", str(PKG.parent / "include"),
        *[str(CSRC / s) for s in SOURCES],
        "-o", str(tmp),
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = r.stdout.splitlines()
    out = "\n".join(l for l in lines if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    check_no_scratch(lines)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


def check_no_scratch(remarks) -> None:
    """The pipelined kernels issue loads from inline assembly and rely on the loaded registers staying
    where they are until the explicit wait; a register spilled to scratch in between would save stale
    data.  Refuse a build in which any kernel of the library needs scratch memory."""
    name = None
    for line in remarks:
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size != 0:
                raise RuntimeError("kernel %s spills %d bytes/lane to scratch; reduce its register pressure" % (name, size))


def is_stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    deps = [CSRC / s for s in SOURCES + HEADERS] + [PKG.parent / "include" / "fp6.h"]
    return any(d.stat().st_mtime > t for d in deps)


if __name__ == "__main__":
    build_library(verbose=True, extra_flags=sys.argv[1:])
    print("built", LIB)
