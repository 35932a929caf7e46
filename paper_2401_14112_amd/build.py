"""Builds libfp6_mi355x.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile
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
    # the device assembly of the same sources, compiled alongside, for the check of the hand-issued loads
    asm_file = tempfile.NamedTemporaryFile(suffix=".s", delete=False)
    asm_file.close()
    asm_cmd = [c for c in cmd if c not in ("-shared", "-fPIC", "-Rpass-analysis=kernel-resource-usage")]
    asm_cmd[asm_cmd.index("-o") + 1] = asm_file.name
    asm_cmd[1:1] = ["--cuda-device-only", "-S"]
    asm_proc = subprocess.Popen(asm_cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    try:
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        asm_out, _ = asm_proc.communicate()
        lines = r.stdout.splitlines()
        out = "\n".join(l for l in lines if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if asm_proc.returncode != 0:
            raise RuntimeError("hipcc -S failed:\n" + asm_out)
        check_no_scratch(lines)
        with open(asm_file.name) as f:
            check_loads_in_flight(f.read())
    finally:
        if asm_proc.poll() is None:
            asm_proc.kill()
        if os.path.exists(asm_file.name):
            os.unlink(asm_file.name)
        if tmp.exists() and (sys.exc_info()[0] is not None):
            tmp.unlink()
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


_REG = re.compile(r"\b([va])(?:(\d+)|\[(\d+):(\d+)\])")
_VMEM = re.compile(r"^(buffer|global|flat|scratch)_(load|store|atomic)")
_LABEL = re.compile(r"^[A-Za-z_.$][\w.$]*:$")


def _registers(text: str) -> set:
    out = set()
    for m in _REG.finditer(text):
        if m.group(2) is not None:
            out.add((m.group(1), int(m.group(2))))
        else:
            out.update((m.group(1), i) for i in range(int(m.group(3)), int(m.group(4)) + 1))
    return out


def loads_in_flight_problems(asm: str) -> list:
    """The second half of the same rule, checked on the generated code: between a hand-issued load and
    the wait that covers it the compiler believes the destination already holds the data, so it may copy
    it (a loop-carried value it could not keep in place) or reuse it - a stale read, or a late write into
    a register that has a new owner.  Linear scan of every kernel of `asm`: the destinations of vector
    memory loads are in flight until an `s_waitcnt vmcnt(n)` leaves at most n younger requests
    outstanding (they complete in order; stores and copies to LDS count as requests without a
    destination); any instruction that names such a register before that is reported as
    (kernel, line number, instruction, the load).  Code reached only by a jump starts with nothing in
    flight.  One pattern is exempt: the 64-bit multiply-add that the compiler uses for 32-bit address
    arithmetic takes a register pair as addend and leaves its high half undefined, so that half may be
    any register."""
    problems = []
    kernel, queue, after_jump = None, [], False
    for number, raw in enumerate(asm.splitlines(), 1):
        line = raw.split(";")[0].strip()
        if not line:
            continue
        if _LABEL.match(line):
            if not line.startswith(".L"):
                kernel, queue, after_jump = line[:-1], [], False
            elif after_jump:
                queue, after_jump = [], False
            continue
        if line.startswith("."):
            continue
        op = line.split()[0]
        operands = line[len(op):]
        if op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", line)
            if m:
                del queue[:max(0, len(queue) - int(m.group(1)))]
            elif "cnt" not in operands:
                queue = []  # a raw immediate: the compiler writes those for full waits
            continue
        if op in ("s_endpgm", "s_branch", "s_setpc_b64"):
            after_jump = True
            continue
        used = _registers(operands)
        if op in ("v_mad_u64_u32", "v_mad_i64_i32"):
            addend = _registers(operands.split(",")[-1])
            if len(addend) == 2:
                used = (used - addend) | {min(addend)} | _registers(",".join(operands.split(",")[:-1]))
        for dest, what in queue:
            if used & dest:
                problems.append((kernel, number, line, what))
                break
        if _VMEM.match(op):
            dest = set()
            to_lds = operands.split()[-1] == "lds" if operands.split() else False
            if "_load" in op and not to_lds:
                dest = _registers(operands.split(",")[0])
            elif "_atomic" in op and (" sc0" in operands or " glc" in operands):
                dest = _registers(operands.split(",")[0])
            queue.append((dest, "line %d: %s" % (number, line)))
    return problems


def check_loads_in_flight(asm: str) -> None:
    problems = loads_in_flight_problems(asm)
    if problems:
        kernel, number, line, what = problems[0]
        raise RuntimeError("%d instruction(s) touch a register with a load in flight, first in %s, line %d of the "
                           "generated assembly: `%s` (load: %s)" % (len(problems), kernel, number, line, what))


def is_stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    deps = [CSRC / s for s in SOURCES + HEADERS] + [PKG.parent / "include" / h for h in ("fp6.h", "fp6_bench.h")]
    return any(d.stat().st_mtime > t for d in deps)


if __name__ == "__main__":
    build_library(verbose=True, extra_flags=sys.argv[1:])
    print("built", LIB)
