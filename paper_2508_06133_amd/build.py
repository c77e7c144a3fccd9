"""Compile libkvsched.so (hand-written HIP, gfx950 only) next to this file.

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is installed.

timeline_reg.hip keeps per-timeline state in a block of physical VGPRs (v30 upward) that only
its inline-assembly blocks touch.  That is sound only while everything the compiler allocates in those
kernels (its own code and the operand registers it hands to the assembly statements) stays below v30,
so the build emits the device assembly of that file and fails if a timeline_reg_kernel names a VGPR of
the block anywhere but in the hand-written row code, or if it did not see every instantiation.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvsched.so")
SOURCES = ["api.hip", "simulate.hip", "timeline_reg.hip", "sortedf.hip", "localswap.hip", "exactdp.hip", "horizon.hip", "permute.hip", "prefix.hip", "online.hip", "predicted.hip"]
DEVICE_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    # packed fp32 instructions are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
FLAGS = DEVICE_FLAGS + ["-fPIC", "-shared", "-Wall", "-Wno-unused-function"]
RESERVED_VGPR_BASE = 30  # KVS_PB in timeline_reg.hip


def lib_path() -> str:
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "kvsched.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def timeline_reg_instantiations() -> int:
    """Kernel instantiations kvs_launch_simulate_reg can reach: one per launch statement of launch_reg
    and profile-file size."""
    src = open(os.path.join(CSRC, "timeline_reg.hip")).read()
    launches = len(re.findall(r"hipLaunchKernelGGL\(\(timeline_reg_kernel<NR, (?:WPB|1),", src))
    sizes = len(re.findall(r"return launch_reg<\d+, \d+>\(p, st\);", src))
    return launches * sizes


def reserved_vgpr_scan(asm_text: str, base: int = RESERVED_VGPR_BASE) -> tuple[list[str], int]:
    """(offending lines, kernel bodies scanned) for the timeline_reg_kernel bodies of a device assembly.

    The profile block of an instantiation with NR rows (read off the kernel's mangled name) is
    v[base, base + NR).  It belongs to the hand-written assembly alone, which names it only as
    v[<base>+...].  Offending are therefore: a compiler-generated line that names a VGPR of the block in
    any form, and a line INSIDE an assembly statement that names one as plain vN or v[a:b] -- an operand
    register the compiler substituted (temporaries and inputs of the statements must lie outside the
    block as well).  A body runs from the kernel's label to its .Lfunc_end label (s_endpgm may come
    early, for the exits in the prologue); inline assembly sits between the ASMSTART / ASMEND (or APP /
    NO_APP) comment lines the compiler emits around it.
    """
    bad = []
    bodies = 0
    in_kernel = in_asm = False
    top = base
    for line in asm_text.splitlines():
        s = line.strip()
        m = re.match(r"^_Z\w*timeline_reg_kernelILi(\d+)E\w*:", s)
        if m:
            in_kernel, in_asm = True, False
            top = base + int(m.group(1))
            bodies += 1
            continue
        if not in_kernel:
            continue
        if s.startswith(".Lfunc_end"):
            in_kernel = False
            continue
        if s.startswith((";;#ASMSTART", ";APP", "#APP")):
            in_asm = True
            continue
        if s.startswith((";;#ASMEND", ";NO_APP", "#NO_APP")):
            in_asm = False
            continue
        if not s or s.startswith(";") or (not in_asm and s.startswith(".")):
            continue
        code = s.split(";", 1)[0]
        regs = [(int(m), int(m)) for m in re.findall(r"\bv(\d+)\b", code)]
        regs += [(int(lo), int(hi)) for lo, hi in re.findall(r"\bv\[(\d+):(\d+)\]", code)]
        if any(lo < top and hi >= base for lo, hi in regs):
            bad.append(s)
    return bad, bodies


def reserved_vgpr_violations(asm_text: str, base: int = RESERVED_VGPR_BASE) -> list[str]:
    return reserved_vgpr_scan(asm_text, base)[0]


def emit_timeline_reg_assembly(hipcc: str) -> str:
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "timeline_reg.s")
        cmd = [hipcc, *DEVICE_FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, "timeline_reg.hip"), "-o", out]
        subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
        return open(out).read()


def check_reserved_vgprs(hipcc: str, verbose: bool = False) -> None:
    bad, bodies = reserved_vgpr_scan(emit_timeline_reg_assembly(hipcc))
    want = timeline_reg_instantiations()
    if bodies != want or want == 0:
        raise RuntimeError(f"scanned {bodies} timeline_reg_kernel bodies, the launcher can reach {want}")
    if bad:
        raise RuntimeError("the reserved VGPR block (v%d..) is named outside the hand-written row code:\n  "
                           % RESERVED_VGPR_BASE + "\n  ".join(bad[:10]))
    if verbose:
        print(f"reserved VGPR block untouched in all {bodies} timeline_reg_kernel bodies", flush=True)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc, *FLAGS, *[os.path.join(CSRC, f) for f in SOURCES], "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    try:
        check_reserved_vgprs(hipcc, verbose)
    except Exception:
        os.remove(tmp)
        raise
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
