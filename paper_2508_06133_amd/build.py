"""Compile libkvsched.so (hand-written HIP, gfx950 only) next to this file.

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is installed.

timeline_reg.hip keeps per-timeline state in a block of physical VGPRs (v24 upward) that only
its inline-assembly blocks touch.  That is sound only while the compiler-generated part of those
kernels stays below v24, so the build emits the device assembly of that file and fails if any
compiler-generated instruction of a timeline_reg_kernel names a VGPR of the block.
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
RESERVED_VGPR_BASE = 24  # KVS_PB in timeline_reg.hip


def lib_path() -> str:
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "kvsched.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def reserved_vgpr_violations(asm_text: str, base: int = RESERVED_VGPR_BASE) -> list[str]:
    """Compiler-generated lines inside timeline_reg_kernel bodies that name a VGPR >= base.

    A body runs from the kernel's label to its .Lfunc_end label (s_endpgm may come early, for the
    exits in the prologue); inline assembly sits between the ASMSTART / ASMEND (or APP / NO_APP)
    comment lines the compiler emits around it.
    """
    bad = []
    in_kernel = in_asm = False
    for line in asm_text.splitlines():
        s = line.strip()
        if re.match(r"^_Z\w*timeline_reg_kernel\w*:", s):
            in_kernel, in_asm = True, False
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
        if in_asm or not s or s.startswith((";", ".")):
            continue
        code = s.split(";", 1)[0]
        regs = [int(m) for m in re.findall(r"\bv(\d+)\b", code)]
        for lo, hi in re.findall(r"\bv\[(\d+):(\d+)\]", code):
            regs += [int(lo), int(hi)]
        if any(r >= base for r in regs):
            bad.append(s)
    return bad


def check_reserved_vgprs(hipcc: str, verbose: bool = False) -> None:
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "timeline_reg.s")
        cmd = [hipcc, *DEVICE_FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, "timeline_reg.hip"), "-o", out]
        subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
        text = open(out).read()
    if "timeline_reg_kernel" not in text:
        raise RuntimeError("device assembly of timeline_reg.hip holds no timeline_reg_kernel")
    bad = reserved_vgpr_violations(text)
    if bad:
        raise RuntimeError("compiler-generated code uses the reserved VGPR block (v%d..):\n  " % RESERVED_VGPR_BASE
                           + "\n  ".join(bad[:10]))
    if verbose:
        print("reserved VGPR block untouched by compiler-generated code", flush=True)


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
