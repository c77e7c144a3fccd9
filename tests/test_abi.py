"""The C-ABI library loads and exports every symbol the header declares (no compute calls)."""
import ctypes
import os
import re

from conftest import ROOT


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "kvsched.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvsched_[a-zA-Z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_calls():
    names = _declared_functions()
    for must in ("kvsched_simulate", "kvsched_sortedF", "kvsched_best_neighbor", "kvsched_create", "kvsched_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2508_06133_amd import build

    assert os.path.exists(build.lib_path()), "libkvsched.so has not been built"
    lib = ctypes.CDLL(build.lib_path())
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_strerror_needs_no_gpu():
    from paper_2508_06133_amd import build

    lib = ctypes.CDLL(build.lib_path())
    lib.kvsched_strerror.restype = ctypes.c_char_p
    assert lib.kvsched_strerror(0) == b"ok"
    assert b"range" in lib.kvsched_strerror(-2)


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_06133_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src, f


def test_reserved_vgpr_scan_of_the_build():
    # host logic of the build: inside a timeline_reg_kernel with NR profile rows nothing but the
    # hand-written row code (v[<base>+...]) may name a VGPR of the block v[base, base + NR): neither a
    # compiler-generated line nor an operand register substituted into an assembly statement; other
    # functions are not looked at
    from paper_2508_06133_amd import build

    text = "\n".join([
        "_ZN12_GLOBAL__N_119timeline_reg_kernelILi9ELi4ELb0ELb0ELb0EEEv9SimParams: ; @x",
        "\tv_add_u32_e32 v31, v1, v2",
        "\t;;#ASMSTART",
        "  v_mov_b32 v[32+kvs_r], 64*kvs_r",
        "v_sub_u32 v40, s3, v14",  # an operand of the statement inside the block
        "v_sub_u32 v41, s3, v14",  # just above the block of 9 rows: allowed
        "\t;;#ASMEND",
        "\ts_endpgm",  # an early exit of the prologue: the body goes on to .Lfunc_end
        "\tv_add_u32_e32 v33, v1, v2",
        "\t;APP",
        "v_mov_b32 v3, 0",
        "\t;NO_APP",
        "\tv_mov_b64_e32 v[30:33], 0",
        "\tv_mov_b64_e32 v[41:42], 0",
        "\ts_endpgm",
        ".Lfunc_end0:",
        "\tv_mov_b32_e32 v35, 0",
        "_Z5otherv:",
        "\tv_mov_b32_e32 v36, 0",
    ])
    bad, bodies = build.reserved_vgpr_scan(text, base=32)
    assert bodies == 1
    assert bad == ["v_sub_u32 v40, s3, v14", "v_add_u32_e32 v33, v1, v2", "v_mov_b64_e32 v[30:33], 0"]
    clean = text.replace("v40", "v4").replace("v33", "v3").replace("v[30:33]", "v[28:31]")
    assert build.reserved_vgpr_scan(clean, base=32) == ([], 1)


def test_build_scans_every_instantiation_of_the_register_kernel():
    # on the real emitted assembly: as many kernel bodies scanned as the launcher can reach (five
    # profile-file sizes x five launch statements), none of them touching its block
    import os as _os

    from paper_2508_06133_amd import build

    assert build.timeline_reg_instantiations() == 25
    text = build.emit_timeline_reg_assembly(_os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"))
    bad, bodies = build.reserved_vgpr_scan(text)
    assert bodies == 25 and bad == []
