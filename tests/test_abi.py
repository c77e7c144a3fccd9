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
    # host logic of the build: compiler-generated lines inside a timeline_reg_kernel may not
    # name a VGPR of the block its inline assembly owns (v24 upward); asm blocks and other
    # functions are not looked at
    from paper_2508_06133_amd import build

    text = "\n".join([
        "_ZN12_GLOBAL__N_119timeline_reg_kernelILi33ELi4ELb0EEEv9SimParams: ; @x",
        "\tv_add_u32_e32 v31, v1, v2",
        "\t;;#ASMSTART",
        "  v_mov_b32 v[32+kvs_r], 64*kvs_r",
        "v_mov_b32 v40, 0",
        "\t;;#ASMEND",
        "\ts_endpgm",  # an early exit of the prologue: the body goes on to .Lfunc_end
        "\tv_add_u32_e32 v33, v1, v2",
        "\t;APP",
        "v_mov_b32 v41, 0",
        "\t;NO_APP",
        "\tv_mov_b64_e32 v[30:33], 0",
        "\ts_endpgm",
        ".Lfunc_end0:",
        "\tv_mov_b32_e32 v51, 0",
        "_Z5otherv:",
        "\tv_mov_b32_e32 v50, 0",
    ])
    assert build.reserved_vgpr_violations(text, base=32) == ["v_add_u32_e32 v33, v1, v2", "v_mov_b64_e32 v[30:33], 0"]
    assert build.reserved_vgpr_violations(text.replace("v33", "v3").replace("v[30:33]", "v[28:31]"), base=32) == []
