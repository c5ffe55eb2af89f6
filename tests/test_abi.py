"""The C-ABI library loads and exports every symbol include/asl.h declares (no GPU needed)."""
import ctypes
import os
import re
import shutil
import subprocess

from paper_2601_07667_amd import asl as libasl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "asl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(asl_[a-z_]+)\s*\(", text)))


def test_header_symbols_exported():
    names = _declared()
    assert set(names) == set(libasl.EXPORTS)
    lib = libasl.load()
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_sizes_match_header_layout():
    assert ctypes.sizeof(libasl.AslParams) == 72
    assert ctypes.sizeof(libasl.AslState) == 24
    assert ctypes.sizeof(libasl.AslStat) == 40


def test_workspace_bytes_is_host_only_and_monotone():
    lib = libasl.load()
    a = lib.asl_workspace_bytes(32768, 8, 1024)
    b = lib.asl_workspace_bytes(131072, 8, 1024)
    assert 0 < a < b
    assert lib.asl_workspace_bytes(1, 8, 1024) == 0          # invalid limits


def test_header_is_plain_c_and_layouts_agree(tmp_path):
    """include/asl.h compiles as strict C99; a C client sees the struct layouts the ctypes binding
    assumes and can call a host-only entry point of the built library."""
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of the toolchain this repository builds with"
    pkg = os.path.dirname(os.path.abspath(libasl.LIB_PATH))
    exe = str(tmp_path / "abi_client")
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "abi_client.c"), "-o", exe, "-L", pkg, "-lasl",
                    "-Wl,-rpath," + pkg, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split("\n")
    rows = {ln.split()[0]: [int(x) for x in ln.split()[1:]] for ln in out if ln.strip()}
    P, S, R = libasl.AslParams, libasl.AslState, libasl.AslStat
    assert rows["params"] == [ctypes.sizeof(P), P.k_stride_head.offset, P.v_stride_tok.offset, P.scale.offset,
                              P.flags.offset]
    assert rows["state"] == [ctypes.sizeof(S), S.init_set.offset, S.last_layer.offset]
    assert rows["stat"] == [ctypes.sizeof(R), R.rel_var.offset, R.numerator.offset, R.union_size.offset,
                            R.selected.offset]
    assert rows["workspace"] == [libasl.load().asl_workspace_bytes(131072, 9, 1024)]
    assert rows["status"] == [0, -1, -2, -3, -4]
