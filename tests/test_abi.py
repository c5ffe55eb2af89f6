"""The C-ABI library loads and exports every symbol include/asl.h declares (no GPU needed)."""
import ctypes
import os
import re

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
