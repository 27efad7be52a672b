"""The C-ABI library loads without a GPU and exports every entry point the header declares."""
import ctypes
import os
import re

import paper_1911_02497_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "condensa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(condensa_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = P.library()
    names = header_functions()
    assert {"condensa_prune", "condensa_filter_prune", "condensa_block_prune", "condensa_quantize",
            "condensa_lc_step"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(P.exported_symbols()) == names


def test_host_only_calls():
    lib = P.library()
    assert lib.condensa_version() >= 100
    assert lib.condensa_status_string(0) == b"ok"
    assert P.condensa_workspace_bytes(3, 100, 0, 1, 1, 0) == 0           # quantize needs none
    assert P.condensa_workspace_bytes(0, 1 << 20, 0, 1, 1, 0) > 0
    assert P.condensa_workspace_bytes(0, 1 << 20, 0, 1, 17, 0) == 0       # too many densities
    assert P.condensa_workspace_bytes(9, 1 << 20, 0, 1, 1, 0) == 0
    assert P.condensa_workspace_bytes(0, 1 << 20, 0, 1, 1, 0) % 256 == 0
    P.condensa_set_option(P.OPT_SELECT_PATH, 1)
    assert P.condensa_get_option(P.OPT_SELECT_PATH) == 1
    P.condensa_set_option(P.OPT_SELECT_PATH, 0)
    try:
        P.condensa_set_option(99, 1)
        raise AssertionError("bad option accepted")
    except P.CondensaError as e:
        assert e.code == -6


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(P.binding.Tensor) == 48
    assert len(P.binding.SELECT_FIELDS) * 8 == 64
