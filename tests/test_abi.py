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


def test_bench_refuses_more_than_one_gpu():
    """Only the one-GPU path exists: asking for more must end with a message, before anything touches a GPU."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_workspace_sizes_are_monotone_and_cover_the_documented_cases():
    from paper_1911_02497_amd import binding as B
    lib = B.library()
    n = 1207959552
    big = lib.condensa_workspace_bytes(B.OP_LC_STEP, n, 0, 64, 1, B.SCOPE_GLOBAL)
    assert 0.5e9 < big < 1.0e9                         # candidate capacity N/32 x 28 B dominates
    assert lib.condensa_workspace_bytes(B.OP_LC_STEP, n // 2, 0, 64, 1, B.SCOPE_GLOBAL) < big
    assert lib.condensa_workspace_bytes(B.OP_PRUNE, n, 0, 64, 16, B.SCOPE_GLOBAL) > 0
    assert lib.condensa_workspace_bytes(B.OP_PRUNE, n, 0, 64, 17, B.SCOPE_GLOBAL) == 0      # too many densities
    assert lib.condensa_workspace_bytes(B.OP_QUANTIZE, n, 0, 1, 1, B.SCOPE_GLOBAL) == 0      # needs none
    assert lib.condensa_workspace_bytes(99, n, 0, 1, 1, B.SCOPE_GLOBAL) == 0
