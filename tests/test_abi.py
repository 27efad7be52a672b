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


def test_argument_errors_are_found_on_the_host_before_any_launch():
    """Bad arguments must come back as a status before anything touches a GPU (so these run without one)."""
    from paper_1911_02497_amd import binding as B
    lib = B.library()
    null = None
    fake = ctypes.c_void_p(256)                          # never dereferenced: the calls fail first
    for fn in (lib.condensa_quantize, lib.condensa_quantize_bf16):
        assert fn(null, 4, fake, fake, null) == -1                       # x missing
        assert fn(fake, 4, null, null, null) == -1                       # no output wanted
        assert fn(fake, (3 << 32) + 1, fake, null, null) == -2           # too many elements
        assert fn(null, 0, null, null, null) == 0                        # nothing to do
    for fmt in (0, 1):
        assert lib.condensa_quantize_fp8(null, 4, fmt, fake, fake, null) == -1
        assert lib.condensa_quantize_fp8(fake, 4, fmt, null, null, null) == -1
        assert lib.condensa_quantize_fp8(fake, (3 << 32) + 1, fmt, fake, null, null) == -2
        assert lib.condensa_quantize_fp8(null, 0, fmt, null, null, null) == 0
        assert lib.condensa_dequantize_fp8(null, 4, fmt, fake, null) == -1
        assert lib.condensa_dequantize_fp8(null, 0, fmt, null, null) == 0
    assert lib.condensa_quantize_fp8(fake, 4, 2, fake, fake, null) == -6          # unknown format
    assert lib.condensa_dequantize_fp8(fake, 4, -1, fake, null) == -6
    for fn in (lib.condensa_dequantize, lib.condensa_dequantize_bf16):
        assert fn(null, 4, fake, null) == -1
        assert fn(fake, 4, null, null) == -1
        assert fn(null, 0, null, null) == 0
    t = (B.Tensor * 1)()
    t[0].w = 256
    t[0].shape[0] = 16
    t[0].ndim = 1
    dens = (ctypes.c_double * 1)(0.5)
    res = ctypes.c_void_p(512)
    ws = ctypes.c_void_p(4096)
    # density out of range, too many densities, bad scope, workspace too small / misaligned / missing
    bad = (ctypes.c_double * 1)(1.5)
    assert lib.condensa_prune(t, 1, bad, 1, 0, null, null, null, res, ws, 1 << 30, null) == -3
    assert lib.condensa_prune(t, 1, dens, 17, 0, null, null, null, res, ws, 1 << 30, null) == -2
    assert lib.condensa_prune(t, 1, dens, 1, 7, null, null, null, res, ws, 1 << 30, null) == -6
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, res, ws, 16, null) == -5
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, res, ctypes.c_void_p(4100), 1 << 30, null) == -5
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, res, null, 1 << 30, null) == -5
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, null, ws, 1 << 30, null) == -1
    t[0].ndim = 5
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, res, ws, 1 << 30, null) == -4
    t[0].ndim = 1
    # filter pruning wants 4-D tensors, block pruning 2-D ones whose dimensions the block divides
    assert lib.condensa_filter_prune(t, 1, 0.5, 0, null, null, null, null, null, null, res, ws, 1 << 30, null) == -4
    t[0].shape[0], t[0].shape[1], t[0].ndim = 6, 8, 2
    assert lib.condensa_block_prune(t, 1, 4, 4, 0.5, 0, null, null, null, null, null, null, res, ws, 1 << 30, null) == -4
    assert lib.condensa_block_prune(t, 1, 0, 4, 0.5, 0, null, null, null, null, null, null, res, ws, 1 << 30, null) == -4
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        assert len(lib.condensa_status_string(code)) > 0
