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
    assert P.condensa_config().select_path == 1          # a fresh config starts from the process-wide defaults
    P.condensa_set_option(P.OPT_SELECT_PATH, 0)
    assert P.condensa_config().select_path == 0
    try:
        P.condensa_set_option(99, 1)
        raise AssertionError("bad option accepted")
    except P.CondensaError as e:
        assert e.code == -6


def test_per_call_configuration():
    """The knobs travel with the call: a config sizes the workspace and is validated like the defaults'
    setter, and nothing process-wide changes."""
    from paper_1911_02497_amd import binding as B
    lib = B.library()
    assert ctypes.sizeof(B.Config) == 32
    c = P.condensa_config()
    assert (c.select_path, c.sample_log2, c.window_margin, c.cand_shift, c.profile, c.apply_threads, c.fused_sweep) == \
        (0, 0, P.WINDOW_MARGIN_DEFAULT, 0, 0, 0, 0)
    base = P.condensa_workspace_bytes(B.OP_PRUNE, 1 << 28, 0, 4, 1, B.SCOPE_GLOBAL)
    assert P.condensa_workspace_bytes(B.OP_PRUNE, 1 << 28, 0, 4, 1, B.SCOPE_GLOBAL, P.condensa_config()) == base
    small = P.condensa_workspace_bytes(B.OP_PRUNE, 1 << 28, 0, 4, 1, B.SCOPE_GLOBAL, {"sample_log2": 12, "cand_shift": 8})
    assert 0 < small < base
    assert P.condensa_get_option(P.OPT_SAMPLE_LOG2) == 0 and P.condensa_get_option(P.OPT_CAND_SHIFT) == 0
    # invalid fields: the size query answers 0, the calls CONDENSA_ERR_ARG, before anything else is looked at
    t = (B.Tensor * 1)()
    t[0].w, t[0].shape[0], t[0].ndim = 1 << 40, 16, 1
    dens = (ctypes.c_double * 1)(0.5)
    res, ws = ctypes.c_void_p(1 << 41), ctypes.c_void_p(1 << 42)
    for field, value in (("select_path", 3), ("sample_log2", 5), ("cand_shift", 31), ("profile", 1 << 5),
                         ("apply_threads", 96), ("fused_sweep", 2), ("window_margin", -1), ("reserved", 1)):
        c = P.condensa_config()
        setattr(c, field, value)
        assert lib.condensa_workspace_bytes(B.OP_PRUNE, 1 << 20, 0, 1, 1, 0, ctypes.byref(c)) == 0, field
        assert lib.condensa_prune(t, 1, dens, 1, 0, None, None, None, res, ws, 1 << 30, None, ctypes.byref(c)) == -6, field
        assert lib.condensa_lc_step(t, 1, None, None, 1e-3, 0.5, None, None, None, res, ws, 1 << 30, None,
                                    ctypes.byref(c)) == -6, field


def test_overlapping_buffers_are_rejected():
    """Byte ranges are compared, not start addresses: an output that overlaps an input at an offset, two
    outputs that share bytes, a workspace laid over a tensor.  The calls that pass the check get a workspace
    size of 16 bytes and stop at CONDENSA_ERR_WORKSPACE, still before any launch."""
    from paper_1911_02497_amd import binding as B
    lib = B.library()
    n = 1000
    W, LAM, A, Bf, C, D, E = (x << 40 for x in range(1, 8))       # far apart: never dereferenced
    res, ws = ctypes.c_void_p(1 << 50), ctypes.c_void_p(1 << 51)
    tiny = 16

    def table(*ptrs):
        arr = (ctypes.c_void_p * len(ptrs))(*ptrs)
        return ctypes.cast(arr, ctypes.c_void_p), arr

    t = (B.Tensor * 1)()
    t[0].w, t[0].shape[0], t[0].ndim = W, n, 1
    dens = (ctypes.c_double * 2)(0.5, 0.25)

    def prune(theta=None, f16=None, mask=None, J=1, workspace=ws, results=res, ws_bytes=tiny):
        tabs = [table(*(x if isinstance(x, tuple) else (x,))) if x is not None else (None, None) for x in (theta, f16, mask)]
        return lib.condensa_prune(t, 1, dens, J, 0, tabs[0][0], tabs[1][0], tabs[2][0], results, workspace, ws_bytes, None, None)

    assert prune(theta=A, f16=Bf, mask=C) == -5                   # disjoint: passes the check
    assert prune(theta=W) == -5                                   # exact in-place form, one density
    assert prune(theta=(W, A), J=2) == -6                         # in place with two densities
    assert prune(theta=W + 16) == -6                              # theta laid over the weights at an offset
    assert prune(theta=W - 4 * n + 4) == -6                       # ... ending inside them
    assert prune(mask=W + 4 * n - 1) == -6                        # last byte of the weights
    assert prune(mask=W + 4 * n) == -5                            # directly behind them: fine
    assert prune(f16=W + 2) == -6
    assert prune(theta=A, mask=A + 400) == -6                     # two outputs share bytes
    assert prune(theta=(A, A + 4), J=2) == -6                     # thetas of two densities overlap
    assert prune(theta=W, mask=W) == -6                           # in-place theta and a mask over it
    assert prune(theta=A, workspace=ctypes.c_void_p(W - 256), ws_bytes=1 << 30) == -6   # workspace over the weights
    assert prune(theta=A, workspace=ctypes.c_void_p(W - 256)) == -5          # the 16 bytes it claims end before them
    assert prune(theta=A, results=ctypes.c_void_p(A + 8)) == -6   # record inside an output
    # two tensors: the output of one over the input of the other
    t2 = (B.Tensor * 2)()
    t2[0].w, t2[0].shape[0], t2[0].ndim = W, n, 1
    t2[1].w, t2[1].shape[0], t2[1].ndim = LAM, n, 1
    th, keep = table(A, W + 8)
    assert lib.condensa_prune(t2, 2, dens, 1, 0, th, None, None, res, ws, tiny, None, None) == -6
    th, keep = table(A, Bf)
    assert lib.condensa_prune(t2, 2, dens, 1, 0, th, None, None, res, ws, tiny, None, None) == -5

    def lc(lam=LAM, lam_out=A, theta=Bf, grad=C, mask=D, f16=None, nnz=None):
        tabs = {k: table(v) if v is not None else (None, None) for k, v in
                dict(lam=lam, lam_out=lam_out, theta=theta, grad=grad, mask=mask, f16=f16).items()}
        if f16 is None:
            return lib.condensa_lc_step(t, 1, tabs["lam"][0], tabs["lam_out"][0], 1e-3, 0.5, tabs["theta"][0],
                                        tabs["grad"][0], tabs["mask"][0], res, ws, tiny, None, None)
        return lib.condensa_lc_step_pq(t, 1, tabs["lam"][0], tabs["lam_out"][0], 1e-3, 0.5, tabs["theta"][0],
                                       tabs["f16"][0], tabs["grad"][0], tabs["mask"][0], nnz, res, ws, tiny, None, None)

    assert lc() == -5
    assert lc(lam_out=None) == -5                                 # lambda updated in place
    assert lc(lam_out=LAM) == -5                                  # the same, spelled out
    assert lc(grad=A) == -6                                       # grad and lambda_out are one buffer
    assert lc(theta=C) == -6                                      # theta and grad are one buffer
    assert lc(theta=W + 4) == -6
    assert lc(lam_out=LAM + 4) == -6                              # lambda_out over lambda at an offset
    assert lc(lam=W, lam_out=None) == -6                          # in-place multipliers that are the weights
    assert lc(lam=W + 4 * n - 4, lam_out=None) == -6              # in-place multipliers overlap the weights
    assert lc(lam=W + 4 * n - 4) == -5                            # read-only overlap of two inputs corrupts nothing
    assert lc(mask=LAM + 100) == -6
    assert lc(f16=E) == -5
    assert lc(f16=Bf + 2) == -6
    assert lc(f16=E, nnz=ctypes.c_void_p(E + 2 * n)) == -5          # the count directly behind the codes: fine
    assert lc(f16=E, nnz=ctypes.c_void_p(E + 2 * n - 8)) == -6      # ... inside them

    # structure pruning: in-place theta is allowed, everything else must be disjoint
    t4 = (B.Tensor * 1)()
    t4[0].w, t4[0].ndim = W, 4
    t4[0].shape[0], t4[0].shape[1], t4[0].shape[2], t4[0].shape[3] = 10, 4, 5, 5

    def fp(theta=None, mask=None, sumsq=None, norms=None, keep_idx=None, smask=None):
        th = table(theta) if theta is not None else (None, None)
        mk = table(mask) if mask is not None else (None, None)
        return lib.condensa_filter_prune(t4, 1, 0.5, 0, th[0], mk[0], sumsq, norms, keep_idx, smask, res, ws, tiny, None, None)

    assert fp(theta=A, mask=Bf, sumsq=C, norms=D, keep_idx=E, smask=E + 64) == -5
    assert fp(theta=W) == -5
    assert fp(theta=W + 4) == -6
    assert fp(theta=A, sumsq=A + 8) == -6
    assert fp(keep_idx=E, smask=E + 39) == -6                     # ten 4-byte ids end at E + 40
    assert fp(keep_idx=E, smask=E + 40) == -5
    assert fp(norms=W + 100) == -6

    # L-step update: the five buffers of a tensor must be disjoint
    def sgd(grad=A, theta=Bf, lam=C, mom=D):
        tabs = [table(x) for x in (grad, theta, lam, mom)]
        return lib.condensa_lc_sgd_step(t, 1, tabs[0][0], tabs[1][0], tabs[2][0], tabs[3][0], 1e-3, 0.1, 0.9, ws, tiny,
                                        None, None)

    assert sgd() == -5
    assert sgd(mom=W + 4) == -6
    assert sgd(grad=W + 4 * n - 4) == -6                          # an input over the weights, which are written
    assert sgd(theta=C + 4) == -5                                 # two read-only inputs may overlap
    assert sgd(mom=A) == -6

    shape = (ctypes.c_int64 * 4)(8, 4, 3, 3)
    assert lib.condensa_thin(W, shape, 4, None, 0, 0, None, 0, 0, W + 8 * 4 * 9 * 4 - 4, None) == -6


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(P.binding.Tensor) == 48
    assert ctypes.sizeof(P.binding.Config) == 32
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
    big = lib.condensa_workspace_bytes(B.OP_LC_STEP, n, 0, 64, 1, B.SCOPE_GLOBAL, None)
    assert 0.5e9 < big < 1.0e9                         # candidate capacity N/32 x 28 B dominates
    assert lib.condensa_workspace_bytes(B.OP_LC_STEP, n // 2, 0, 64, 1, B.SCOPE_GLOBAL, None) < big
    assert lib.condensa_workspace_bytes(B.OP_PRUNE, n, 0, 64, 16, B.SCOPE_GLOBAL, None) > 0
    assert lib.condensa_workspace_bytes(B.OP_PRUNE, n, 0, 64, 17, B.SCOPE_GLOBAL, None) == 0      # too many densities
    assert lib.condensa_workspace_bytes(B.OP_QUANTIZE, n, 0, 1, 1, B.SCOPE_GLOBAL, None) == 0      # needs none
    assert lib.condensa_workspace_bytes(99, n, 0, 1, 1, B.SCOPE_GLOBAL, None) == 0


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
    assert lib.condensa_prune(t, 1, bad, 1, 0, null, null, null, res, ws, 1 << 30, null, null) == -3
    assert lib.condensa_prune(t, 1, dens, 17, 0, null, null, null, res, ws, 1 << 30, null, null) == -2
    assert lib.condensa_prune(t, 1, dens, 1, 7, null, null, null, res, ws, 1 << 30, null, null) == -6
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, res, ws, 16, null, null) == -5
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, res, ctypes.c_void_p(4100), 1 << 30, null, null) == -5
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, res, null, 1 << 30, null, null) == -5
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, null, ws, 1 << 30, null, null) == -1
    t[0].ndim = 5
    assert lib.condensa_prune(t, 1, dens, 1, 0, null, null, null, res, ws, 1 << 30, null, null) == -4
    t[0].ndim = 1
    # filter pruning wants 4-D tensors, block pruning 2-D ones whose dimensions the block divides
    assert lib.condensa_filter_prune(t, 1, 0.5, 0, null, null, null, null, null, null, res, ws, 1 << 30, null, null) == -4
    t[0].shape[0], t[0].shape[1], t[0].ndim = 6, 8, 2
    assert lib.condensa_block_prune(t, 1, 4, 4, 0.5, 0, null, null, null, null, null, null, res, ws, 1 << 30, null, null) == -4
    assert lib.condensa_block_prune(t, 1, 0, 4, 0.5, 0, null, null, null, null, null, null, res, ws, 1 << 30, null, null) == -4
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        assert len(lib.condensa_status_string(code)) > 0
