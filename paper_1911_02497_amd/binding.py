"""ctypes binding of libcondensa.so: same names as the C entry points, marshalling only.

torch is used for device memory and the current stream; no arithmetic happens here.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# CONDENSA_LIBRARY names another build of the same library (same C ABI), e.g. one compiled elsewhere.
_LIB_PATH = os.environ.get("CONDENSA_LIBRARY") or os.path.join(_HERE, "libcondensa.so")

SCOPE_GLOBAL, SCOPE_PER_TENSOR = 0, 1
OP_PRUNE, OP_FILTER_PRUNE, OP_BLOCK_PRUNE, OP_QUANTIZE, OP_LC_STEP, OP_COUNT_NONZERO, OP_LC_SGD_STEP = range(7)
OPT_SELECT_PATH, OPT_SAMPLE_LOG2, OPT_WINDOW_MARGIN, OPT_CAND_SHIFT, OPT_PROFILE, OPT_APPLY_THREADS, OPT_FUSED_SWEEP = range(7)
WINDOW_MARGIN_DEFAULT = 80          # CONDENSA_OPT_WINDOW_MARGIN as the library starts with
PHASES = ("sample", "sweep", "resolve", "apply", "aggregate")
MAX_DENSITIES = 16

SELECT_FIELDS = ("n", "k", "n_gt", "n_tie_kept", "n_tie", "threshold_key", "tie_end", "path")


class CondensaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"condensa status {code}: {msg}")
        self.code = code


class Config(ctypes.Structure):
    """condensa_config: the tuning / test knobs of one call."""
    _fields_ = [("select_path", ctypes.c_int32), ("sample_log2", ctypes.c_int32), ("window_margin", ctypes.c_int32),
                ("cand_shift", ctypes.c_int32), ("profile", ctypes.c_int32), ("apply_threads", ctypes.c_int32),
                ("fused_sweep", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class Tensor(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("shape", ctypes.c_int64 * 4), ("ndim", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


_PROTOTYPES = {
    "condensa_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int,
                                                   ctypes.c_int, ctypes.c_int, ctypes.POINTER(Config)]),
    "condensa_config_init": (ctypes.c_int32, [ctypes.POINTER(Config)]),
    "condensa_prune_static": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                               ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_void_p]),
    "condensa_prune": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                        ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_filter_prune": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_neuron_prune": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_structure_prune": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                  ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_block_prune_nd": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.POINTER(ctypes.c_int32),
                                                 ctypes.c_int, ctypes.c_double, ctypes.c_int, ctypes.c_void_p,
                                                 ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                 ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                 ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_block_prune": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_double, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_quantize": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_void_p]),
    "condensa_dequantize": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]),
    "condensa_quantize_bf16": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_void_p]),
    "condensa_dequantize_bf16": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]),
    "condensa_quantize_fp8": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_void_p]),
    "condensa_dequantize_fp8": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p,
                                                 ctypes.c_void_p]),
    "condensa_lc_step": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_float, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                          ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_lc_step_pq": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_float, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_count_nonzero": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_lc_sgd_step": (ctypes.c_int32, [ctypes.POINTER(Tensor), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_float,
                                              ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(Config)]),
    "condensa_mu_schedule": (ctypes.c_float, [ctypes.c_double, ctypes.c_double, ctypes.c_int]),
    "condensa_thin": (ctypes.c_int32, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.c_int, ctypes.c_void_p,
                                       ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                       ctypes.c_void_p, ctypes.c_void_p]),
    "condensa_set_option": (ctypes.c_int32, [ctypes.c_int, ctypes.c_int64]),
    "condensa_get_option": (ctypes.c_int64, [ctypes.c_int]),
    "condensa_profile_read": (ctypes.c_int32, [ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                               ctypes.POINTER(ctypes.c_uint64)]),
    "condensa_profile_reset": (ctypes.c_int32, []),
    "condensa_status_string": (ctypes.c_char_p, [ctypes.c_int32]),
    "condensa_last_hip_error": (ctypes.c_int, []),
    "condensa_launch_count": (ctypes.c_uint64, []),
    "condensa_version": (ctypes.c_int, []),
}


def exported_symbols() -> List[str]:
    """Names every entry point declared in include/condensa.h must be exported under."""
    return sorted(_PROTOTYPES)


_lib = None


def library() -> ctypes.CDLL:
    """Loads libcondensa.so (after torch, so both share one HIP runtime).  No fallback exists."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_1911_02497_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        import torch  # noqa: F401  (brings in the HIP runtime the library binds to)
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(code: int) -> None:
    if code != 0:
        lib = library()
        msg = lib.condensa_status_string(code).decode()
        if code == -7:
            msg += f" (hipError {lib.condensa_last_hip_error()})"
        raise CondensaError(code, msg)


def _stream(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


class TensorTable(list):
    """A list of weight tensors together with its marshalled ``condensa_tensor`` array.  Passing one
    instead of a plain list to the calls below skips the per-call marshalling (it matters for models with
    many small tensors, where the Python loop costs more than the GPU work).  The tensors must keep their
    storage: a tensor that is reallocated needs a new table."""

    def __init__(self, tensors):
        super().__init__(tensors)
        self._arr = _marshal_tensors(self)
        self._total = sum(t.numel() for t in self)
        self._cache = {}

    def cached(self, key, make):
        if key not in self._cache:
            self._cache[key] = make()
        return self._cache[key]


def tensor_table(tensors) -> TensorTable:
    return tensors if isinstance(tensors, TensorTable) else TensorTable(tensors)


def _marshal_tensors(tensors):
    import torch
    arr = (Tensor * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
            raise TypeError("weights must be contiguous float32 device tensors")
        if t.dim() < 1 or t.dim() > 4:
            raise ValueError("weights must have 1 to 4 dimensions")
        arr[i].w = t.data_ptr() if t.numel() else None
        for d in range(t.dim()):
            arr[i].shape[d] = t.shape[d]
        arr[i].ndim = t.dim()
        arr[i].reserved = 0
    return arr


def _tensor_table(tensors):
    return tensors._arr if isinstance(tensors, TensorTable) else _marshal_tensors(tensors)


def _total(tensors) -> int:
    return tensors._total if isinstance(tensors, TensorTable) else sum(t.numel() for t in tensors)


def _cached(tensors, key, make):
    return tensors.cached(key, make) if isinstance(tensors, TensorTable) else make()


def _ptr_table(tensors: Optional[Sequence]):
    """Host array of device pointers (None entries become NULL); None -> NULL table."""
    if tensors is None:
        return None, None
    arr = (ctypes.c_void_p * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i] = None if (t is None or t.numel() == 0) else t.data_ptr()
    return arr, ctypes.cast(arr, ctypes.c_void_p)


def condensa_config(**fields) -> Config:
    """A condensa_config holding the process-wide defaults, with the given fields changed
    (select_path, sample_log2, window_margin, cand_shift, profile, apply_threads, fused_sweep)."""
    c = Config()
    _check(library().condensa_config_init(ctypes.byref(c)))
    for k, v in fields.items():
        if k not in {f for f, _ in Config._fields_} or k == "reserved":
            raise KeyError(k)
        setattr(c, k, int(v))
    return c


def _cfg(config):
    """None -> NULL (process-wide defaults); a dict of fields or a Config -> pointer to the struct."""
    if config is None:
        return None
    if isinstance(config, dict):
        config = condensa_config(**config)
    return ctypes.byref(config)


def _workspace(op, total, n_struct, n_tensors, n_dens, scope, device, workspace=None, config=None):
    import torch
    need = int(library().condensa_workspace_bytes(op, total, n_struct, n_tensors, n_dens, scope, _cfg(config)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, need


def condensa_workspace_bytes(op, total_elems, n_structures, n_tensors, n_densities, scope, config=None) -> int:
    return int(library().condensa_workspace_bytes(op, total_elems, n_structures, n_tensors, n_densities, scope,
                                                  _cfg(config)))


def condensa_set_option(option: int, value: int) -> None:
    _check(library().condensa_set_option(option, value))


def condensa_get_option(option: int) -> int:
    return int(library().condensa_get_option(option))


def condensa_launch_count() -> int:
    return int(library().condensa_launch_count())


def condensa_profile_reset() -> None:
    _check(library().condensa_profile_reset())


def condensa_profile_read() -> Dict[str, Dict[str, float]]:
    """Totals of the phase intervals recorded since the last reset: {phase: {ms, intervals}}."""
    out = {}
    for i, name in enumerate(PHASES):
        ms, n = ctypes.c_double(0.0), ctypes.c_uint64(0)
        _check(library().condensa_profile_read(i, ctypes.byref(ms), ctypes.byref(n)))
        out[name] = {"ms": ms.value, "intervals": int(n.value)}
    return out


def select_records(results) -> List[Dict[str, int]]:
    """Device int64 [m, 8] record tensor -> list of dicts (synchronises)."""
    host = results.cpu().numpy().view(np.uint64).reshape(-1, len(SELECT_FIELDS))
    return [{f: int(row[i]) for i, f in enumerate(SELECT_FIELDS)} for row in host]


def condensa_prune(tensors, densities, scope=SCOPE_GLOBAL, theta=True, theta_f16=False, mask=True,
                   in_place=False, workspace=None, stream=None, outputs=None, config=None, static=False):
    """Marshals a call of the C entry point condensa_prune.  ``theta`` / ``theta_f16`` / ``mask`` choose
    which outputs are allocated ([density][tensor] lists of device tensors); ``in_place`` passes the
    weights themselves as theta (one density only).  ``static`` calls condensa_prune_static instead (no
    workspace, GLOBAL scope).  Returns the outputs and the record tensor."""
    import torch
    lib = library()
    dev = tensors[0].device if tensors else torch.device("cuda")
    nt, J = len(tensors), len(densities)
    tab = _tensor_table(tensors)
    dens = (ctypes.c_double * max(J, 1))(*[float(d) for d in densities])
    total = _total(tensors)

    outputs = (outputs or {}).get("_buffers", {})    # ``outputs``: an earlier call's result, whose tensors are reused

    def outs(flag, dtype, name):
        if not flag:
            return None
        if outputs.get(name) is not None:
            return outputs[name]
        return [[torch.empty(t.shape, dtype=dtype, device=dev) for t in tensors] for _ in range(J)]

    th = [list(tensors)] if (theta and in_place) else outs(theta, torch.float32, "theta")
    th16 = outs(theta_f16, torch.int16, "theta_f16")
    mk = outs(mask, torch.uint8, "mask")
    flat = lambda x: None if x is None else [t for row in x for t in row]  # noqa: E731
    k1, p1 = _ptr_table(flat(th))
    k2, p2 = _ptr_table(flat(th16))
    k3, p3 = _ptr_table(flat(mk))
    n_rec = J * (nt if scope == SCOPE_PER_TENSOR else 1)
    results = outputs.get("results")
    if results is None:
        results = torch.zeros((max(n_rec, 1), len(SELECT_FIELDS)), dtype=torch.int64, device=dev)
    if static:
        if scope != SCOPE_GLOBAL or config is not None or workspace is not None:
            raise ValueError("condensa_prune_static: GLOBAL scope, no workspace, built-in settings")
        ws = None
        _check(lib.condensa_prune_static(tab, nt, dens, J, p1, p2, p3, results.data_ptr(), _stream(stream)))
    else:
        ws, need = _workspace(OP_PRUNE, total, 0, nt, J, scope, dev, workspace, config)
        _check(lib.condensa_prune(tab, nt, dens, J, scope, p1, p2, p3, results.data_ptr(), ws.data_ptr(), ws.numel(),
                                  _stream(stream), _cfg(config)))
    return {"theta": th, "theta_f16": th16, "mask": mk, "results": results[:n_rec], "workspace": ws,
            "_keep": (k1, k2, k3),
            "_buffers": {"theta": None if in_place else th, "theta_f16": th16, "mask": mk, "results": results}}


def _structure_call(fn_name, op, tensors, n_struct, density, scope, theta, mask, extra_args, workspace, stream,
                    outputs=None, config=None, fill_keep_idx=False):
    import torch
    lib = library()
    dev = tensors[0].device if tensors else torch.device("cuda")
    nt = len(tensors)
    tab = _tensor_table(tensors)
    total = _total(tensors)
    o = (outputs or {}).get("_buffers", {})      # ``outputs``: an earlier call's result, whose tensors are reused
    F = max(n_struct, 1)
    n_rec = nt if scope == SCOPE_PER_TENSOR else 1

    def reuse(name, make):
        return o[name] if o.get(name) is not None else make()

    th = reuse("theta", lambda: [torch.empty_like(t) for t in tensors]) if theta else None
    mk = reuse("mask", lambda: [torch.empty(t.shape, dtype=torch.uint8, device=dev) for t in tensors]) if mask else None
    k1, p1, k2, p2 = reuse("_tables", lambda: _ptr_table(th) + _ptr_table(mk))
    sumsq = reuse("sumsq", lambda: torch.empty(F, dtype=torch.float64, device=dev))
    norms = reuse("norms", lambda: torch.empty(F, dtype=torch.float32, device=dev))
    keep_idx = reuse("keep_idx", lambda: torch.empty(F, dtype=torch.int32, device=dev))
    if fill_keep_idx:                       # the library writes the first k entries only; on request the rest reads -1
        with torch.cuda.stream(torch.cuda.current_stream() if stream is None else stream):
            keep_idx.fill_(-1)
    smask = reuse("structure_mask", lambda: torch.empty(F, dtype=torch.uint8, device=dev))
    results = reuse("results", lambda: torch.zeros((max(n_rec, 1), len(SELECT_FIELDS)), dtype=torch.int64, device=dev))
    ws, need = _workspace(op, total, n_struct, nt, 1, scope, dev, workspace, config)
    args = [tab, nt] + extra_args + [float(density), scope, p1, p2, sumsq.data_ptr(), norms.data_ptr(),
                                     keep_idx.data_ptr(), smask.data_ptr(), results.data_ptr(), ws.data_ptr(),
                                     ws.numel(), _stream(stream), _cfg(config)]
    _check(getattr(lib, fn_name)(*args))
    return {"theta": th, "mask": mk, "sumsq": sumsq[:n_struct], "norms": norms[:n_struct],
            "keep_idx": keep_idx[:n_struct], "structure_mask": smask[:n_struct], "results": results[:n_rec],
            "workspace": ws, "_keep": (k1, k2),
            "_buffers": {"theta": th, "mask": mk, "sumsq": sumsq, "norms": norms, "keep_idx": keep_idx,
                         "structure_mask": smask, "results": results, "_tables": (k1, p1, k2, p2)}}


def condensa_filter_prune(tensors, density, scope=SCOPE_GLOBAL, theta=True, mask=True, workspace=None, stream=None,
                          outputs=None, **kw):
    n_struct = _cached(tensors, "rows", lambda: sum(t.shape[0] if t.numel() else 0 for t in tensors))
    return _structure_call("condensa_filter_prune", OP_FILTER_PRUNE, tensors, n_struct, density, scope, theta, mask,
                           [], workspace, stream, outputs, **kw)


def condensa_block_prune(tensors, block_h, block_w, density, scope=SCOPE_GLOBAL, theta=True, mask=True,
                         workspace=None, stream=None, outputs=None, **kw):
    n_struct = _cached(tensors, ("blocks", block_h, block_w),
                       lambda: sum((t.shape[0] // block_h) * (t.shape[1] // block_w) for t in tensors if t.dim() == 2))
    return _structure_call("condensa_block_prune", OP_BLOCK_PRUNE, tensors, n_struct, density, scope, theta, mask,
                           [int(block_h), int(block_w)], workspace, stream, outputs, **kw)


def condensa_neuron_prune(tensors, density, scope=SCOPE_GLOBAL, theta=True, mask=True, workspace=None, stream=None,
                          outputs=None, **kw):
    n_struct = _cached(tensors, "rows", lambda: sum(t.shape[0] if t.numel() else 0 for t in tensors))
    return _structure_call("condensa_neuron_prune", OP_FILTER_PRUNE, tensors, n_struct, density, scope, theta, mask,
                           [], workspace, stream, outputs, **kw)


def condensa_structure_prune(tensors, density, scope=SCOPE_GLOBAL, theta=True, mask=True, workspace=None, stream=None,
                             outputs=None, **kw):
    n_struct = _cached(tensors, "rows", lambda: sum(t.shape[0] if t.numel() else 0 for t in tensors))
    return _structure_call("condensa_structure_prune", OP_FILTER_PRUNE, tensors, n_struct, density, scope, theta, mask,
                           [], workspace, stream, outputs, **kw)


def condensa_block_prune_nd(tensors, block_shape, density, scope=SCOPE_GLOBAL, theta=True, mask=True,
                            workspace=None, stream=None, outputs=None, **kw):
    nd = len(block_shape)
    blk = (ctypes.c_int32 * max(nd, 1))(*[int(b) for b in block_shape])
    n_struct = 0
    for t in tensors:
        if t.dim() == nd and t.numel():
            c = 1
            for d, b in zip(t.shape, block_shape):
                c *= -(-d // max(int(b), 1))
            n_struct += c
    return _structure_call("condensa_block_prune_nd", OP_BLOCK_PRUNE, tensors, n_struct, density, scope, theta, mask,
                           [blk, nd], workspace, stream, outputs, **kw)


def _quantize(fn_name, x, want_q, want_dq, stream):
    import torch
    q = torch.empty(x.shape, dtype=torch.int16, device=x.device) if want_q else None
    dq = torch.empty_like(x) if want_dq else None
    _check(getattr(library(), fn_name)(x.data_ptr() if x.numel() else None, x.numel(),
                                       q.data_ptr() if q is not None else None,
                                       dq.data_ptr() if dq is not None else None, _stream(stream)))
    return q, dq


def _dequantize(fn_name, q, stream):
    import torch
    dq = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    _check(getattr(library(), fn_name)(q.data_ptr() if q.numel() else None, q.numel(), dq.data_ptr(), _stream(stream)))
    return dq


def condensa_quantize(x, want_q=True, want_dq=True, stream=None):
    """binary16 codes (int16 views of the bits) and / or their exact widening."""
    return _quantize("condensa_quantize", x, want_q, want_dq, stream)


def condensa_dequantize(q, stream=None):
    return _dequantize("condensa_dequantize", q, stream)


def condensa_quantize_bf16(x, want_q=True, want_dq=True, stream=None):
    """bfloat16 codes (int16 views of the bits) and / or their exact widening."""
    return _quantize("condensa_quantize_bf16", x, want_q, want_dq, stream)


def condensa_dequantize_bf16(q, stream=None):
    return _dequantize("condensa_dequantize_bf16", q, stream)


FP8_E4M3, FP8_E5M2 = 0, 1


def condensa_quantize_fp8(x, fmt, want_q=True, want_dq=True, stream=None):
    """8-bit floating-point codes (uint8; fmt = FP8_E4M3 or FP8_E5M2) and / or their exact widening."""
    import torch
    q = torch.empty(x.shape, dtype=torch.uint8, device=x.device) if want_q else None
    dq = torch.empty_like(x) if want_dq else None
    _check(library().condensa_quantize_fp8(x.data_ptr() if x.numel() else None, x.numel(), int(fmt),
                                           q.data_ptr() if q is not None else None,
                                           dq.data_ptr() if dq is not None else None, _stream(stream)))
    return q, dq


def condensa_dequantize_fp8(q, fmt, stream=None):
    import torch
    dq = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    _check(library().condensa_dequantize_fp8(q.data_ptr() if q.numel() else None, q.numel(), int(fmt), dq.data_ptr(),
                                             _stream(stream)))
    return dq


def condensa_lc_step(tensors, lambdas, mu, density, lambda_out=None, in_place=False, theta=True, grad=True,
                     mask=True, outputs=None, workspace=None, stream=None, pq=False, config=None, nnz=False):
    """Marshals condensa_lc_step.  By default fresh lambda_out tensors are allocated (lambda is left
    untouched); ``in_place`` updates lambda itself.  ``outputs`` may carry preallocated
    theta / grad / mask / lambda_out lists to reuse."""
    import torch
    lib = library()
    dev = tensors[0].device if tensors else torch.device("cuda")
    nt = len(tensors)
    tab = _tensor_table(tensors)
    total = _total(tensors)
    outputs = outputs or {}
    # an output that is switched off is not written, whether or not `outputs` holds buffers for it
    th = (outputs.get("theta") or [torch.empty_like(t) for t in tensors]) if theta else None
    gr = (outputs.get("grad") or [torch.empty_like(t) for t in tensors]) if grad else None
    mk = (outputs.get("mask") or [torch.empty(t.shape, dtype=torch.uint8, device=dev) for t in tensors]) if mask else None
    if in_place:
        lo = None
    else:
        lo = lambda_out or outputs.get("lambda") or [torch.empty_like(t) for t in tensors]
    kl, pl = _ptr_table(lambdas)
    klo, plo = _ptr_table(lo)
    k1, p1 = _ptr_table(th)
    k2, p2 = _ptr_table(gr)
    k3, p3 = _ptr_table(mk)
    results = outputs.get("results")
    if results is None:
        results = torch.zeros((1, len(SELECT_FIELDS)), dtype=torch.int64, device=dev)
    ws, need = _workspace(OP_LC_STEP, total, 0, nt, 1, SCOPE_GLOBAL, dev, workspace, config)
    th16, k4, count = None, None, None
    if pq:
        th16 = outputs.get("theta_f16") or [torch.empty(t.shape, dtype=torch.int16, device=dev) for t in tensors]
        k4, p4 = _ptr_table(th16)
        if nnz:                              # the footprint objective, counted inside the step
            count = outputs.get("nnz")
            if count is None:
                count = torch.zeros(1, dtype=torch.int64, device=dev)
        _check(lib.condensa_lc_step_pq(tab, nt, pl, plo, float(mu), float(density), p1, p4, p2, p3,
                                       None if count is None else count.data_ptr(),
                                       results.data_ptr(), ws.data_ptr(), ws.numel(), _stream(stream), _cfg(config)))
    else:
        _check(lib.condensa_lc_step(tab, nt, pl, plo, float(mu), float(density), p1, p2, p3, results.data_ptr(),
                                    ws.data_ptr(), ws.numel(), _stream(stream), _cfg(config)))
    return {"theta": th, "theta_f16": th16, "grad": gr, "mask": mk, "lambda": lambdas if in_place else lo, "nnz": count,
            "results": results, "workspace": ws, "_keep": (kl, klo, k1, k2, k3, k4)}


def condensa_lc_step_pq(tensors, lambdas, mu, density, **kw):
    """condensa_lc_step_pq: the L-C step of the composed prune + fp16 scheme (theta_f16 holds int16 views of the bits)."""
    return condensa_lc_step(tensors, lambdas, mu, density, pq=True, **kw)


def condensa_count_nonzero(tensors, workspace=None, stream=None):
    """Non-zero count of float32 tensors, of 16-bit floating-point codes when the tensors are int16 / float16 /
    bfloat16, or of 8-bit floating-point codes when they are uint8."""
    import torch
    lib = library()
    dev = tensors[0].device if tensors else torch.device("cuda")
    kinds = [(torch.float32,), (torch.int16, torch.float16, torch.bfloat16), (torch.uint8,)]
    kind = next((k for k, ds in enumerate(kinds) if tensors and tensors[0].dtype in ds), 0)
    nt = len(tensors)
    arr = (Tensor * max(nt, 1))()
    for i, t in enumerate(tensors):
        want = kinds[kind]
        if not (t.is_cuda and t.is_contiguous() and t.dtype in want and 1 <= t.dim() <= 4):
            raise TypeError("contiguous device tensors of one element type, 1 to 4 dimensions")
        arr[i].w = t.data_ptr() if t.numel() else None
        for d in range(t.dim()):
            arr[i].shape[d] = t.shape[d]
        arr[i].ndim = t.dim()
    total = _total(tensors)
    count = torch.zeros(1, dtype=torch.int64, device=dev)
    ws, need = _workspace(OP_COUNT_NONZERO, total, 0, nt, 1, SCOPE_GLOBAL, dev, workspace)
    _check(lib.condensa_count_nonzero(arr, nt, kind, count.data_ptr(), ws.data_ptr(), ws.numel(), _stream(stream), None))
    return count


def condensa_thin(w, keep_out=None, keep_in=None, keep_out_offset=0, keep_in_offset=0, stream=None):
    """Marshals condensa_thin: ``keep_out`` / ``keep_in`` are device int32 id tensors or None (keep all)."""
    import torch
    lib = library()
    if not (w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and 2 <= w.dim() <= 4):
        raise TypeError("w must be a contiguous float32 device tensor with 2 to 4 dimensions")
    for k in (keep_out, keep_in):
        if k is not None and not (k.is_cuda and k.dtype == torch.int32 and k.is_contiguous() and k.dim() == 1):
            raise TypeError("keep lists are contiguous 1-D int32 device tensors")
    n_out = w.shape[0] if keep_out is None else keep_out.numel()
    n_in = w.shape[1] if keep_in is None else keep_in.numel()
    out = torch.empty((n_out, n_in) + tuple(w.shape[2:]), dtype=torch.float32, device=w.device)
    if out.numel() == 0:                     # an empty keep list: nothing to gather (NULL would mean "keep all")
        return out
    shape = (ctypes.c_int64 * 4)(*list(w.shape) + [1] * (4 - w.dim()))
    _check(lib.condensa_thin(w.data_ptr() if w.numel() else None, shape, w.dim(),
                             None if keep_out is None else (keep_out.data_ptr() if keep_out.numel() else None),
                             0 if keep_out is None else keep_out.numel(), int(keep_out_offset),
                             None if keep_in is None else (keep_in.data_ptr() if keep_in.numel() else None),
                             0 if keep_in is None else keep_in.numel(), int(keep_in_offset),
                             out.data_ptr() if out.numel() else None, _stream(stream)))
    return out


def condensa_lc_sgd_step(tensors, grad_loss, theta, lambdas, momentum_buf, mu, lr, momentum, workspace=None, stream=None):
    """Marshals condensa_lc_sgd_step: ``tensors`` (weights) and ``momentum_buf`` are updated in place."""
    import torch
    lib = library()
    dev = tensors[0].device if tensors else torch.device("cuda")
    nt = len(tensors)
    tab = _tensor_table(tensors)
    total = _total(tensors)
    k1, p1 = _ptr_table(grad_loss)
    k2, p2 = _ptr_table(theta)
    k3, p3 = _ptr_table(lambdas)
    k4, p4 = _ptr_table(momentum_buf)
    ws, need = _workspace(OP_LC_SGD_STEP, total, 0, nt, 1, SCOPE_GLOBAL, dev, workspace)
    _check(lib.condensa_lc_sgd_step(tab, nt, p1, p2, p3, p4, float(mu), float(lr), float(momentum), ws.data_ptr(),
                                    ws.numel(), _stream(stream), None))
    return ws


def condensa_mu_schedule(mu0: float, a: float, j: int) -> float:
    return float(library().condensa_mu_schedule(float(mu0), float(a), int(j)))
