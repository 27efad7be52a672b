"""CPU oracle for the compression step -- TEST INFRASTRUCTURE ONLY.

Thin numpy front end of ``condensa_oracle.c`` (plain C, scalar, sort based).
Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the GPU library never does, and nothing here imports the GPU
library.  Inputs are lists of C-contiguous float32 numpy arrays (one per weight
tensor); the flat index of an element is its position in the concatenation of
the tensors in list order (Section 3.1: schemes act on the whole model, layer
by layer).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "condensa_oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")

SCOPE_GLOBAL = 0
SCOPE_PER_TENSOR = 1


class Select(ctypes.Structure):
    _fields_ = [(name, ctypes.c_uint64) for name in
                ("n", "k", "n_gt", "n_tie_kept", "n_tie", "threshold_key", "tie_end")]

    def as_dict(self) -> Dict[str, int]:
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no contraction, no fast-math)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-msse2", "-mfpmath=sse", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u64, dbl, vp, f32 = ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p, ctypes.c_float
        L.oracle_kept_count.restype = u64
        L.oracle_kept_count.argtypes = [dbl, u64]
        for name, args in {
            "oracle_magnitude_keys": [vp, u64, vp],
            "oracle_aggregate_keys": [vp, u64, vp],
            "oracle_sort_desc": [vp, u64],
            "oracle_select_keep": [vp, vp, u64, u64, ctypes.POINTER(Select), vp],
            "oracle_apply_keep": [vp, vp, u64, vp],
            "oracle_quantize_f16": [vp, u64, vp, vp],
            "oracle_quantize_bf16": [vp, u64, vp, vp],
            "oracle_dequantize_bf16": [vp, u64, vp],
            "oracle_quantize_fp8": [vp, u64, ctypes.c_int, vp, vp],
            "oracle_dequantize_fp8": [vp, u64, ctypes.c_int, vp],
            "oracle_dequantize_f16": [vp, u64, vp],
            "oracle_filter_sumsq": [vp, u64, u64, vp],
            "oracle_block_sumsq": [vp, u64, u64, u64, u64, vp],
            "oracle_norms": [vp, u64, vp],
            "oracle_filter_apply": [vp, u64, u64, vp, vp, vp],
            "oracle_block_apply": [vp, u64, u64, u64, u64, vp, vp, vp],
            "oracle_block_sumsq_nd": [vp, vp, vp, vp],
            "oracle_block_apply_nd": [vp, vp, vp, vp, vp, vp],
            "oracle_lc_shifted": [vp, vp, u64, f32, vp],
            "oracle_lc_update": [vp, vp, vp, vp, u64, f32, vp, vp, vp],
            "oracle_lc_sgd_step": [vp, vp, vp, vp, vp, u64, f32, f32, f32, vp, vp],
            "oracle_thin": [vp, u64, u64, u64, vp, u64, vp, u64, vp],
            "oracle_lc_update_pq": [vp, vp, vp, vp, u64, f32, vp, vp, vp, vp],
        }.items():
            fn = getattr(L, name)
            fn.restype = None
            fn.argtypes = args
        for name in ("oracle_quantize_fp8", "oracle_dequantize_fp8"):
            getattr(L, name).restype = ctypes.c_int
        for name in ("oracle_count_nonzero_f32", "oracle_count_nonzero_f16", "oracle_count_nonzero_u8"):
            fn = getattr(L, name)
            fn.restype = u64
            fn.argtypes = [vp, u64]
        _lib = L
    return _lib


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs are float32")
    return a


def _flat(tensors: Sequence[np.ndarray]) -> np.ndarray:
    if len(tensors) == 0:
        return np.zeros(0, np.float32)
    return np.concatenate([_f32(t).reshape(-1) for t in tensors])


def _split(flat: np.ndarray, like: Sequence[np.ndarray]) -> List[np.ndarray]:
    out, o = [], 0
    for t in like:
        out.append(flat[o:o + t.size].reshape(t.shape))
        o += t.size
    return out


# ------------------------------------------------------------------ pieces --

def kept_count(density: float, n: int) -> int:
    """k = llround(density * n) clamped to [0, n] (product in binary64)."""
    return int(lib().oracle_kept_count(float(density), int(n)))


def magnitude_keys(x: np.ndarray) -> np.ndarray:
    x = _f32(x).reshape(-1)
    keys = np.empty(x.size, np.uint64)
    lib().oracle_magnitude_keys(_p(x), x.size, _p(keys))
    return keys


def aggregate_keys(s: np.ndarray) -> np.ndarray:
    s = np.ascontiguousarray(s, dtype=np.float64).reshape(-1)
    keys = np.empty(s.size, np.uint64)
    lib().oracle_aggregate_keys(_p(s), s.size, _p(keys))
    return keys


def sort_desc(keys: np.ndarray) -> np.ndarray:
    out = np.ascontiguousarray(keys, dtype=np.uint64).copy()
    lib().oracle_sort_desc(_p(out), out.size)
    return out


def select_keep(keys: np.ndarray, k: int, sorted_desc: np.ndarray | None = None):
    """(select record, keep flags) of the k largest keys, ties to the lowest index."""
    keys = np.ascontiguousarray(keys, dtype=np.uint64)
    if sorted_desc is None:
        sorted_desc = sort_desc(keys)
    sel = Select()
    keep = np.empty(keys.size, np.uint8)
    lib().oracle_select_keep(_p(keys), _p(sorted_desc), keys.size, int(k), ctypes.byref(sel), _p(keep))
    return sel.as_dict(), keep


def apply_keep(x: np.ndarray, keep: np.ndarray) -> np.ndarray:
    x = _f32(x).reshape(-1)
    theta = np.empty_like(x)
    lib().oracle_apply_keep(_p(x), _p(keep), x.size, _p(theta))
    return theta


# ------------------------------------------------------------- operators ----

def quantize_f16(x: np.ndarray):
    """binary32 -> binary16 bits (round to nearest even) and the exact widening back."""
    xf = _f32(x).reshape(-1)
    q = np.empty(xf.size, np.uint16)
    dq = np.empty(xf.size, np.float32)
    lib().oracle_quantize_f16(_p(xf), xf.size, _p(q), _p(dq))
    return q.reshape(np.shape(x)), dq.reshape(np.shape(x))


def dequantize_f16(q: np.ndarray) -> np.ndarray:
    qf = np.ascontiguousarray(q, dtype=np.uint16).reshape(-1)
    dq = np.empty(qf.size, np.float32)
    lib().oracle_dequantize_f16(_p(qf), qf.size, _p(dq))
    return dq.reshape(np.shape(q))


def quantize_bf16(x: np.ndarray):
    """binary32 -> bfloat16 bits (round to nearest even) and the exact widening back."""
    xf = _f32(x).reshape(-1)
    q = np.empty(xf.size, np.uint16)
    dq = np.empty(xf.size, np.float32)
    lib().oracle_quantize_bf16(_p(xf), xf.size, _p(q), _p(dq))
    return q.reshape(np.shape(x)), dq.reshape(np.shape(x))


def dequantize_bf16(q: np.ndarray) -> np.ndarray:
    qf = np.ascontiguousarray(q, dtype=np.uint16).reshape(-1)
    dq = np.empty(qf.size, np.float32)
    lib().oracle_dequantize_bf16(_p(qf), qf.size, _p(dq))
    return dq.reshape(np.shape(q))


FP8_E4M3, FP8_E5M2 = 0, 1


def quantize_fp8(x: np.ndarray, fmt: int):
    """binary32 -> 8-bit floating point codes (E4M3 or E5M2: nearest finite value, ties to even, saturating)
    and the exact widening back."""
    xf = _f32(x).reshape(-1)
    q = np.empty(xf.size, np.uint8)
    dq = np.empty(xf.size, np.float32)
    if lib().oracle_quantize_fp8(_p(xf), xf.size, int(fmt), _p(q), _p(dq)) != 0:
        raise ValueError("unknown 8-bit format")
    return q.reshape(np.shape(x)), dq.reshape(np.shape(x))


def dequantize_fp8(q: np.ndarray, fmt: int) -> np.ndarray:
    qf = np.ascontiguousarray(q, dtype=np.uint8).reshape(-1)
    dq = np.empty(qf.size, np.float32)
    if lib().oracle_dequantize_fp8(_p(qf), qf.size, int(fmt), _p(dq)) != 0:
        raise ValueError("unknown 8-bit format")
    return dq.reshape(np.shape(q))


def _prune_flat(x: np.ndarray, densities: Sequence[float]):
    keys = magnitude_keys(x)
    srt = sort_desc(keys)
    out = []
    for d in densities:
        sel, keep = select_keep(keys, kept_count(d, x.size), srt)
        out.append((sel, keep, apply_keep(x, keep)))
    return out


def prune(tensors: Sequence[np.ndarray], densities: Sequence[float], scope: int = SCOPE_GLOBAL):
    """Unstructured magnitude pruning.  Returns one dict per density with
    ``theta`` / ``mask`` (lists, one array per tensor) and ``select`` (one
    record for GLOBAL scope, a list with one record per tensor otherwise)."""
    tensors = [_f32(t) for t in tensors]
    results = []
    if scope == SCOPE_GLOBAL:
        flat = _flat(tensors)
        for sel, keep, theta in _prune_flat(flat, densities):
            results.append({"theta": _split(theta, tensors), "mask": _split(keep, tensors), "select": sel})
    else:
        per_t = [_prune_flat(t.reshape(-1), densities) for t in tensors]
        for j in range(len(densities)):
            results.append({
                "theta": [per_t[i][j][2].reshape(t.shape) for i, t in enumerate(tensors)],
                "mask": [per_t[i][j][1].reshape(t.shape) for i, t in enumerate(tensors)],
                "select": [per_t[i][j][0] for i in range(len(tensors))],
            })
    return results


def filter_sumsq(t: np.ndarray) -> np.ndarray:
    """Sum of squares of every output filter of a [Cout, ...] tensor (binary64)."""
    t = _f32(t)
    f = t.shape[0]
    length = t.size // f if f else 0
    s = np.empty(f, np.float64)
    lib().oracle_filter_sumsq(_p(t), f, length, _p(s))
    return s


def block_sumsq(t: np.ndarray, bh: int, bw: int) -> np.ndarray:
    t = _f32(t)
    rows, cols = t.shape
    if rows % bh or cols % bw:
        raise ValueError("block shape must divide the matrix")
    s = np.empty((rows // bh) * (cols // bw), np.float64)
    lib().oracle_block_sumsq(_p(t), rows, cols, bh, bw, _p(s))
    return s


def norms_of(s: np.ndarray) -> np.ndarray:
    s = np.ascontiguousarray(s, dtype=np.float64)
    out = np.empty(s.size, np.float32)
    lib().oracle_norms(_p(s), s.size, _p(out))
    return out


def _structure_prune(tensors, sums: List[np.ndarray], density: float, scope: int, apply_one):
    counts = [s.size for s in sums]
    all_s = np.concatenate(sums) if sums else np.zeros(0, np.float64)
    keys = aggregate_keys(all_s)
    if scope == SCOPE_GLOBAL:
        sel, keep = select_keep(keys, kept_count(density, keys.size))
        select = sel
    else:
        keep = np.empty(keys.size, np.uint8)
        select, o = [], 0
        for c in counts:
            sel, kp = select_keep(keys[o:o + c], kept_count(density, c))
            keep[o:o + c] = kp
            select.append(sel)
            o += c
    theta, mask, o = [], [], 0
    for t, c in zip(tensors, counts):
        th = np.empty_like(t)
        mk = np.empty(t.shape, np.uint8)
        apply_one(t, np.ascontiguousarray(keep[o:o + c]), th, mk)
        theta.append(th)
        mask.append(mk)
        o += c
    return {"theta": theta, "mask": mask, "sumsq": all_s, "norms": norms_of(all_s),
            "keep_idx": np.flatnonzero(keep).astype(np.int32), "structure_mask": keep, "select": select}


def filter_prune(tensors: Sequence[np.ndarray], density: float, scope: int = SCOPE_GLOBAL):
    """Filter pruning by sum of squares (ranking by L2 norm); density counts filters."""
    tensors = [_f32(t) for t in tensors]

    def apply_one(t, keep, th, mk):
        f = t.shape[0]
        lib().oracle_filter_apply(_p(t), f, t.size // f if f else 0, _p(keep), _p(th), _p(mk))

    return _structure_prune(tensors, [filter_sumsq(t) for t in tensors], density, scope, apply_one)


def block_prune(tensors: Sequence[np.ndarray], bh: int, bw: int, density: float, scope: int = SCOPE_GLOBAL):
    """2-D block pruning of matrices by block sum of squares; density counts blocks."""
    tensors = [_f32(t) for t in tensors]

    def apply_one(t, keep, th, mk):
        lib().oracle_block_apply(_p(t), t.shape[0], t.shape[1], bh, bw, _p(keep), _p(th), _p(mk))

    return _structure_prune(tensors, [block_sumsq(t, bh, bw) for t in tensors], density, scope, apply_one)


def _dims4(shape, block):
    """Left-pad shape and block with ones to rank 4."""
    if len(shape) != len(block) or not 1 <= len(shape) <= 4:
        raise ValueError("block rank must equal tensor rank (1..4)")
    if any(int(b) < 1 for b in block):
        raise ValueError("block sizes must be positive")
    pad = 4 - len(shape)
    d = np.array([1] * pad + [int(x) for x in shape], np.uint64)
    b = np.array([1] * pad + [int(x) for x in block], np.uint64)
    return d, b


def block_sumsq_nd(t: np.ndarray, block: Sequence[int]) -> np.ndarray:
    """Sums of squares of the n-D blocks of one tensor; edge blocks may be smaller (ragged)."""
    t = _f32(t)
    d, b = _dims4(t.shape, block)
    n_blocks = int(np.prod((d + b - np.uint64(1)) // b)) if t.size else 0
    s = np.empty(n_blocks, np.float64)
    if n_blocks:
        lib().oracle_block_sumsq_nd(_p(t), _p(d), _p(b), _p(s))
    return s


def block_prune_nd(tensors: Sequence[np.ndarray], block: Sequence[int], density: float, scope: int = SCOPE_GLOBAL):
    """BlockPrune with n-D blocks and ragged edges (every tensor has the rank of ``block``)."""
    tensors = [_f32(t) for t in tensors]

    def apply_one(t, keep, th, mk):
        if t.size:
            d, b = _dims4(t.shape, block)
            lib().oracle_block_apply_nd(_p(t), _p(d), _p(b), _p(keep), _p(th), _p(mk))

    return _structure_prune(tensors, [block_sumsq_nd(t, block) for t in tensors], density, scope, apply_one)


def neuron_prune(tensors: Sequence[np.ndarray], density: float, scope: int = SCOPE_GLOBAL):
    """NeuronPrune: a neuron is a row of a [out, in] matrix (a 1-D block), ranked by sum of squares."""
    for t in tensors:
        if t.ndim != 2:
            raise ValueError("neuron pruning takes [out, in] matrices")
    return filter_prune(tensors, density, scope)


def structure_prune(tensors: Sequence[np.ndarray], density: float, scope: int = SCOPE_GLOBAL):
    """StructurePrune: neurons of the 2-D tensors and filters of the 4-D tensors in one ranking."""
    for t in tensors:
        if t.ndim not in (2, 4):
            raise ValueError("structure pruning takes [out, in] matrices and [Cout, Cin, kh, kw] tensors")
    return filter_prune(tensors, density, scope)


def lc_step(tensors: Sequence[np.ndarray], lambdas: Sequence[np.ndarray], mu: float, density: float):
    """One compression step with multiplier and penalty-gradient update (global scope)."""
    tensors = [_f32(t) for t in tensors]
    lambdas = [_f32(t) for t in lambdas]
    w, lam = _flat(tensors), _flat(lambdas)
    if w.size != lam.size:
        raise ValueError("lambda must match w")
    mu32 = float(np.float32(mu))
    v = np.empty_like(w)
    lib().oracle_lc_shifted(_p(w), _p(lam), w.size, mu32, _p(v))
    keys = magnitude_keys(v)
    sel, keep = select_keep(keys, kept_count(density, w.size))
    theta, lam_out, grad = np.empty_like(w), np.empty_like(w), np.empty_like(w)
    lib().oracle_lc_update(_p(w), _p(lam), _p(v), _p(keep), w.size, mu32, _p(theta), _p(lam_out), _p(grad))
    return {"theta": _split(theta, tensors), "lambda": _split(lam_out, tensors), "grad": _split(grad, tensors),
            "mask": _split(keep, tensors), "select": sel, "v": _split(v, tensors)}


def lc_step_pq(tensors: Sequence[np.ndarray], lambdas: Sequence[np.ndarray], mu: float, density: float):
    """L-C compression step for Compose([Prune(), Quantize(float16)]): theta is stored as binary16 and
    the multiplier update sees its exact widening."""
    tensors = [_f32(t) for t in tensors]
    lambdas = [_f32(t) for t in lambdas]
    w, lam = _flat(tensors), _flat(lambdas)
    if w.size != lam.size:
        raise ValueError("lambda must match w")
    mu32 = float(np.float32(mu))
    v = np.empty_like(w)
    lib().oracle_lc_shifted(_p(w), _p(lam), w.size, mu32, _p(v))
    sel, keep = select_keep(magnitude_keys(v), kept_count(density, w.size))
    theta16 = np.empty(w.size, np.uint16)
    theta, lam_out, grad = np.empty_like(w), np.empty_like(w), np.empty_like(w)
    lib().oracle_lc_update_pq(_p(w), _p(lam), _p(v), _p(keep), w.size, mu32, _p(theta16), _p(theta), _p(lam_out), _p(grad))
    return {"theta_f16": _split(theta16, tensors), "theta": _split(theta, tensors), "lambda": _split(lam_out, tensors),
            "grad": _split(grad, tensors), "mask": _split(keep, tensors), "select": sel, "v": _split(v, tensors)}


def count_nonzero(tensors: Sequence[np.ndarray]) -> int:
    """Non-zero parameters of float32 tensors or of 16-bit / 8-bit floating-point codes (uint16 / uint8); -0 is zero."""
    total = 0
    for t in tensors:
        t = np.ascontiguousarray(t)
        if t.dtype == np.float32:
            total += int(lib().oracle_count_nonzero_f32(_p(t), t.size))
        elif t.dtype == np.uint16:
            total += int(lib().oracle_count_nonzero_f16(_p(t), t.size))
        elif t.dtype == np.uint8:
            total += int(lib().oracle_count_nonzero_u8(_p(t), t.size))
        else:
            raise TypeError("float32 values, uint16 or uint8 floating-point codes")
    return total


def thin(t: np.ndarray, keep_out=None, keep_in=None) -> np.ndarray:
    """Network thinning of one [Cout, Cin, ...] tensor: keep the listed output structures (filters /
    neurons) and the listed input channels, in list order, as a dense smaller tensor."""
    t = _f32(t)
    c_out, c_in = t.shape[0], t.shape[1]
    ksize = t.size // (c_out * c_in) if c_out * c_in else 0
    ko = None if keep_out is None else np.ascontiguousarray(keep_out, dtype=np.int32)
    ki = None if keep_in is None else np.ascontiguousarray(keep_in, dtype=np.int32)
    n_out = c_out if ko is None else ko.size
    n_in = c_in if ki is None else ki.size
    out = np.empty((n_out, n_in) + t.shape[2:], np.float32)
    if out.size:
        lib().oracle_thin(_p(t), c_out, c_in, ksize, None if ko is None else _p(ko), n_out,
                          None if ki is None else _p(ki), n_in, _p(out))
    return out


def lc_sgd_step(ws, grads, thetas, lambdas, bufs, mu: float, lr: float, momentum: float):
    """One SGD-with-momentum update of the learning step with the L-C penalty gradient folded in.
    Returns (new weights, new momentum buffers) as lists."""
    w_out, b_out = [], []
    for w, g, th, lam, b in zip(ws, grads, thetas, lambdas, bufs):
        w, g, th, lam, b = (_f32(x) for x in (w, g, th, lam, b))
        wn, bn = np.empty_like(w), np.empty_like(w)
        lib().oracle_lc_sgd_step(_p(w), _p(g), _p(th), _p(lam), _p(b), w.size, float(np.float32(mu)),
                                 float(np.float32(lr)), float(np.float32(momentum)), _p(wn), _p(bn))
        w_out.append(wn)
        b_out.append(bn)
    return w_out, b_out


def mu_schedule(mu0: float, a: float, j: int) -> float:
    """mu_j = mu_0 a^j ("L-C Optimizer Settings": mu_0 = 1e-3, a = 1.1), evaluated in binary64, returned as binary32."""
    return float(np.float32(float(mu0) * float(a) ** int(j)))
