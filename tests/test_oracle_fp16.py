"""Pins for the oracle's binary32 -> binary16 rounding (CPU only).

Checked against hand-worked points of the IEEE 754 formats (tests/golden),
against numpy's independent float16 conversion over the whole binary32 space,
and against nearest-value optimality (the quantised theta_i is the closest
binary16 to w_i; Section 3.3, low-precision approximation).
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "binary16_points.txt")


def golden_points():
    pts = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            a, b = line.split()
            pts.append((int(a, 16), int(b, 16)))
    return pts


def test_hand_worked_points():
    pts = golden_points()
    assert len(pts) >= 20
    x = np.array([p[0] for p in pts], np.uint32).view(np.float32)
    q, _ = oracle.quantize_f16(x)
    assert [hex(v) for v in q.tolist()] == [hex(p[1]) for p in pts]


def _check_range(lo, hi):
    bits = np.arange(lo, hi, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    q, dq = oracle.quantize_f16(x)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16)
    nan = np.isnan(x)
    assert np.array_equal(q[~nan], ref.view(np.uint16)[~nan])
    assert np.all(np.isnan(q[nan].view(np.float16)))
    assert np.array_equal((q[nan] & 0x8000) != 0, (bits[nan] >> 31) != 0)
    # exact widening
    assert np.array_equal(dq[~nan].view(np.uint32), ref.astype(np.float32)[~nan].view(np.uint32))


def test_against_numpy_on_stratified_bit_patterns():
    """Every sign/exponent with all low-13-bit patterns under four high-mantissa settings,
    plus exhaustive sweeps of the subnormal-result and overflow bands."""
    hi10 = np.array([0, 1, 0x2AA, 0x3FF], np.uint32)
    low = np.arange(1 << 13, dtype=np.uint32)
    se = np.arange(1 << 9, dtype=np.uint32)
    bits = (se[:, None, None] << 23) | (hi10[None, :, None] << 13) | low[None, None, :]
    x = bits.reshape(-1).view(np.float32)
    q, _ = oracle.quantize_f16(x)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(q[~nan], ref[~nan])
    for e in (101, 102, 103, 112, 113, 142, 143):       # band edges, both signs below
        _check_range(e << 23, (e + 1) << 23)
    _check_range((1 << 31) | (102 << 23), (1 << 31) | (103 << 23))
    _check_range(0x7F000000, 0x80000000)                # top exponents, inf and NaN


@pytest.mark.slow
def test_against_numpy_on_all_2_to_32_patterns():
    step = 1 << 24
    for lo in range(0, 1 << 32, step):
        _check_range(lo, lo + step)


def test_result_is_the_nearest_binary16():
    rng = np.random.default_rng(16)
    x = np.concatenate([rng.standard_normal(2000) * s for s in (1e-7, 1e-4, 0.02, 1.0, 300.0, 4e4)]).astype(np.float32)
    q, dq = oracle.quantize_f16(x)
    finite = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)   # all non-negative finite
    ax = np.abs(x.astype(np.float64))
    idx = np.searchsorted(finite, ax)
    lo = finite[np.clip(idx - 1, 0, len(finite) - 1)]
    hi = finite[np.clip(idx, 0, len(finite) - 1)]
    best = np.minimum(np.abs(ax - lo), np.abs(ax - hi))
    inb = ax < 65504
    got = np.abs(dq.astype(np.float64))
    assert np.all(np.abs(got[inb] - ax[inb]) <= best[inb])
    assert np.array_equal(np.signbit(dq), np.signbit(x))


def test_idempotent_and_dequantize_roundtrip():
    allh = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    dq = oracle.dequantize_f16(allh)
    ref = allh.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(dq[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    assert np.all(np.isnan(dq[nan]))
    q2, _ = oracle.quantize_f16(dq)
    assert np.array_equal(q2[~nan], allh[~nan])          # q(dq(h)) == h for every non-NaN binary16


def test_pruned_zero_stays_zero_under_quantisation():
    """P+Q (Compose([Prune(), Quantize(float16)])): +0 -> +0, so the mask is unchanged."""
    x = (np.random.default_rng(1).standard_normal(4096) * 0.02).astype(np.float32)
    res = oracle.prune([x], [0.1])[0]
    q, _ = oracle.quantize_f16(res["theta"][0])
    assert np.all(q[res["mask"][0] == 0] == 0)


def test_table2_footprint_bound():
    """Footprint = bytes of non-zero parameters; P+Q at sparsity s gives at most 2/(1-s)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "table2_footprint.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for _, s, rc in rows:
        assert float(rc) <= 2.0 / (1.0 - (float(s) + 0.005)) + 1e-9
    # the same arithmetic on the oracle's own output: N fp32 bytes over nnz fp16 bytes
    x = (np.random.default_rng(2).standard_normal(100000) * 0.02).astype(np.float32)
    for s in (0.99, 0.95, 0.93, 0.92):
        res = oracle.prune([x], [1.0 - s])[0]
        q, _ = oracle.quantize_f16(res["theta"][0])
        nnz = int(np.count_nonzero(q & 0x7FFF))
        assert nnz == res["select"]["k"]                 # no kept weight of this scale underflows
        assert abs(4.0 * x.size / (2.0 * nnz) - 2.0 / (1.0 - s)) < 0.05 * 2.0 / (1.0 - s)
