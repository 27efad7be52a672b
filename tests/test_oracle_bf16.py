"""Pins of the oracle's bfloat16 conversion: hand-worked points, PyTorch's independent CPU conversion over
a stratified pattern set and exhaustive bands, nearest-value optimality, round trip of all 65 536 codes."""
import numpy as np
import torch

import oracle


def _bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


def test_hand_worked_points():
    # (binary32 bits, expected bfloat16 bits): ties to even, carries, overflow, signed zeros, subnormals
    pts = [
        (0x3F800000, 0x3F80),    # 1.0
        (0x3F808000, 0x3F80),    # 1 + 2^-8: exactly halfway, even below -> stays
        (0x3F818000, 0x3F82),    # 1 + 3*2^-8: halfway, odd below -> up
        (0x3F808001, 0x3F81),    # just above halfway -> up
        (0x3F807FFF, 0x3F80),    # just below halfway -> down
        (0x3FFF8000, 0x4000),    # 1.99609375 + half ulp: carry into the exponent -> 2.0
        (0x7F7F8000, 0x7F80),    # largest finite binary32 region rounds to +inf
        (0x7F7F7FFF, 0x7F7F),    # just below stays the largest finite bfloat16
        (0xFF7FFFFF, 0xFF80),    # -FLT_MAX -> -inf
        (0x00000000, 0x0000), (0x80000000, 0x8000),
        (0x00008000, 0x0000),    # subnormal, halfway to the smallest bfloat16 subnormal, even -> 0
        (0x00008001, 0x0001),    # just above -> smallest subnormal
        (0x00018000, 0x0002),    # halfway, odd -> up
        (0x7F800000, 0x7F80), (0xFF800000, 0xFF80),
    ]
    x = np.array([p[0] for p in pts], np.uint32).view(np.float32)
    q, dq = oracle.quantize_bf16(x)
    assert [int(v) for v in q] == [p[1] for p in pts]
    assert np.array_equal(dq.view(np.uint32), q.astype(np.uint32) << 16)
    qn, _ = oracle.quantize_bf16(np.array([0x7FC00001, 0xFF800001, 0x7FFFFFFF], np.uint32).view(np.float32))
    assert [int(v) for v in qn] == [0x7FC0, 0xFFC0, 0x7FFF]           # NaN: sign and upper payload kept, quiet


def test_against_torch_cpu_conversion():
    rng = np.random.default_rng(7)
    pats = [rng.integers(0, 1 << 32, 4_000_000, dtype=np.uint64).astype(np.uint32)]
    for e in (0, 1, 2, 126, 127, 128, 253, 254):                       # whole exponent bands, both signs below
        band = (np.uint32(e) << 23) + np.arange(1 << 23, dtype=np.uint32)
        pats.append(band[:: 7])
        pats.append(band[:: 7] | np.uint32(0x80000000))
    for base in (0x3F800000, 0x00000000, 0x7F7F0000, 0x00800000):      # every dropped-bit pattern near these
        pats.append(np.uint32(base) + np.arange(1 << 18, dtype=np.uint32))
    u = np.concatenate(pats)
    x = u.view(np.float32)
    finite_or_inf = ~np.isnan(x)
    q, _ = oracle.quantize_bf16(x)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(q[finite_or_inf], want[finite_or_inf])
    nan_codes = q[~finite_or_inf]
    assert np.all((nan_codes & 0x7F80) == 0x7F80) and np.all((nan_codes & 0x007F) != 0)


def test_nearest_value_and_round_trip():
    allh = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    back = oracle.dequantize_bf16(allh)
    assert np.array_equal(back.view(np.uint32), allh.astype(np.uint32) << 16)
    q, _ = oracle.quantize_bf16(back)
    is_nan = np.isnan(back)
    assert np.array_equal(q[~is_nan], allh[~is_nan])                   # q(dq(h)) = h
    # optimality: no representable neighbour is closer (finite results away from the overflow edge)
    rng = np.random.default_rng(8)
    x = (rng.standard_normal(200_000) * np.exp(rng.standard_normal(200_000) * 20)).astype(np.float32)
    q, dq = oracle.quantize_bf16(x)
    ok = np.isfinite(dq) & (np.abs(dq) < 1e38) & (np.abs(dq) > 1e-37)
    up = oracle.dequantize_bf16((q + 1).astype(np.uint16))
    dn = oracle.dequantize_bf16((q - 1).astype(np.uint16))
    xd, d0 = x.astype(np.float64), np.abs(dq.astype(np.float64) - x.astype(np.float64))
    same_sign_up = ((q + 1) & 0x8000) == (q & 0x8000)
    same_sign_dn = (((q - 1) & 0x8000) == (q & 0x8000)) & ((q & 0x7FFF) != 0)
    assert np.all(d0[ok & same_sign_up] <= np.abs(up.astype(np.float64) - xd)[ok & same_sign_up])
    assert np.all(d0[ok & same_sign_dn] <= np.abs(dn.astype(np.float64) - xd)[ok & same_sign_dn])
