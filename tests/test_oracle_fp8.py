"""Pins of the oracle's 8-bit floating-point conversions (E4M3 and E5M2 of the OCP 8-bit floating point
specification): the formats' published extreme values, hand-worked rounding points, PyTorch's independent
CPU conversions wherever the two conventions coincide (PyTorch does not saturate), all 256 codes against
PyTorch's widening, an arithmetic round-to-nearest-even written here with numpy, and the saturation rule."""
import numpy as np
import pytest
import torch

import oracle

E4M3, E5M2 = oracle.FP8_E4M3, oracle.FP8_E5M2
TORCH_DTYPE = {E4M3: torch.float8_e4m3fn, E5M2: torch.float8_e5m2}
# (fraction bits, bias, largest finite value, smallest subnormal, largest finite code)
GEOMETRY = {E4M3: (3, 7, 448.0, 2.0 ** -9, 0x7E), E5M2: (2, 15, 57344.0, 2.0 ** -16, 0x7B)}


def test_published_extreme_values_and_special_codes():
    for fmt, (mb, bias, vmax, vmin, cmax) in GEOMETRY.items():
        codes = np.array([cmax, 0x01, 1 << mb, 0x00, 0x80, cmax | 0x80], np.uint8)
        vals = oracle.dequantize_fp8(codes, fmt)
        assert list(vals[:3]) == [vmax, vmin, 2.0 ** (1 - bias)]            # largest, smallest subnormal, smallest normal
        assert vals[3] == 0 and not np.signbit(vals[3]) and vals[4] == 0 and np.signbit(vals[4])
        assert vals[5] == -vmax
    assert np.isnan(oracle.dequantize_fp8(np.array([0x7F, 0xFF], np.uint8), E4M3)).all()      # the only NaN codes of E4M3
    assert np.isfinite(oracle.dequantize_fp8(np.arange(0x7F, dtype=np.uint8), E4M3)).all()    # and it has no infinity
    special = oracle.dequantize_fp8(np.array([0x7C, 0xFC, 0x7D, 0x7E, 0x7F], np.uint8), E5M2)
    assert special[0] == np.inf and special[1] == -np.inf and np.isnan(special[2:]).all()


def test_hand_worked_rounding_points():
    # E4M3 near 1: neighbours 1.0 (0x38), 1.125 (0x39), 1.25 (0x3A)
    x = np.array([1.0, 1.0625, 1.0626, 1.1875, 1.06249, 0.0, -0.0, 2.0 ** -10, 1.5 * 2.0 ** -9, 2.0 ** -10 * 1.0001,
                  448.0, 464.0, 479.9, 1e30, np.inf, -np.inf, -1e30], np.float32)
    q, dq = oracle.quantize_fp8(x, E4M3)
    assert [int(v) for v in q] == [0x38, 0x38, 0x39, 0x3A, 0x38, 0x00, 0x80, 0x00, 0x02, 0x01,
                                   0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE]
    assert dq[1] == 1.0 and dq[3] == 1.25 and dq[13] == 448.0 and dq[15] == -448.0
    # E5M2 near 1: neighbours 1.0 (0x3C), 1.25 (0x3D), 1.5 (0x3E); infinities are kept, finite overflow saturates
    x = np.array([1.0, 1.125, 1.375, 1.1251, 2.0 ** -17, 2.0 ** -17 * 1.001, 3 * 2.0 ** -17, 57344.0, 61439.0, 61440.0,
                  1e30, np.inf, -np.inf], np.float32)
    q, dq = oracle.quantize_fp8(x, E5M2)
    assert [int(v) for v in q] == [0x3C, 0x3C, 0x3E, 0x3D, 0x00, 0x01, 0x02, 0x7B, 0x7B, 0x7B, 0x7B, 0x7C, 0xFC]
    assert dq[10] == 57344.0 and dq[11] == np.inf
    # NaN keeps its sign and becomes the format's NaN; widening gives the binary32 quiet NaN
    nan = np.array([0x7FC00000, 0xFFC00001, 0x7F800001], np.uint32).view(np.float32)
    q4, d4 = oracle.quantize_fp8(nan, E4M3)
    q5, d5 = oracle.quantize_fp8(nan, E5M2)
    assert [int(v) for v in q4] == [0x7F, 0xFF, 0x7F] and [int(v) for v in q5] == [0x7E, 0xFE, 0x7E]
    assert list(d4.view(np.uint32)) == [0x7FC00000, 0xFFC00000, 0x7FC00000] == list(d5.view(np.uint32))


@pytest.mark.parametrize("fmt", [E4M3, E5M2])
def test_all_codes_widen_as_in_torch_and_round_trip(fmt):
    codes = np.arange(256, dtype=np.uint8)
    back = oracle.dequantize_fp8(codes, fmt)
    want = torch.from_numpy(codes.copy()).view(TORCH_DTYPE[fmt]).to(torch.float32).numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(back), nan)
    assert np.array_equal(back[~nan].view(np.uint32), want[~nan].view(np.uint32))
    again, _ = oracle.quantize_fp8(back, fmt)
    assert np.array_equal(again[~nan], codes[~nan])                       # every non-NaN code is a fixed point
    mags = back[:0x80][~nan[:0x80]]
    assert np.all(np.diff(mags) > 0)                                      # code order = value order


@pytest.mark.parametrize("fmt", [E4M3, E5M2])
def test_against_torch_cpu_conversion_where_nothing_saturates(fmt):
    mb, bias, vmax, vmin, cmax = GEOMETRY[fmt]
    rng = np.random.default_rng(11 + fmt)
    limit = vmax * (1 + 2.0 ** -(mb + 2))          # below the midpoint to the next (absent) value both agree
    codes = np.arange(cmax + 1, dtype=np.uint8)
    vals = oracle.dequantize_fp8(codes, fmt).astype(np.float64)
    mids = (vals[:-1] + vals[1:]) / 2               # every tie point, and its two binary32 neighbours
    mids32 = mids.astype(np.float32)
    x = np.concatenate([
        (rng.standard_normal(300_000) * 0.02).astype(np.float32),
        np.exp(rng.uniform(np.log(vmin / 8), np.log(limit), 300_000)).astype(np.float32) * rng.choice([-1.0, 1.0], 300_000).astype(np.float32),
        vals.astype(np.float32), mids32, np.nextafter(mids32, np.float32(np.inf)), np.nextafter(mids32, np.float32(-np.inf)),
        -mids32, np.array([0.0, -0.0, 1e-30, -1e-30, 1e-45], np.float32)])
    x = x[np.abs(x) < limit]
    q, _ = oracle.quantize_fp8(x, fmt)
    want = torch.from_numpy(x.copy()).to(TORCH_DTYPE[fmt]).view(torch.uint8).numpy()
    assert np.array_equal(q, want)


@pytest.mark.parametrize("fmt", [E4M3, E5M2])
def test_against_arithmetic_round_to_nearest_even(fmt):
    """An independent construction: scale to the spacing of the value's binade, round half to even with
    numpy's rint in binary64 (exact for these magnitudes), clamp to the largest finite value."""
    mb, bias, vmax, vmin, cmax = GEOMETRY[fmt]
    rng = np.random.default_rng(5 + fmt)
    x = np.concatenate([np.exp(rng.uniform(np.log(vmin / 4), np.log(vmax * 4), 200_000)),
                        rng.standard_normal(200_000) * 3]).astype(np.float32)
    a = np.abs(x.astype(np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -60)))
    e = np.maximum(e, 1 - bias)                                           # subnormals share the spacing of the first binade
    step = 2.0 ** (e - mb)
    want = np.minimum(np.rint(a / step) * step, vmax) * np.sign(x)
    _, dq = oracle.quantize_fp8(x, fmt)
    assert np.array_equal(dq.astype(np.float64), want)


def test_saturation_never_produces_a_special_code_from_a_finite_input():
    x = np.array([449.0, 465.0, 1e6, 3.4e38, -465.0, 61440.0, 65536.0, -7e4], np.float32)
    q4, _ = oracle.quantize_fp8(x, E4M3)
    q5, _ = oracle.quantize_fp8(x, E5M2)
    assert [int(v) & 0x7F for v in q4] == [0x7E] * 8
    assert [int(v) & 0x7F for v in q5] == [0x5F, 0x5F, 0x7B, 0x7B, 0x5F, 0x7B, 0x7B, 0x7B]
    with pytest.raises(ValueError):
        oracle.quantize_fp8(x, 2)
